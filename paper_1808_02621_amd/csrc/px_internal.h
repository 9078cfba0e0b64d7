// Private declarations shared by the HIP sources of libpx (gfx950 only).
#ifndef PX_INTERNAL_H_
#define PX_INTERNAL_H_

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

#include "px.h"

struct px_ctx {
    int device;
    uint64_t* d_words;   // device: pointer / offset tables uploaded per call
    uint32_t* d_flags;   // device: [0] sticky error flag
    uint32_t* h_flags;   // pinned host mirror for px_device_status
    void* part_scratch;  // device address of the partition's built-in scratch on this GPU (not owned)
    unsigned long long* d_part_pub;   // device: PX_PART_PUB_WORDS words, shard counts published by a single-launch partition
    uint32_t part_call;  // number of the last single-launch partition on this context (tags the published words)
    int wait_polls;      // polls before a workgroup gives up a bounded wait (px_set_wait_limit)
    char err[512];
};

// d_words holds, per call, [idx pointers | value pointers | row prefix (n + 1)] for coalesce
// and [buffer pointers] for the dense mean.
enum { PXW_TOTAL = 3 * PX_MAX_SOURCES + 8 };

enum { PX_WAIT_POLLS_DEFAULT = 1 << 18 };   // about a third of a second of polling

enum { PX_PART_PUB_WORDS = 2048 };   // most (blocks x shards) of a single-launch partition: 8 words per thread to read

enum { PXF_BAD_ID = 1u, PXF_NOT_UNIQUE = 2u, PXF_INTERNAL = 4u };   // bits of d_flags[0]; any set bit stops later updates

px_status px_fail(px_ctx* ctx, px_status s, const char* fmt, ...);
px_status px_check_hip(px_ctx* ctx, hipError_t e, const char* what);
// Looks up the device address of the partition's built-in scratch; ctx->device must be current.
px_status px_partition_noalloc_setup(px_ctx* ctx);

// Up to PX_UPLOAD_WORDS 64-bit words can ride inside the arguments of a kernel launch.
enum { PX_UPLOAD_WORDS = 256 };
struct px_word_pack {
    uint64_t w[PX_UPLOAD_WORDS];
};

// Copies `n` host words into device memory at `dst` through kernel arguments
// (no host staging buffer, safe to capture), and zeroes `nzero` 32-bit words at `zero`.
px_status px_upload_words(px_ctx* ctx, uint64_t* dst, const uint64_t* host_words, int n,
                          uint32_t* zero, int nzero, hipStream_t stream);

static inline size_t px_align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// ---------------------------------------------------------------- radix passes
// One stable 8-bit counting pass = histogram per block, prefix over blocks, scatter.
#ifndef PX_SORT_MAX_BLOCKS_
#define PX_SORT_MAX_BLOCKS_ 512
#endif
#ifndef PX_SORT_ITEMS_PER_THREAD
#define PX_SORT_ITEMS_PER_THREAD 4     // 1,024-item tiles: the passes are chains of dependent steps, and short tiles make short chains
#endif
enum {
    PX_SORT_THREADS = 256,
    PX_SORT_ITEMS = PX_SORT_ITEMS_PER_THREAD,
    PX_SORT_TILE = PX_SORT_THREADS * PX_SORT_ITEMS,   // items ranked at once in LDS
    PX_SORT_MAX_BLOCKS = PX_SORT_MAX_BLOCKS_,     // multiple of 64
    PX_RADIX_MAX_BITS = 11,       // widest digit of a counting pass
    PX_RADIX_MAX = 1 << PX_RADIX_MAX_BITS
};
#ifndef PX_OWN_PREFIX_BLOCKS
#define PX_OWN_PREFIX_BLOCKS 32   // up to this many blocks a scatter block sums the histogram rows itself
#endif

struct px_sort_geom {
    int n_blocks;      // blocks of a pass
    int64_t chunk;     // items per block, a multiple of PX_SORT_TILE
};

static inline px_sort_geom px_sort_geometry(int64_t n) {
    px_sort_geom g;
    int64_t per = (n + PX_SORT_MAX_BLOCKS - 1) / PX_SORT_MAX_BLOCKS;
    g.chunk = (per + PX_SORT_TILE - 1) / PX_SORT_TILE * PX_SORT_TILE;
    if (g.chunk < PX_SORT_TILE) g.chunk = PX_SORT_TILE;
    g.n_blocks = (int) ((n + g.chunk - 1) / g.chunk);
    if (g.n_blocks < 1) g.n_blocks = 1;
    return g;
}

// Workgroups are handed to the chip's 8 dies (each with its own L2) in turn, so consecutive
// workgroup numbers land on different dies.  A streaming kernel that gives workgroup b the b-th
// few-KB piece of a buffer therefore has every die touch every 8th piece, which concentrates its
// traffic on a few of its L2 channels.  This maps the hardware's workgroup number to a logical one
// such that each die works on one contiguous eighth of the grid.  The grid must be a multiple of 8
// (round it up; surplus workgroups find nothing to do).
#ifdef __HIPCC__
__device__ __forceinline__ unsigned px_die_contiguous_block(unsigned b, unsigned n_blocks) {
    return (b & 7u) * (n_blocks >> 3) + (b >> 3);
}
#endif
static inline unsigned px_round_up_8(unsigned n) { return (n + 7u) & ~7u; }

#endif  // PX_INTERNAL_H_
