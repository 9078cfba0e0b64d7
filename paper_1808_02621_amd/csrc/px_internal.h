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
    char err[512];
};

// d_words holds, per call, [idx pointers | value pointers | row prefix (n + 1)] for coalesce
// and [buffer pointers] for the dense mean.
enum { PXW_TOTAL = 3 * PX_MAX_SOURCES + 8 };

enum {
    PXF_BAD_ID = 1u,      // a row id outside the table reached the device
    PXF_INTERNAL = 2u     // a bounded wait between workgroups ran out (never seen in practice)
};                        // bits of d_flags[0]
enum { PXD_PARTITION_DONE = 8 };   // d_flags[8]: blocks of the shard count kernel that have finished (returns to 0)

px_status px_fail(px_ctx* ctx, px_status s, const char* fmt, ...);
px_status px_check_hip(px_ctx* ctx, hipError_t e, const char* what);

// Copies `n` host words into device memory at `dst` through kernel arguments
// (no host staging buffer, safe to capture), and zeroes `nzero` 32-bit words at `zero`.
px_status px_upload_words(px_ctx* ctx, uint64_t* dst, const uint64_t* host_words, int n,
                          uint32_t* zero, int nzero, hipStream_t stream);

static inline size_t px_align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// ---------------------------------------------------------------- radix passes
// One stable 8-bit counting pass ranks tiles of PX_SORT_TILE items in LDS.
enum {
    PX_SORT_THREADS = 256,
    PX_SORT_ITEMS = 8,
    PX_SORT_TILE = PX_SORT_THREADS * PX_SORT_ITEMS,
    PX_RADIX = 256
};

static inline int64_t px_sort_tiles(int64_t n) {
    int64_t t = (n + PX_SORT_TILE - 1) / PX_SORT_TILE;
    return t < 1 ? 1 : t;
}

#endif  // PX_INTERNAL_H_
