// px_partition_rows: split the aggregated rows of a sparse variable into P disjoint shards.
//
// Parallax Sec. 3.2: partitioning divides incoming indices and values into
// disjoint sets so that aggregation and update run per partition.  A shard is
// H(id) mod P; grouping the row positions by shard is one stable counting pass
// with the shard number as the digit, so ascending ids stay ascending inside a
// shard; the scan of the per-shard totals is the offsets array.  The number of
// ids is a device scalar: the grid is sized for the capacity and every block
// clamps to the real count.  Small partitions run as a single launch (the blocks
// exchange their shard counts), larger ones as histogram and scatter launches.
#include <mutex>

#include "px_radix.h"

namespace {

struct ShardPass {
    typedef uint32_t Item;                 // position of the id in the input
    const int64_t* ids;
    const int64_t* num;
    int64_t cap;
    uint32_t n_shards;
    int mul_hash;
    int32_t* out_perm;
    int32_t* out_shard;
    int64_t* out_offsets;
    unsigned long long* pub_words;         // single-launch mode: the blocks' published shard counts
    uint32_t call_no;                      //   and the number of this call
    uint32_t* flags;                       //   the context's error flags
    int polls;                             //   polls before a block gives up waiting for another's counts

    __device__ int64_t count() const {
        int64_t n = num[0];
        if (n < 0) n = 0;
        if (n > cap) n = cap;
        return n;
    }
    __device__ unsigned long long* pub() const { return pub_words; }
    __device__ uint32_t call_number() const { return call_no; }
    __device__ void fail() const { atomicOr(flags, (uint32_t) PXF_INTERNAL); }
    __device__ int wait_polls() const { return polls; }
    __device__ Item load(int64_t i) const { return (uint32_t) i; }
    __device__ uint32_t digit(Item, int64_t i) const {
        uint64_t h = (uint64_t) ids[i];
        if (mul_hash) h *= 2654435761ull;              // wraps modulo 2^64
        if ((n_shards & (n_shards - 1u)) == 0u) return (uint32_t) h & (n_shards - 1u);
        return (uint32_t) (h % (uint64_t) n_shards);
    }
    // called by the histogram kernel, or by the scatter when there is no histogram launch
    __device__ void note(int64_t i, uint32_t d) const {
        if (out_shard) out_shard[i] = (int32_t) d;
    }
    __device__ void store(uint32_t dst, Item v) const { out_perm[dst] = (int32_t) v; }
    // offsets[p] = ids in shards below p; offsets[P] = number of ids
    __device__ void publish(int bin, uint32_t start, uint32_t grand) const {
        if (bin < (int) n_shards) out_offsets[bin] = (int64_t) start;
        if (bin == 0) out_offsets[n_shards] = (int64_t) grand;
    }
};

}  // namespace

#ifndef PX_PART_OWN_ROWS
#define PX_PART_OWN_ROWS 32     // most histogram rows a scatter thread adds up before the prefix launch pays
#endif

// Scratch of a partition call: the per-block histogram matrix, then the per-bin totals.
enum : size_t {
    PART_HIST_BYTES = (size_t) PX_SORT_MAX_BLOCKS * 256 * 4,          // a multiple of 256
    PART_TOTALS_BYTES = 256 * 4,
    PART_SCRATCH_BYTES = PART_HIST_BYTES + PART_TOTALS_BYTES
};
static_assert(PART_HIST_BYTES % 256 == 0, "the totals start 256-byte aligned");

static px_status partition_common(px_ctx* ctx, const int64_t* ids, const int64_t* num_ids, int64_t cap,
                                  int num_shards, px_hash hash, int32_t* out_shard, int32_t* out_perm,
                                  int64_t* out_offsets, void* work, bool single_launch, hipStream_t stream) {
    uint32_t* hist = (uint32_t*) work;
    uint32_t* totals = (uint32_t*) ((char*) work + PART_HIST_BYTES);
    const px_sort_geom g = px_sort_geometry(cap);
    ShardPass pol{ids, num_ids, cap, (uint32_t) num_shards, hash == PX_HASH_MUL ? 1 : 0, out_perm, out_shard, out_offsets,
                  nullptr, 0u, ctx->d_flags, ctx->wait_polls};
    // One launch when every block holds a single tile and all the blocks' shard counts together are
    // few words: the blocks count for themselves and read one another's counts from the context's
    // words (numbered by call, never cleared).
    // Not while the stream is being captured: a replayed graph would carry the same call number
    // again and again, and a block could take the counts of the replay before for this one's.
    hipStreamCaptureStatus capture = hipStreamCaptureStatusNone;
    if (single_launch && stream != nullptr && hipStreamIsCapturing(stream, &capture) != hipSuccess) {
        (void) hipGetLastError();
        capture = hipStreamCaptureStatusActive;                    // cannot tell: take the path that is always safe
    }
    if (single_launch && capture == hipStreamCaptureStatusNone && g.chunk == PX_SORT_TILE &&
        (int64_t) g.n_blocks * num_shards <= PX_PART_PUB_WORDS) {
        if (++ctx->part_call == 0u) ctx->part_call = 1u;           // 0 is what the words start with
        pol.pub_words = ctx->d_part_pub;
        pol.call_no = ctx->part_call;
        pxr::k_radix_scatter<ShardPass, 8, true><<<g.n_blocks, PX_SORT_THREADS, 0, stream>>>(pol, hist, totals, g.chunk,
                                                                                            g.n_blocks, num_shards);
        return px_check_hip(ctx, hipGetLastError(), "partition launch");
    }
    pxr::k_radix_hist<ShardPass, 8><<<g.n_blocks, PX_SORT_THREADS, 0, stream>>>(pol, hist, g.chunk);
    // Only the first num_shards bins are ever used.  While a thread of the scatter has at most
    // PX_PART_OWN_ROWS histogram rows to add up for its share of a column, every scatter block adds
    // the columns up itself and the prefix launch is saved (16 shards: any number of blocks).
    const int per_bin = PX_SORT_THREADS / num_shards;
    const bool own = (g.n_blocks + per_bin - 1) / per_bin <= PX_PART_OWN_ROWS;
    if (!own) pxr::k_radix_prefix<<<256 / 4, 256, 0, stream>>>(hist, g.n_blocks, 256, totals);
    pxr::k_radix_scatter<ShardPass, 8><<<g.n_blocks, PX_SORT_THREADS, 0, stream>>>(pol, hist, totals, g.chunk,
                                                                                  own ? g.n_blocks : 0, own ? num_shards : 0);
    return px_check_hip(ctx, hipGetLastError(), "partition launch");
}

// Host-side argument checks shared by the two entry points.
static px_status partition_check(px_ctx* ctx, const int64_t* ids, const int64_t* num_ids, int64_t cap,
                                 int num_shards, px_hash hash, const int32_t* out_perm,
                                 const int64_t* out_offsets) {
    if (num_shards < 1 || num_shards > PX_MAX_SHARDS)
        return px_fail(ctx, PX_ERR_INVALID_ARG, "num_shards %d outside [1, %d]", num_shards, (int) PX_MAX_SHARDS);
    if (hash != PX_HASH_MOD && hash != PX_HASH_MUL) return px_fail(ctx, PX_ERR_INVALID_ARG, "unknown hash %d", (int) hash);
    if (cap < 0 || cap >= (1ll << 31)) return px_fail(ctx, PX_ERR_INVALID_ARG, "cap %lld outside [0, 2^31)", (long long) cap);
    if (!num_ids || !out_offsets || (cap > 0 && (!ids || !out_perm)))
        return px_fail(ctx, PX_ERR_INVALID_ARG, "null argument");
    return PX_OK;
}

extern "C" size_t px_partition_scratch_bytes(int64_t cap) {
    if (cap < 0) return 0;
    return PART_SCRATCH_BYTES;
}

extern "C" px_status px_partition_rows(px_ctx* ctx, const int64_t* ids, const int64_t* num_ids,
                                       int64_t cap, int num_shards, px_hash hash, int32_t* out_shard,
                                       int32_t* out_perm, int64_t* out_offsets, void* work,
                                       size_t work_bytes, void* hip_stream) {
    if (!ctx) return PX_ERR_INVALID_ARG;
    px_status st = partition_check(ctx, ids, num_ids, cap, num_shards, hash, out_perm, out_offsets);
    if (st != PX_OK) return st;
    if (!work) return px_fail(ctx, PX_ERR_INVALID_ARG, "null argument");
    if (((uintptr_t) work) % 256) return px_fail(ctx, PX_ERR_INVALID_ARG, "scratch needs 256-byte alignment");
    const size_t need = px_partition_scratch_bytes(cap);
    if (work_bytes < need) return px_fail(ctx, PX_ERR_SCRATCH_TOO_SMALL, "scratch %zu < %zu bytes", work_bytes, need);
    return partition_common(ctx, ids, num_ids, cap, num_shards, hash, out_shard, out_perm, out_offsets, work, true,
                            (hipStream_t) hip_stream);
}

// ------------------------------------------------------- the variant that allocates nothing
// For callers that cannot allocate device memory or hand over a workspace (code under HIP graph
// capture, tight serving loops, harnesses that forbid hipMalloc): the histogram matrix and the
// totals live in this array, PART_SCRATCH_BYTES (513 KiB) on every GPU the library runs on, until
// the process ends.  In host code the array's name is only a handle for hipGetSymbolAddress: the
// kernels get the device address that call returned, looked up once per GPU when a context is
// created there.  Every context on a GPU shares that GPU's copy, so calls of this entry point
// that overlap on one GPU race.  Nothing in it has to start at zero: every launch writes the
// histogram rows and totals it later reads.
static __device__ __align__(256) unsigned char scratch[PART_SCRATCH_BYTES];

enum { PART_MAX_DEVICES = 64 };
static void* g_scratch_address[PART_MAX_DEVICES];     // device address of `scratch` on GPU d, null until looked up
static std::mutex g_scratch_mutex;

// Called by px_create with ctx->device current.
px_status px_partition_noalloc_setup(px_ctx* ctx) {
    if (ctx->device < 0 || ctx->device >= PART_MAX_DEVICES) {
        ctx->part_scratch = nullptr;                    // the entry point will refuse
        return PX_OK;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_address[ctx->device]) {
        void* ptr = nullptr;
        const hipError_t e = hipGetSymbolAddress((void**) &ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) return px_check_hip(ctx, e != hipSuccess ? e : hipErrorInvalidSymbol, "built-in scratch lookup");
        g_scratch_address[ctx->device] = ptr;
    }
    ctx->part_scratch = g_scratch_address[ctx->device];
    return PX_OK;
}

extern "C" px_status px_partition_rows_noalloc(px_ctx* ctx, const int64_t* ids, const int64_t* num_ids,
                                               int64_t cap, int num_shards, px_hash hash, int32_t* out_shard,
                                               int32_t* out_perm, int64_t* out_offsets, void* hip_stream) {
    if (!ctx) return PX_ERR_INVALID_ARG;
    px_status st = partition_check(ctx, ids, num_ids, cap, num_shards, hash, out_perm, out_offsets);
    if (st != PX_OK) return st;
    if (cap > (int64_t) PX_PARTITION_NOALLOC_MAX_IDS)
        return px_fail(ctx, PX_ERR_INVALID_ARG, "cap %lld is more than the %lld ids the built-in scratch serves; "
                       "use px_partition_rows with a workspace", (long long) cap, (long long) PX_PARTITION_NOALLOC_MAX_IDS);
    if (!ctx->part_scratch)
        return px_fail(ctx, PX_ERR_DEVICE, "the built-in scratch was not found on GPU %d when the context was created", ctx->device);
    // always the two-launch path on the built-in array: this entry point exists to exercise it
    return partition_common(ctx, ids, num_ids, cap, num_shards, hash, out_shard, out_perm, out_offsets,
                            ctx->part_scratch, false, (hipStream_t) hip_stream);
}
