// px_partition_rows: split the aggregated rows of a sparse variable into P disjoint shards.
//
// Parallax Sec. 3.2: partitioning divides incoming indices and values into
// disjoint sets so that aggregation and update run per partition.  A shard is
// H(id) mod P; grouping the row positions by shard is one stable counting pass
// with the shard number as the digit, so ascending ids stay ascending inside a
// shard; the scan of the per-shard totals is the offsets array.  Two kernels:
// count (shard of every id, per-block and total counts) and the pass itself.
// The number of ids is a device scalar: the grid is sized for the capacity and
// every block clamps to the real count.
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

    __device__ int64_t count() const {
        int64_t n = num[0];
        if (n < 0) n = 0;
        if (n > cap) n = cap;
        return n;
    }
    __device__ Item load(int64_t i) const { return (uint32_t) i; }
    __device__ uint32_t digit(Item, int64_t i) const {
        uint64_t h = (uint64_t) ids[i];
        if (mul_hash) h *= 2654435761ull;              // wraps modulo 2^64
        if ((n_shards & (n_shards - 1u)) == 0u) return (uint32_t) h & (n_shards - 1u);
        return (uint32_t) (h % (uint64_t) n_shards);
    }
    __device__ void store(uint32_t dst, Item v) const { out_perm[dst] = (int32_t) v; }
    // offsets[p] = ids in shards below p; offsets[P] = number of ids
    __device__ void publish(int bin, uint32_t start, uint32_t grand) const {
        if (bin < (int) n_shards) out_offsets[bin] = (int64_t) start;
        if (bin == 0) out_offsets[n_shards] = (int64_t) grand;
    }
};

// Shard of every id (written to out_shard when asked for) and the per-shard totals.  Each block
// leaves its counts in hist[block][256]; the block that finishes last adds them up.  It also
// clears what the pass needs cleared: its own tile's look-back words (every block), the ticket
// and the done counter (the last block).
__global__ __launch_bounds__(PX_SORT_THREADS) void k_shard_count(ShardPass p, uint32_t* __restrict__ hist,
                                                                 uint32_t* __restrict__ totals,
                                                                 uint64_t* __restrict__ state,
                                                                 uint32_t* __restrict__ ticket,
                                                                 uint32_t* __restrict__ done) {
    __shared__ uint32_t s_hist[PX_RADIX];
    __shared__ uint32_t s_last;
    const int tid = threadIdx.x;
    s_hist[tid] = 0u;
    state[(size_t) blockIdx.x * PX_RADIX + tid] = 0ull;
    __syncthreads();
    const int64_t n = p.count();
    const int64_t begin = (int64_t) blockIdx.x * PX_SORT_TILE;
#pragma unroll
    for (int j = 0; j < PX_SORT_ITEMS; ++j) {
        const int64_t i = begin + j * PX_SORT_THREADS + tid;
        if (i < n) {
            const uint32_t d = p.digit(0u, i);
            if (p.out_shard) p.out_shard[i] = (int32_t) d;
            atomicAdd(&s_hist[d], 1u);
        }
    }
    __syncthreads();
    hist[(size_t) blockIdx.x * PX_RADIX + tid] = s_hist[tid];
    __threadfence();                                   // this block's counts are visible before it signs off
    __syncthreads();
    if (tid == 0) s_last = (atomicAdd(done, 1u) == gridDim.x - 1u) ? 1u : 0u;
    __syncthreads();
    if (!s_last) return;
    __threadfence();
    uint32_t sum = 0;
    for (unsigned b = 0; b < gridDim.x; b += 8) {
        uint32_t v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j)
            v[j] = (b + j < gridDim.x) ? __hip_atomic_load(hist + (size_t) (b + j) * PX_RADIX + tid, __ATOMIC_RELAXED,
                                                           __HIP_MEMORY_SCOPE_AGENT)
                                       : 0u;
#pragma unroll
        for (int j = 0; j < 8; ++j) sum += v[j];
    }
    totals[tid] = sum;
    if (tid == 0) {
        ticket[0] = 0u;
        done[0] = 0u;                                  // ready for the next call on this context
    }
}

}  // namespace

extern "C" size_t px_partition_scratch_bytes(int64_t cap) {
    if (cap < 0) return 0;
    const size_t tiles = (size_t) px_sort_tiles(cap);
    return px_align_up(tiles * PX_RADIX * 8, 256)      // look-back words
           + px_align_up(tiles * PX_RADIX * 4, 256)    // per-block counts
           + px_align_up(PX_RADIX * 4, 256)            // totals
           + 256;                                      // ticket
}

extern "C" px_status px_partition_rows(px_ctx* ctx, const int64_t* ids, const int64_t* num_ids,
                                       int64_t cap, int num_shards, px_hash hash, int32_t* out_shard,
                                       int32_t* out_perm, int64_t* out_offsets, void* scratch,
                                       size_t scratch_bytes, void* hip_stream) {
    if (!ctx) return PX_ERR_INVALID_ARG;
    hipStream_t stream = (hipStream_t) hip_stream;
    if (num_shards < 1 || num_shards > PX_MAX_SHARDS)
        return px_fail(ctx, PX_ERR_INVALID_ARG, "num_shards %d outside [1, %d]", num_shards, (int) PX_MAX_SHARDS);
    if (hash != PX_HASH_MOD && hash != PX_HASH_MUL) return px_fail(ctx, PX_ERR_INVALID_ARG, "unknown hash %d", (int) hash);
    if (cap < 0 || cap >= (1ll << 31)) return px_fail(ctx, PX_ERR_INVALID_ARG, "cap %lld outside [0, 2^31)", (long long) cap);
    if (!num_ids || !out_offsets || !scratch || (cap > 0 && (!ids || !out_perm)))
        return px_fail(ctx, PX_ERR_INVALID_ARG, "null argument");
    if (((uintptr_t) scratch) % 256) return px_fail(ctx, PX_ERR_INVALID_ARG, "scratch needs 256-byte alignment");
    const size_t need = px_partition_scratch_bytes(cap);
    if (scratch_bytes < need) return px_fail(ctx, PX_ERR_SCRATCH_TOO_SMALL, "scratch %zu < %zu bytes", scratch_bytes, need);

    const size_t tiles = (size_t) px_sort_tiles(cap);
    char* base = (char*) scratch;
    uint64_t* state = (uint64_t*) base;
    base += px_align_up(tiles * PX_RADIX * 8, 256);
    uint32_t* hist = (uint32_t*) base;
    base += px_align_up(tiles * PX_RADIX * 4, 256);
    uint32_t* totals = (uint32_t*) base;
    base += px_align_up(PX_RADIX * 4, 256);
    uint32_t* ticket = (uint32_t*) base;
    ShardPass pol{ids, num_ids, cap, (uint32_t) num_shards, hash == PX_HASH_MUL ? 1 : 0, out_perm, out_shard, out_offsets};
    k_shard_count<<<(unsigned) tiles, PX_SORT_THREADS, 0, stream>>>(pol, hist, totals, state, ticket,
                                                                   ctx->d_flags + PXD_PARTITION_DONE);
    pxr::k_radix_sweep<ShardPass><<<(unsigned) tiles, PX_SORT_THREADS, 0, stream>>>(pol, totals, state, ticket, ctx->d_flags);
    return px_check_hip(ctx, hipGetLastError(), "partition launch");
}
