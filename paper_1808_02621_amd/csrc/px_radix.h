// Stable 8-bit counting pass for wave64: the building block of the id sort
// (least-significant-digit radix sort) and of the shard partition.
//
// A pass is ONE kernel.  The digit totals of the whole input are known before it
// starts (counted by the kernel that produced the input).  Every workgroup takes
// the next tile of 2048 items from a ticket counter, ranks it in LDS by wave-wide
// digit matching (ballots; one LDS counter row per wave, so equal digits keep
// their input order), publishes its per-digit counts, and learns how many items
// with each digit lie in earlier tiles by looking back over the published
// counts of its predecessors (decoupled look-back): a predecessor has published
// either its own count or already the running total up to itself.
//
// Waiting is bounded and cannot deadlock: tile numbers are handed out in the
// order workgroups start, so every tile a workgroup may wait for belongs to a
// workgroup that is already running, and tile 0 waits for nobody.  A wait that
// still exceeds PX_SPIN_LIMIT polls gives up: the tile marks its state poisoned,
// raises PXF_INTERNAL in the context's flag word and writes nothing, and every
// later tile that meets the poison does the same, so the kernel always drains.
#ifndef PX_RADIX_H_
#define PX_RADIX_H_

#include "px_internal.h"

#ifndef PX_SPIN_LIMIT
#define PX_SPIN_LIMIT (1u << 22)   // polls; a legitimate wait is a few microseconds
#endif

namespace pxr {

enum : uint64_t {
    LB_EMPTY = 0ull,
    LB_COUNT = 1ull << 62,     // low bits: items of this tile alone
    LB_TOTAL = 2ull << 62,     // low bits: items of this tile and of all tiles before it
    LB_POISON = 3ull << 62,
    LB_FLAGS = 3ull << 62
};

__device__ __forceinline__ void lb_store(uint64_t* p, uint64_t v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint64_t lb_load(const uint64_t* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Sum of the published counts of the tiles before `tile` in one state column;
// state[t * stride] is tile t's word.  False if a predecessor is poisoned or never shows up.
__device__ __forceinline__ bool look_back(const uint64_t* state, size_t stride, int64_t tile, uint32_t* sum) {
    uint32_t acc = 0;
    for (int64_t t = tile - 1; t >= 0; --t) {
        uint64_t v;
        uint32_t spins = 0;
        do {
            v = lb_load(state + (size_t) t * stride);
        } while ((v & LB_FLAGS) == LB_EMPTY && ++spins < PX_SPIN_LIMIT);
        const uint64_t f = v & LB_FLAGS;
        if (f == LB_EMPTY || f == LB_POISON) return false;
        acc += (uint32_t) v;
        if (f == LB_TOTAL) break;
    }
    *sum = acc;
    return true;
}

__device__ __forceinline__ uint32_t lane_id() { return __lane_id(); }

__device__ __forceinline__ uint64_t lanes_below() {
    uint32_t l = lane_id();
    return l == 0 ? 0ull : (~0ull >> (64u - l));
}

__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v) {
    uint32_t l = lane_id();
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        uint32_t t = __shfl_up(v, o);
        if (l >= (uint32_t) o) v += t;
    }
    return v;
}

// Exclusive scan over the 256 threads of a block; *total gets the block sum.
// s_wave: 4 words of LDS.  Contains two __syncthreads.
__device__ __forceinline__ uint32_t block_exclusive_scan_256(uint32_t v, uint32_t* s_wave,
                                                             uint32_t* total) {
    uint32_t l = lane_id(), w = threadIdx.x >> 6;
    uint32_t incl = wave_inclusive_scan(v);
    if (l == 63) s_wave[w] = incl;
    __syncthreads();
    uint32_t base = 0, tot = 0;
#pragma unroll
    for (uint32_t i = 0; i < 4; ++i) {
        uint32_t x = s_wave[i];
        if (i < w) base += x;
        tot += x;
    }
    __syncthreads();
    *total = tot;
    return base + incl - v;
}

// Policy P supplies: typedef Item; count(); load(i); digit(item, i); store(dst, item);
// publish(bin, start, grand): called once per bin by tile 0 with the bin's first output position
// and the item count.
//
// digit_totals[256]: items per digit in the whole input.  state[n_tiles][256] and ticket: zeroed
// before the launch.  Grid: at least ceil(count / PX_SORT_TILE) blocks.
template <class P>
__global__ __launch_bounds__(PX_SORT_THREADS) void k_radix_sweep(P p, const uint32_t* __restrict__ digit_totals,
                                                                 uint64_t* __restrict__ state,
                                                                 uint32_t* __restrict__ ticket,
                                                                 uint32_t* __restrict__ flags) {
    typedef typename P::Item Item;
    __shared__ Item s_items[PX_SORT_TILE];
    __shared__ uint8_t s_dig[PX_SORT_TILE];
    __shared__ uint32_t s_wcnt[4][PX_RADIX];
    __shared__ uint32_t s_binstart[PX_RADIX];
    __shared__ uint32_t s_gdst[PX_RADIX];
    __shared__ uint32_t s_wave[4];
    __shared__ uint32_t s_tile;

    const int tid = threadIdx.x;
    const uint32_t lane = lane_id();
    const int wave = tid >> 6;
    const uint64_t below = lanes_below();

    if (tid == 0) s_tile = atomicAdd(ticket, 1u);
#pragma unroll
    for (int w = 0; w < 4; ++w) s_wcnt[w][tid] = 0u;
    __syncthreads();
    const int64_t tile = (int64_t) s_tile;
    const int64_t n = p.count();
    const int64_t tile0 = tile * PX_SORT_TILE;
    if (tile0 >= n && tile > 0) return;                       // uniform: nobody waits for an empty tile
    const int tcount = (int) (n <= tile0 ? 0 : ((n - tile0) < PX_SORT_TILE ? (n - tile0) : PX_SORT_TILE));

    // Where each digit starts in the output.
    uint32_t grand;
    const uint32_t bin_start = block_exclusive_scan_256(digit_totals[tid], s_wave, &grand);
    if (tile == 0) p.publish(tid, bin_start, grand);          // also when the input is empty

    Item it[PX_SORT_ITEMS];
    uint32_t dg[PX_SORT_ITEMS], rk[PX_SORT_ITEMS];
#pragma unroll
    for (int i = 0; i < PX_SORT_ITEMS; ++i) {
        const int local = wave * (64 * PX_SORT_ITEMS) + i * 64 + (int) lane;
        const bool valid = local < tcount;
        Item v = Item(0);
        uint32_t d = 0;
        if (valid) {
            v = p.load(tile0 + local);
            d = p.digit(v, tile0 + local);
        }
        uint64_t same = __ballot(valid);
#pragma unroll
        for (int bit = 0; bit < 8; ++bit) {
            const bool one = (d >> bit) & 1u;
            const uint64_t bb = __ballot(one);
            same &= one ? bb : ~bb;
        }
        const uint32_t r = (uint32_t) __popcll(same & below);
        uint32_t old = 0;
        if (valid && r == 0) {                     // first lane holding this digit
            old = s_wcnt[wave][d];
            s_wcnt[wave][d] = old + (uint32_t) __popcll(same);
        }
        const int leader = valid ? (__ffsll((unsigned long long) same) - 1) : (int) lane;
        old = __shfl(old, leader);
        it[i] = v;
        dg[i] = d;
        rk[i] = old + r;
    }
    __syncthreads();

    // Per bin: exclusive prefix over the four waves.
    const uint32_t c0 = s_wcnt[0][tid], c1 = s_wcnt[1][tid], c2 = s_wcnt[2][tid], c3 = s_wcnt[3][tid];
    s_wcnt[0][tid] = 0u;
    s_wcnt[1][tid] = c0;
    s_wcnt[2][tid] = c0 + c1;
    s_wcnt[3][tid] = c0 + c1 + c2;
    const uint32_t tot = c0 + c1 + c2 + c3;

    // Publish this tile's count of digit `tid`, then add up the tiles before it.
    uint64_t* mine = state + (size_t) tile * PX_RADIX + tid;
    lb_store(mine, LB_COUNT | (uint64_t) tot);
    uint32_t before = 0;
    const bool ok = look_back(state + tid, PX_RADIX, tile, &before);
    if (__syncthreads_or(ok ? 0 : 1)) {
        lb_store(mine, LB_POISON);
        if (tid == 0) atomicOr(flags, (uint32_t) PXF_INTERNAL);
        return;
    }
    lb_store(mine, LB_TOTAL | (uint64_t) (before + tot));

    uint32_t tile_total;
    const uint32_t bs = block_exclusive_scan_256(tot, s_wave, &tile_total);
    s_binstart[tid] = bs;
    s_gdst[tid] = bin_start + before - bs;         // wraps; the sum below is exact mod 2^32
    __syncthreads();

#pragma unroll
    for (int i = 0; i < PX_SORT_ITEMS; ++i) {
        const int local = wave * (64 * PX_SORT_ITEMS) + i * 64 + (int) lane;
        if (local < tcount) {
            const uint32_t pos = s_binstart[dg[i]] + s_wcnt[wave][dg[i]] + rk[i];
            s_items[pos] = it[i];
            s_dig[pos] = (uint8_t) dg[i];
        }
    }
    __syncthreads();
    for (int j = tid; j < tcount; j += PX_SORT_THREADS) {
        const uint32_t d = s_dig[j];
        p.store(s_gdst[d] + (uint32_t) j, s_items[j]);
    }
}

}  // namespace pxr

#endif  // PX_RADIX_H_
