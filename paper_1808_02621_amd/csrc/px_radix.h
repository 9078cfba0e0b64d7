// Stable counting pass (8- to 11-bit digits) for wave64: the building block of the id sort
// (least-significant-digit radix sort) and of the shard partition.
//
// A pass is up to three kernels; in that form it uses no atomics on global memory and no
// waiting between workgroups:
//   hist     block b counts the digits of its chunk        -> hist[b][bins]
//   prefix   one wave per digit turns its column of hist into an exclusive prefix
//            over the blocks and writes the digit's total  -> hist[b][bins], totals[bins]
//   scatter  block b scans the totals, adds its own prefix row, then ranks its
//            chunk tile by tile in LDS and writes every item to its final place.
// With at most PX_OWN_PREFIX_BLOCKS blocks the prefix kernel is skipped: every scatter block
// adds up the (few) raw histogram rows itself, which costs less than a launch.  A pass whose
// digit takes only a few values (the shard partition) skips it at any size, and, while
// blocks x values is small, the histogram kernel too: the scatter blocks then count for
// themselves and read one another's counts (see k_radix_scatter).
// Ranking inside a tile is by wave-wide digit matching (ballots), with one LDS
// counter row per wave, so equal digits keep their input order.
#ifndef PX_RADIX_H_
#define PX_RADIX_H_

#include "px_internal.h"

namespace pxr {

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

// Policy P supplies: typedef Item; count(); load(i); digit(item, i) < 2^BITS; note(i, d);
// store(dst, item); publish(bin, start, grand): called once per bin by block 0 of the scatter
// with the bin's first output position and the item count.
//
// BITS is the digit width, 8 ... 11: 2^BITS bins, each thread of a block owns 2^BITS / 256
// consecutive bins.  Wider digits cost more LDS and a longer ranking loop per pass and save whole
// passes: ids of 17 to 22 bits sort in two passes instead of three.

template <class P, int BITS>
__global__ __launch_bounds__(PX_SORT_THREADS) void k_radix_hist(P p, uint32_t* __restrict__ hist,
                                                                int64_t chunk) {
    enum { BINS = 1 << BITS };
    __shared__ uint32_t s_hist[BINS];
    const int tid = threadIdx.x;
    for (int b = tid; b < BINS; b += PX_SORT_THREADS) s_hist[b] = 0u;
    __syncthreads();
    const int64_t n = p.count();
    const int64_t begin = (int64_t) blockIdx.x * chunk;
    int64_t end = begin + chunk;
    if (end > n) end = n;
    // PX_SORT_ITEMS items per thread at a time: their loads are requested together
    for (int64_t i0 = begin + tid; i0 < end; i0 += (int64_t) PX_SORT_THREADS * PX_SORT_ITEMS) {
        typename P::Item v[PX_SORT_ITEMS];
#pragma unroll
        for (int j = 0; j < PX_SORT_ITEMS; ++j) {
            const int64_t i = i0 + (int64_t) j * PX_SORT_THREADS;
            v[j] = i < end ? p.load(i) : typename P::Item(0);
        }
#pragma unroll
        for (int j = 0; j < PX_SORT_ITEMS; ++j) {
            const int64_t i = i0 + (int64_t) j * PX_SORT_THREADS;
            if (i < end) {
                uint32_t d = p.digit(v[j], i);
                p.note(i, d);
                atomicAdd(&s_hist[d], 1u);
            }
        }
    }
    __syncthreads();
    for (int b = tid; b < BINS; b += PX_SORT_THREADS) hist[(size_t) blockIdx.x * BINS + b] = s_hist[b];
}

// hist[b][bin] <- sum of hist[b'][bin] over b' < b;  totals[bin] <- sum over all blocks.
// Grid: bins / 4 blocks of 256 threads, one wave per bin; lane l owns blocks [l*per, (l+1)*per).
static __global__ __launch_bounds__(256) void k_radix_prefix(uint32_t* __restrict__ hist, int n_blocks, int bins,
                                                      uint32_t* __restrict__ totals) {
    enum { PER = (PX_SORT_MAX_BLOCKS + 63) / 64 };
    const uint32_t lane = lane_id();
    const int bin = (int) blockIdx.x * 4 + (int) (threadIdx.x >> 6);
    uint32_t v[PER];
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        const int b = (int) lane * PER + j;
        v[j] = b < n_blocks ? hist[(size_t) b * bins + bin] : 0u;
    }
    uint32_t sum = 0;
#pragma unroll
    for (int j = 0; j < PER; ++j) sum += v[j];
    const uint32_t incl = wave_inclusive_scan(sum);
    uint32_t run = incl - sum;
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        const int b = (int) lane * PER + j;
        if (b < n_blocks) hist[(size_t) b * bins + bin] = run;
        run += v[j];
    }
    if (lane == 63) totals[bin] = incl;
}

// own_prefix_blocks > 0: hist holds the raw counts of that many blocks and totals is not read.
// live_bins > 0 (only with own_prefix_blocks > 0): no digit reaches live_bins, and the columns of
// the live bins are added up by all threads together (256 / live_bins threads per column), so
// that a pass with few bins can skip the prefix launch at any number of blocks.
//
// SELF (needs live_bins > 0, own_prefix_blocks = the grid, and a chunk of one tile): there is no
// histogram launch either.  Every block counts its own tile, publishes the live bins' counts in
// p.pub() as 64-bit words (call number << 32 | count), and reads the words of all blocks, waiting
// for those that do not carry this call's number yet.  The call number makes clearing unnecessary:
// the words live in memory that starts at zero and only ever holds numbers of earlier calls.  The
// words are written and read with device-scope atomic accesses.  All blocks of the (small) grid are
// resident together, so the wait ends as soon as the last one has counted; it is bounded all the
// same, and a block that gives up calls p.fail() and goes on with what it has (in bounds, wrong).
template <class P, int BITS, bool SELF = false>
__global__ __launch_bounds__(PX_SORT_THREADS) void k_radix_scatter(P p, const uint32_t* __restrict__ hist,
                                                                   const uint32_t* __restrict__ totals,
                                                                   int64_t chunk, int own_prefix_blocks,
                                                                   int live_bins) {
    typedef typename P::Item Item;
    enum { BINS = 1 << BITS, BPT = BINS / PX_SORT_THREADS };      // bins per thread: tid*BPT .. tid*BPT + BPT - 1
    __shared__ Item s_items[PX_SORT_TILE];
    __shared__ uint16_t s_dig[PX_SORT_TILE];
    __shared__ uint32_t s_wcnt[4][BINS];
    __shared__ uint32_t s_binstart[BINS];
    __shared__ uint32_t s_gdst[BINS];
    __shared__ uint32_t s_wave[4];

    const int tid = threadIdx.x;
    const uint32_t lane = lane_id();
    const int wave = tid >> 6;
    const uint64_t below = lanes_below();

    const int64_t n = p.count();
    const int64_t begin = (int64_t) blockIdx.x * chunk;
    int64_t end = begin + chunk;
    if (end > n) end = n;

    // The items of a tile are requested together; those of the first tile before anything else, so
    // that they travel while the block works out where its bins start.
    Item it[PX_SORT_ITEMS];
    uint32_t dg[PX_SORT_ITEMS];
    auto load_tile = [&](int64_t tile0) {
        const int64_t left = end - tile0;
#pragma unroll
        for (int i = 0; i < PX_SORT_ITEMS; ++i) {
            const int local = wave * (64 * PX_SORT_ITEMS) + i * 64 + (int) lane;
            it[i] = Item(0);
            dg[i] = 0u;
            if ((int64_t) local < left) {
                it[i] = p.load(tile0 + local);
                dg[i] = p.digit(it[i], tile0 + local);
            }
        }
    };
    load_tile(begin);

    // Where this thread's bins start in the output, for this block.
    uint32_t gpos[BPT];
    {
        uint32_t bin_total[BPT], before[BPT];
        if (live_bins > 0) {
            // s_binstart / s_gdst double as the columns' totals / sums over the blocks before this one
            for (int b = tid; b < BINS; b += PX_SORT_THREADS) {
                s_binstart[b] = 0u;
                s_gdst[b] = 0u;
            }
            __syncthreads();
            if constexpr (SELF) {
                // own counts (in s_wcnt[0], which the tile loop clears again), published, then everyone's
                for (int b = tid; b < live_bins; b += PX_SORT_THREADS) s_wcnt[0][b] = 0u;
                __syncthreads();
#pragma unroll
                for (int i = 0; i < PX_SORT_ITEMS; ++i) {
                    const int local = wave * (64 * PX_SORT_ITEMS) + i * 64 + (int) lane;
                    if ((int64_t) local < end - begin) {
                        atomicAdd(&s_wcnt[0][dg[i]], 1u);
                        p.note(begin + local, dg[i]);
                    }
                }
                __syncthreads();
                unsigned long long* pub = p.pub();
                const unsigned long long tag = (unsigned long long) p.call_number() << 32;
                for (int b = tid; b < live_bins; b += PX_SORT_THREADS)
                    __hip_atomic_store(&pub[(size_t) blockIdx.x * live_bins + b], tag | s_wcnt[0][b], __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
                const int words = own_prefix_blocks * live_bins;
                for (int i = tid; i < words; i += PX_SORT_THREADS) {
                    const int b = i / live_bins, bin = i - b * live_bins;
                    unsigned long long v = __hip_atomic_load(&pub[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    for (int spin = 0; (v >> 32) != (tag >> 32) && spin < p.wait_polls(); ++spin) {
                        __builtin_amdgcn_s_sleep(2);
                        v = __hip_atomic_load(&pub[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    }
                    if ((v >> 32) != (tag >> 32)) {
                        p.fail();
                        v = 0ull;
                    }
                    const uint32_t c = (uint32_t) v;
                    atomicAdd(&s_binstart[bin], c);
                    if (b < (int) blockIdx.x) atomicAdd(&s_gdst[bin], c);
                }
                __syncthreads();
            }
            const int per_bin = PX_SORT_THREADS / live_bins;           // threads per column (live_bins <= 256)
            if (!SELF && tid < per_bin * live_bins) {
                const int bin = tid % live_bins, slot = tid / live_bins;
                uint32_t tot = 0u, bef = 0u;
#pragma unroll 8
                for (int b = slot; b < own_prefix_blocks; b += per_bin) {
                    const uint32_t c = hist[(size_t) b * BINS + bin];
                    tot += c;
                    bef += b < (int) blockIdx.x ? c : 0u;
                }
                atomicAdd(&s_binstart[bin], tot);
                atomicAdd(&s_gdst[bin], bef);
            }
            __syncthreads();
        }
#pragma unroll
        for (int k = 0; k < BPT; ++k) {
            const int bin = tid * BPT + k;
            if (live_bins > 0) {
                bin_total[k] = s_binstart[bin];
                before[k] = s_gdst[bin];
            } else if (own_prefix_blocks > 0) {
                bin_total[k] = 0u;
                before[k] = 0u;
#pragma unroll 8
                for (int b = 0; b < own_prefix_blocks; ++b) {
                    const uint32_t c = hist[(size_t) b * BINS + bin];
                    bin_total[k] += c;
                    before[k] += b < (int) blockIdx.x ? c : 0u;
                }
            } else {
                bin_total[k] = totals[bin];
                before[k] = hist[(size_t) blockIdx.x * BINS + bin];
            }
        }
        uint32_t mine = 0;
#pragma unroll
        for (int k = 0; k < BPT; ++k) mine += bin_total[k];
        uint32_t grand;
        uint32_t start = block_exclusive_scan_256(mine, s_wave, &grand);
#pragma unroll
        for (int k = 0; k < BPT; ++k) {
            gpos[k] = start + before[k];
            if (blockIdx.x == 0) p.publish(tid * BPT + k, start, grand);
            start += bin_total[k];
        }
    }

    for (int64_t tile0 = begin; tile0 < end; tile0 += PX_SORT_TILE) {
        const int tcount = (int) ((end - tile0) < PX_SORT_TILE ? (end - tile0) : PX_SORT_TILE);
#pragma unroll
        for (int w = 0; w < 4; ++w)
#pragma unroll
            for (int k = 0; k < BPT; ++k) s_wcnt[w][tid * BPT + k] = 0u;
        __syncthreads();

        if (tile0 != begin) load_tile(tile0);
        uint32_t rk[PX_SORT_ITEMS];
#pragma unroll
        for (int i = 0; i < PX_SORT_ITEMS; ++i) {
            const int local = wave * (64 * PX_SORT_ITEMS) + i * 64 + (int) lane;
            const bool valid = local < tcount;
            const uint32_t d = dg[i];
            uint64_t same = __ballot(valid);
#pragma unroll
            for (int bit = 0; bit < BITS; ++bit) {
                const bool one = (d >> bit) & 1u;
                const uint64_t bb = __ballot(one);
                same &= one ? bb : ~bb;
            }
            const uint32_t r = (uint32_t) __popcll(same & below);
            uint32_t old = 0;
            if (valid && r == 0) {                 // first lane holding this digit
                old = s_wcnt[wave][d];
                s_wcnt[wave][d] = old + (uint32_t) __popcll(same);
            }
            const int leader = valid ? (__ffsll((unsigned long long) same) - 1) : (int) lane;
            old = __shfl(old, leader);
            rk[i] = old + r;
        }
        __syncthreads();

        // Per bin: exclusive prefix over the four waves, then over the bins.
        uint32_t tot[BPT];
        uint32_t mine = 0;
#pragma unroll
        for (int k = 0; k < BPT; ++k) {
            const int bin = tid * BPT + k;
            const uint32_t c0 = s_wcnt[0][bin], c1 = s_wcnt[1][bin], c2 = s_wcnt[2][bin], c3 = s_wcnt[3][bin];
            s_wcnt[0][bin] = 0u;
            s_wcnt[1][bin] = c0;
            s_wcnt[2][bin] = c0 + c1;
            s_wcnt[3][bin] = c0 + c1 + c2;
            tot[k] = c0 + c1 + c2 + c3;
            mine += tot[k];
        }
        uint32_t tile_total;
        uint32_t bs = block_exclusive_scan_256(mine, s_wave, &tile_total);
#pragma unroll
        for (int k = 0; k < BPT; ++k) {
            const int bin = tid * BPT + k;
            s_binstart[bin] = bs;
            s_gdst[bin] = gpos[k] - bs;            // wraps; the sum below is exact mod 2^32
            gpos[k] += tot[k];
            bs += tot[k];
        }
        __syncthreads();

#pragma unroll
        for (int i = 0; i < PX_SORT_ITEMS; ++i) {
            const int local = wave * (64 * PX_SORT_ITEMS) + i * 64 + (int) lane;
            if (local < tcount) {
                const uint32_t pos = s_binstart[dg[i]] + s_wcnt[wave][dg[i]] + rk[i];
                s_items[pos] = it[i];
                s_dig[pos] = (uint16_t) dg[i];
            }
        }
        __syncthreads();
        for (int j = tid; j < tcount; j += PX_SORT_THREADS) {
            const uint32_t d = s_dig[j];
            p.store(s_gdst[d] + (uint32_t) j, s_items[j]);
        }
        __syncthreads();
    }
}

}  // namespace pxr

#endif  // PX_RADIX_H_
