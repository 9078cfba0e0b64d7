// px_sparse_coalesce: aggregate N workers' sparse gradients of one variable.
//
// Parallax Fig. 3 / Sec. 3.2: the workers' (indices, values) arrays are
// concatenated and values carrying the same index are accumulated.  On the GPU:
//   1. pack    every input row becomes one 64-bit word  id << 32 | worker << LB | local row
//   2. sort    stable least-significant-digit radix sort of the words on the id bits only
//              (ceil(log2 vocab) bits, 8 to 11 per pass); value rows never move
//   3. heads   a row is a run head if its id differs from its predecessor's; counting and
//              ranking the heads yields U, the distinct ids and every run's start.  Every sorted
//              word is also turned into a row reference: the address of its value row, with
//              bit 0 set on the last row of a run
//   4. segsum  the sorted order is cut into windows of T rows; tile t starts at the first head
//              in the leading quarter of window t (else at the window's own border) and ends
//              where tile t+1 starts, so the short runs that dominate never straddle two tiles
//              and tiles stay within T/4 rows of each other in length.  A lane group
//              walks its tile, gathers each value row with 128-bit loads and accumulates in
//              double.  Whole runs are rounded and written at once; a split run leaves one
//              double-precision partial row per tile
//   5. fixup   each split run adds up its partial rows, rounds once, writes its row
// The only wait on another workgroup is the head ranking's (a block reads the head counts of the
// blocks before it; bounded, see k_heads_emit), and global atomics only append to the list of
// split runs, so the sums are deterministic.
#include <string.h>

#include <type_traits>

#include "px_radix.h"
#include "px_update.h"

namespace {

// ------------------------------------------------------------------ geometry

// Tuning constants (overridable at compile time for experiments).
#ifndef PX_TILE_MIN
#define PX_TILE_MIN 32          // smallest segsum window, rows
#endif
#ifndef PX_TILE_MAX
#define PX_TILE_MAX 256         // largest segsum window, rows
#endif
#ifndef PX_TILE_TARGET
#define PX_TILE_TARGET 8192     // grow the window until there are at most this many tiles
#endif
#ifndef PX_TILE_TARGET_FUSED
#define PX_TILE_TARGET_FUSED 16384   // the fused modes do more per finished run: they like shorter tiles on long inputs
#endif
#ifndef PX_WIDE_DIGIT_BLOCKS
#define PX_WIDE_DIGIT_BLOCKS 256   // sorts of up to this many blocks (256K rows) use digits of up to 11 bits
#endif
#ifndef PX_ALIGN_DIV
#define PX_ALIGN_DIV 4          // a tile moves to a head only within the first 1/PX_ALIGN_DIV of its window
#endif

static_assert(PX_TILE_MIN >= 8 && (PX_TILE_MIN & (PX_TILE_MIN - 1)) == 0 && PX_TILE_MAX <= PX_SORT_TILE && PX_SORT_TILE / PX_TILE_MIN <= 256,
              "segsum windows are powers of two between 8 rows and one sort tile, at most 256 of them per sort tile");

// Rows per segsum window (a power of two that divides PX_SORT_TILE): enough tiles to fill the
// chip, few enough partial rows.
inline int tile_rows_for(int64_t m, bool fused) {
    const int64_t target = fused ? PX_TILE_TARGET_FUSED : PX_TILE_TARGET;
    int t = PX_TILE_MIN;
    while (t < PX_TILE_MAX && (int64_t) t * target < m) t <<= 1;
    return t;
}
static_assert(PX_TILE_TARGET_FUSED >= PX_TILE_TARGET, "scratch is carved for the fused modes' (shorter) tiles");

// How a row of `dim` elements is spread over a lane group: G lanes, C pieces per lane, E elements
// per piece; rows wider than G*C pieces take several slabs (grid.y).
struct RowShape {
    int G, C, E, pieces, slabs;
    int64_t pstride;        // doubles per partial row (padded to whole slabs)
};

inline RowShape row_shape(int64_t dim, int es, bool vec) {
    RowShape r;
    r.E = vec ? 16 / es : 1;
    r.pieces = (int) (dim / r.E);
    if (r.pieces <= 16) { r.G = 16; r.C = 1; }
    else if (r.pieces <= 32) { r.G = 32; r.C = 1; }
    else if (r.pieces <= 64) { r.G = 64; r.C = 1; }
    else if (r.pieces <= 128) { r.G = 64; r.C = 2; }
    else { r.G = 64; r.C = 4; }
    r.slabs = (r.pieces + r.G * r.C - 1) / (r.G * r.C);
    r.pstride = (int64_t) r.slabs * r.G * r.C * r.E;
    return r;
}

inline int64_t max_partial_stride(int64_t dim) {
    int64_t best = 0;
    for (int es = 2; es <= 4; es += 2)
        for (int vec = 0; vec < 2; ++vec) {
            if (vec && (dim * es) % 16) continue;
            const int64_t p = row_shape(dim, es, vec != 0).pstride;
            if (p > best) best = p;
        }
    return best;
}

// Per tile: x = first row, y = flags, z = run index of the first row, w = first head at or after the
// first row inside the tile's window (0xffffffff: none).
enum : uint32_t {
    TILE_STARTS_AT_HEAD = 1u,   // the first row is a run head
    TILE_HAS_HEAD = 2u          // some row of the tile's window is a run head
};
// A split run: x = run index, y = tile holding its first row, z = tile holding its last row.
enum { SPAN_LONG_TILES = 32 };  // runs over more tiles than this get a whole workgroup in the fix-up

struct Scratch {
    uint64_t* keys_a;
    uint64_t* keys_b;
    uint32_t* hist;        // [PX_SORT_MAX_BLOCKS][bins], bins <= PX_RADIX_MAX
    uint32_t* totals;      // [bins] items per digit
    uint32_t* hcount;      // heads per 2048-row block, top bit: published (written by the head-ranking kernel)
    uint32_t* run_start;   // [M + 1]
    uint4* tile_info;      // [n_tiles] first row, flags, run index of the first row
    uint4* span_long;      // [n_tiles] split runs over more than SPAN_LONG_TILES tiles
    uint4* span_short;     // [n_tiles] the other split runs
    uint32_t* counters;    // [0] = length of span_long, [1] = length of span_short
    double* pfirst;        // [n_tiles][pstride] partial of the run entering a tile
    double* plast;         // [n_tiles][pstride] partial of the run leaving a tile
    size_t bytes;
};

inline Scratch carve(void* base, int64_t m, int64_t dim) {
    Scratch s;
    const int t = tile_rows_for(m, true);                          // the shorter of the two: at least as many tiles
    const size_t n_tiles = (size_t) ((m + t - 1) / t);
    const size_t n_hblocks = (size_t) ((m + PX_SORT_TILE - 1) / PX_SORT_TILE);
    const size_t pstride = (size_t) max_partial_stride(dim);
    size_t off = 0;
    char* b = (char*) base;
    auto take = [&](size_t bytes) {
        char* p = b + off;
        off += px_align_up(bytes, 256);
        return p;
    };
    s.keys_a = (uint64_t*) take((size_t) m * 8);
    s.keys_b = (uint64_t*) take((size_t) m * 8);
    s.hist = (uint32_t*) take((size_t) PX_SORT_MAX_BLOCKS * PX_RADIX_MAX * 4);
    s.totals = (uint32_t*) take(PX_RADIX_MAX * 4);
    s.hcount = (uint32_t*) take((n_hblocks + 1) * 4);
    s.run_start = (uint32_t*) take(((size_t) m + 1) * 4);
    s.tile_info = (uint4*) take((n_tiles + 1) * 16);
    s.span_long = (uint4*) take((n_tiles + 1) * 16);
    s.span_short = (uint4*) take((n_tiles + 1) * 16);
    s.counters = (uint32_t*) take(64 * 4);
    s.pfirst = (double*) take(n_tiles * pstride * 8);
    s.plast = (double*) take(n_tiles * pstride * 8);
    s.bytes = off;
    return s;
}

// Addresses carried as integers are turned into pointers that name the global address space, so
// that the loads are global (not flat) instructions.
#define PX_GLOBAL __attribute__((address_space(1)))

__device__ __forceinline__ uint32_t key_of(uint64_t w) { return (uint32_t) (w >> 32); }

// ---------------------------------------------------------------------- pack

// The per-worker tables [idx pointers | value pointers | row prefix] come either from the context's
// device table (words) or, when they fit, inside the launch arguments (pack, CARRIED): then block 0
// also stores them to the device table for the kernels that follow and clears the counters, and
// the separate upload launch is saved.
template <bool CARRIED, int BITS>
__global__ __launch_bounds__(PX_SORT_THREADS) void k_pack(uint64_t* __restrict__ words, px_word_pack pack,
                                                          uint32_t* __restrict__ counters, int n_counters,
                                                          int n_workers, int64_t m, int64_t vocab,
                                                          int local_bits, uint64_t* __restrict__ keys,
                                                          uint32_t* __restrict__ hist, int64_t chunk,
                                                          uint32_t* __restrict__ flags,
                                                          uint32_t* __restrict__ hpub) {
    __shared__ uint32_t s_prefix[PX_MAX_SOURCES + 1];
    __shared__ uint64_t s_idx[CARRIED ? PX_UPLOAD_WORDS / 3 + 1 : 1];
    enum { BINS = 1 << BITS };
    __shared__ uint32_t s_hist[BINS];
    const int tid = threadIdx.x;
    if (CARRIED) {
        for (int i = tid; i <= n_workers; i += PX_SORT_THREADS) s_prefix[i] = (uint32_t) pack.w[2 * n_workers + i];
        for (int i = tid; i < n_workers; i += PX_SORT_THREADS) s_idx[i] = pack.w[i];
        if (blockIdx.x == 0) {
            for (int i = tid; i < 3 * n_workers + 1; i += PX_SORT_THREADS) words[i] = pack.w[i];
            for (int i = tid; i < n_counters; i += PX_SORT_THREADS) counters[i] = 0u;
        }
    } else {
        for (int i = tid; i <= n_workers; i += PX_SORT_THREADS) s_prefix[i] = (uint32_t) words[2 * n_workers + i];
    }
    for (int b = tid; b < BINS; b += PX_SORT_THREADS) s_hist[b] = 0u;
    __syncthreads();
    const int64_t begin = (int64_t) blockIdx.x * chunk;
    int64_t end = begin + chunk;
    if (end > m) end = m;
    // the head-ranking kernel publishes one word per PX_SORT_TILE rows: clear those of this chunk
    for (int64_t h = begin / PX_SORT_TILE + tid; h * PX_SORT_TILE < end; h += PX_SORT_THREADS) hpub[h] = 0u;
    // the chunk spans few workers: look for a row's worker only among those
    auto worker_of = [&](int64_t p, int lo, int hi) {               // s_prefix[lo] <= p < s_prefix[hi]
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if ((int64_t) s_prefix[mid] <= p) lo = mid; else hi = mid;
        }
        return lo;
    };
    int w_first = 0, w_last = 0;
    if (begin < end) {
        w_first = worker_of(begin, 0, n_workers);
        w_last = worker_of(end - 1, w_first, n_workers);
    }
    // PX_SORT_ITEMS rows per thread at a time: their ids are requested together
    for (int64_t p0 = begin + tid; p0 < end; p0 += (int64_t) PX_SORT_THREADS * PX_SORT_ITEMS) {
        uint32_t local[PX_SORT_ITEMS];
        int src[PX_SORT_ITEMS];
        int64_t id[PX_SORT_ITEMS];
#pragma unroll
        for (int j = 0; j < PX_SORT_ITEMS; ++j) {
            const int64_t p = p0 + (int64_t) j * PX_SORT_THREADS;
            id[j] = 0;
            src[j] = 0;
            local[j] = 0u;
            if (p < end) {
                const int lo = worker_of(p, w_first, w_last + 1);
                src[j] = lo;
                local[j] = (uint32_t) (p - (int64_t) s_prefix[lo]);
                const PX_GLOBAL int64_t* ids = (const PX_GLOBAL int64_t*) (CARRIED ? s_idx[lo] : words[lo]);
                id[j] = ids[local[j]];
            }
        }
#pragma unroll
        for (int j = 0; j < PX_SORT_ITEMS; ++j) {
            const int64_t p = p0 + (int64_t) j * PX_SORT_THREADS;
            if (p < end) {
                int64_t v = id[j];
                if (v < 0 || v >= vocab) {
                    atomicOr(flags, (uint32_t) PXF_BAD_ID);
                    v = 0;
                }
                keys[p] = ((uint64_t) (uint32_t) v << 32) | (uint64_t) (((uint32_t) src[j] << local_bits) | local[j]);
                atomicAdd(&s_hist[(uint32_t) v & (uint32_t) (BINS - 1)], 1u);
            }
        }
    }
    __syncthreads();
    for (int b = tid; b < BINS; b += PX_SORT_THREADS) hist[(size_t) blockIdx.x * BINS + b] = s_hist[b];
}

struct SortWords {
    typedef uint64_t Item;
    const uint64_t* in;
    uint64_t* out;
    int64_t n;
    int shift;                                      // bit offset inside the id
    uint32_t mask;                                  // 2^digit width - 1
    __device__ int64_t count() const { return n; }
    __device__ Item load(int64_t i) const { return in[i]; }
    __device__ uint32_t digit(Item v, int64_t) const { return (uint32_t) (v >> (32 + shift)) & mask; }
    __device__ void note(int64_t, uint32_t) const {}
    __device__ void store(uint32_t dst, Item v) const { out[dst] = v; }
    __device__ void publish(int, uint32_t, uint32_t) const {}
};

// --------------------------------------------------------------------- heads

// Ranks the heads: distinct ids, run starts, U; and for every window of tile_rows rows the tile
// that starts there: its first row (the first head in the leading part of the window, else the
// window's own first row), the run that row belongs to, and the first head at or after that row
// inside the window.  It also writes every row's reference for the segmented sum: the address of
// its value row, with bit 0 set when the row is the last of its run (value rows are at least
// 2-byte aligned, so the bit is free).
//
// The rank of a head needs the number of heads in all blocks before this one.  Every block
// publishes its own count in hpub (cleared by the pack kernel) with the top bit as the "valid"
// mark, then reads the words of all blocks before it, waiting for those not yet valid.  A block
// only ever waits for blocks with smaller numbers, which the hardware starts no later than it, and
// those never wait for it; the wait is bounded all the same (wait_polls polls), and a block that
// gives up raises PXF_INTERNAL: its ranks are then too small, which keeps every store of this kernel
// in bounds, and the kernels that would follow the ranks (segmented sum, fix-up) leave at once.  The words are written and read with device-scope atomic accesses, which the
// dies' separate L2 caches do not hold back.
__global__ __launch_bounds__(256) void k_heads_emit(const uint64_t* __restrict__ sorted, int64_t m,
                                                    uint32_t* __restrict__ hpub, int tile_rows,
                                                    const uint64_t* __restrict__ words, int n_workers,
                                                    int local_bits, int64_t row_bytes,
                                                    uint64_t* __restrict__ rowref,
                                                    int64_t* __restrict__ out_ids,
                                                    uint32_t* __restrict__ run_start,
                                                    uint4* __restrict__ tile_info,
                                                    int64_t* __restrict__ out_num_unique,
                                                    uint32_t* __restrict__ flags, int wait_polls) {
    __shared__ uint32_t s_wave[4];
    __shared__ uint32_t s_first[PX_SORT_TILE / PX_TILE_MIN];        // first aligning head of each window of this block
    __shared__ uint32_t s_head[PX_SORT_TILE / PX_TILE_MIN];         // first head of the window, 0xffffffff if it has none
    __shared__ uint64_t s_vbase[PX_MAX_SOURCES];           // the workers' value buffers
    const int tid = threadIdx.x;
    if (tid < PX_SORT_TILE / PX_TILE_MIN) {
        s_first[tid] = 0xffffffffu;
        s_head[tid] = 0xffffffffu;
    }
    for (int i = tid; i < n_workers; i += 256) s_vbase[i] = words[n_workers + i];
    __syncthreads();

    const uint32_t block_base = blockIdx.x * (uint32_t) PX_SORT_TILE;
    const int64_t base = (int64_t) block_base + (int64_t) tid * PX_SORT_ITEMS;
    // A head at a window's first row always starts the tile (align_rows >= 1), so every tile gets a start.
    const uint32_t align_rows = (uint32_t) tile_rows / PX_ALIGN_DIV > 0u ? (uint32_t) tile_rows / PX_ALIGN_DIV : 1u;
    uint64_t w[PX_SORT_ITEMS];
    uint32_t flag[PX_SORT_ITEMS];
    uint32_t prev = 0;
    if (base > 0 && base - 1 < m) prev = key_of(sorted[base - 1]);
    uint32_t cnt = 0;
#pragma unroll
    for (int j = 0; j < PX_SORT_ITEMS; ++j) w[j] = (base + j < m) ? sorted[base + j] : 0ull;
#pragma unroll
    for (int j = 0; j < PX_SORT_ITEMS; ++j) {
        const int64_t i = base + j;
        flag[j] = 0;
        if (i < m) {
            flag[j] = (i == 0 || key_of(w[j]) != prev) ? 1u : 0u;
            prev = key_of(w[j]);
            if (flag[j]) {
                const uint32_t win = ((uint32_t) i - block_base) / (uint32_t) tile_rows;
                atomicMin(&s_head[win], (uint32_t) i);
                if ((uint32_t) i % (uint32_t) tile_rows < align_rows) atomicMin(&s_first[win], (uint32_t) i);
            }
        }
        cnt += flag[j];
    }
    uint32_t block_total;
    uint32_t rank = pxr::block_exclusive_scan_256(cnt, s_wave, &block_total);   // syncs
    if (tid == 0)
        __hip_atomic_store(&hpub[blockIdx.x], 0x80000000u | block_total, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const uint32_t local_mask = (local_bits >= 32) ? 0xffffffffu : ((1u << local_bits) - 1u);
    // row references, consecutive lanes on consecutive rows so that the stores coalesce; they need no
    // rank, so they are written while the other blocks' counts are on their way
#pragma unroll
    for (int j = 0; j < PX_SORT_ITEMS; ++j) {
        const int64_t i = (int64_t) block_base + j * 256 + tid;
        if (i < m) {
            const uint64_t wi = sorted[i];
            const bool tail = i + 1 >= m || key_of(sorted[i + 1]) != key_of(wi);
            const uint32_t payload = (uint32_t) wi;
            const uint32_t worker = (local_bits >= 32) ? 0u : (payload >> local_bits);
            rowref[i] = (s_vbase[worker] + (uint64_t) (payload & local_mask) * (uint64_t) row_bytes) | (tail ? 1ull : 0ull);
        }
    }
    // heads in all blocks before this one
    uint32_t part = 0;
    for (int b = tid; b < (int) blockIdx.x; b += 256) {
        uint32_t v = __hip_atomic_load(&hpub[b], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        for (int spin = 0; !(v & 0x80000000u) && spin < wait_polls; ++spin) {
            __builtin_amdgcn_s_sleep(2);
            v = __hip_atomic_load(&hpub[b], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        if (!(v & 0x80000000u)) {
            atomicOr(flags, (uint32_t) PXF_INTERNAL);      // never seen: the ranks of this call are wrong, and say so
            v = 0u;
        }
        part += v & 0x7fffffffu;
    }
    uint32_t before;
    pxr::block_exclusive_scan_256(part, s_wave, &before);
    rank += before;
#pragma unroll
    for (int j = 0; j < PX_SORT_ITEMS; ++j) {
        const int64_t i = base + j;
        if (i < m) {
            const uint32_t win = ((uint32_t) i - block_base) / (uint32_t) tile_rows;
            const uint32_t t = (uint32_t) i / (uint32_t) tile_rows;
            if (flag[j]) {
                out_ids[rank] = (int64_t) key_of(w[j]);
                run_start[rank] = (uint32_t) i;
                if (s_first[win] == (uint32_t) i)
                    tile_info[t] = make_uint4((uint32_t) i, TILE_STARTS_AT_HEAD | TILE_HAS_HEAD, rank, (uint32_t) i);
                ++rank;
            } else if ((uint32_t) i % (uint32_t) tile_rows == 0u && s_first[win] == 0xffffffffu) {
                // no head to move to: the tile keeps its border and continues the run row i belongs to
                tile_info[t] = make_uint4((uint32_t) i, s_head[win] != 0xffffffffu ? TILE_HAS_HEAD : 0u, rank - 1u,
                                          s_head[win]);
            }
        }
    }
    if (tid == 0 && (int64_t) (blockIdx.x + 1) * PX_SORT_TILE >= m) {     // block holding the last row
        const uint32_t u = before + block_total;
        run_start[u] = (uint32_t) m;
        out_num_unique[0] = (flags[0] & PXF_BAD_ID) ? 0 : (int64_t) u;
    }
}

__global__ void k_write_zero_count(int64_t* out_num_unique) {
    if (threadIdx.x == 0 && blockIdx.x == 0) out_num_unique[0] = 0;
}

// -------------------------------------------------------------------- segsum

#ifndef PX_SEG_ACC
#define PX_SEG_ACC double       // accumulator type of the segmented sum
#endif
#ifndef PX_SEG_ROWS
#define PX_SEG_ROWS 8           // rows per batch and lane group, one piece per lane (two batches are in flight)
#endif
#ifndef PX_SEG_ROWS_2
#define PX_SEG_ROWS_2 4         // two pieces per lane
#endif
#ifndef PX_SEG_ROWS_WIDE
#define PX_SEG_ROWS_WIDE 2      // four pieces per lane
#endif
#ifndef PX_FUSED_STATE_PIECES
#define PX_FUSED_STATE_PIECES 8 // fused modes: 16-byte table / accumulator pieces a lane holds per batch
#endif
typedef PX_SEG_ACC seg_acc_t;

typedef uint32_t seg_v4u __attribute__((ext_vector_type(4)));
// Value rows are read exactly once.
__device__ __forceinline__ uint4 seg_load16(const char* p) {
    const PX_GLOBAL seg_v4u* g = (const PX_GLOBAL seg_v4u*) (uintptr_t) p;
#ifdef PX_SEG_TEMPORAL
    seg_v4u v = *g;
#else
    seg_v4u v = __builtin_nontemporal_load(g);      // stream past the caches
#endif
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ float seg_load_f32(const char* p) { return *(const PX_GLOBAL float*) (uintptr_t) p; }
__device__ __forceinline__ uint16_t seg_load_u16(const char* p) { return *(const PX_GLOBAL uint16_t*) (uintptr_t) p; }

typedef float seg_v4f __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void seg_store16(float* p, float4 v) {
#ifdef PX_SEG_NT_STORE
    seg_v4f t = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(t, (seg_v4f*) p);
#else
    *(float4*) p = v;
#endif
}

template <typename T, bool VEC> struct RowLoad;

template <> struct RowLoad<float, true> {
    typedef uint4 Raw;
    enum { E = 4 };
    static __device__ __forceinline__ Raw load(const char* p) { return seg_load16(p); }
    static __device__ __forceinline__ void add(seg_acc_t* acc, const Raw& r) {
        acc[0] += (seg_acc_t) __uint_as_float(r.x);
        acc[1] += (seg_acc_t) __uint_as_float(r.y);
        acc[2] += (seg_acc_t) __uint_as_float(r.z);
        acc[3] += (seg_acc_t) __uint_as_float(r.w);
    }
};
template <> struct RowLoad<float, false> {
    typedef float Raw;
    enum { E = 1 };
    static __device__ __forceinline__ Raw load(const char* p) { return seg_load_f32(p); }
    static __device__ __forceinline__ void add(seg_acc_t* acc, const Raw& r) { acc[0] += (seg_acc_t) r; }
};
// bfloat16 is the upper half of a float32: widening is a shift.
template <> struct RowLoad<uint16_t, true> {
    typedef uint4 Raw;
    enum { E = 8 };
    static __device__ __forceinline__ Raw load(const char* p) { return seg_load16(p); }
    static __device__ __forceinline__ void add(seg_acc_t* acc, const Raw& r) {
        acc[0] += (seg_acc_t) __uint_as_float(r.x << 16);
        acc[1] += (seg_acc_t) __uint_as_float(r.x & 0xffff0000u);
        acc[2] += (seg_acc_t) __uint_as_float(r.y << 16);
        acc[3] += (seg_acc_t) __uint_as_float(r.y & 0xffff0000u);
        acc[4] += (seg_acc_t) __uint_as_float(r.z << 16);
        acc[5] += (seg_acc_t) __uint_as_float(r.z & 0xffff0000u);
        acc[6] += (seg_acc_t) __uint_as_float(r.w << 16);
        acc[7] += (seg_acc_t) __uint_as_float(r.w & 0xffff0000u);
    }
};
template <> struct RowLoad<uint16_t, false> {
    typedef uint16_t Raw;
    enum { E = 1 };
    static __device__ __forceinline__ Raw load(const char* p) { return seg_load_u16(p); }
    static __device__ __forceinline__ void add(seg_acc_t* acc, const Raw& r) {
        acc[0] += (seg_acc_t) __uint_as_float((uint32_t) r << 16);
    }
};

enum { MODE_ROWS = 0, MODE_SGD = 1, MODE_ADAGRAD = 2 };   // what becomes of a finished run

struct SegsumArgs {
    const uint64_t* rowref;       // per row in id order: address of its value row | 1 if it ends its run
    const uint64_t* sorted;       // packed words in id order (the fused modes read the ids)
    const uint4* tile_info;
    const uint32_t* run_start;
    double* pfirst;
    double* plast;
    uint4* span_long;
    uint4* span_short;
    uint32_t* counters;
    float* out_rows;              // MODE_ROWS: the aggregated rows
    float* table;                 // fused modes: the variable, updated in place
    float* accum;                 // MODE_ADAGRAD: its accumulator
    const uint32_t* flags;
    int64_t m;
    int64_t n_tiles;
    int64_t dim;                  // elements per row
    int64_t pstride;              // doubles per partial row
    int tile_rows;
    int pieces;                   // row pieces (E elements each) per row
    float scale;
    float lr;
    float eps;
};

// G lanes walk one tile; lane l owns pieces slab*G*C + c*G + l, c < C, E elements each.
// A partial row is stored lane-interleaved so that every store instruction writes one contiguous
// block: pair p of piece c sits at ((slab*C + c)*(E/2) + p)*G + l.
//
// A tile is walked in two stretches.  Rows before its first head continue the run that entered
// from the tile before: they are only added up, and the sum is left as the tile's "first" partial
// row.  From the first head on, every row whose reference carries the tail bit finishes a run that
// lies wholly inside the tile: MODE_ROWS writes its sum as a float row, the fused modes apply the
// optimizer to the variable's row instead (Parallax Sec. 4.3 puts the aggregation next to the
// variable so the aggregate never travels).  What is left when the tile ends belongs to a run
// that goes on into the next tile (the "last" partial row).
//
// Each stretch keeps two batches of rows in flight (B rows each in the stretch with tails, BH in the
// stretch without heads; they differ only in the fused modes): while batch k is added up, the rows of
// batch k + 1 (and, in the fused modes, the table and accumulator rows of its tails) are on
// their way and the references of batch k + 2 are being fetched.  Loads are unconditional, so the
// hardware counters tell exactly which of them a wait is for: past the end of the stretch they
// repeat its last row, and lanes beyond the row's width read piece 0; neither is used.
//
// A block holds 256/G consecutive tiles.  When all of them lie strictly inside one run (no head
// inside, and the run goes on into the next block) their sums are added in LDS, in tile order,
// and stored once, as the partial row of the block's first tile: a long run then leaves one
// partial row per block instead of one per tile.
template <typename T, bool VEC, int G, int C, int B, int BH, int MODE>
__global__ __launch_bounds__(256) void k_segsum(SegsumArgs a) {
    typedef RowLoad<T, VEC> L;
    typedef typename L::Raw Raw;
    enum { E = L::E, TPB = 256 / G, MERGE = (C * E <= 16) ? 1 : 0, FUSED = MODE != MODE_ROWS ? 1 : 0,
           SV = VEC ? E / 4 : 1 };                                // state vectors (float4 or float) per piece
    typedef typename std::conditional<VEC, float4, float>::type StateV;
    __shared__ double s_part[MERGE ? TPB * G * C * E : 1];
    // uniform: the head ranking gave up a wait, so ranks and run starts cannot be trusted (any mode);
    // or, fused modes, an error flag is up: touch nothing
    if ((a.flags[0] & PXF_INTERNAL) || (FUSED && a.flags[0])) return;

    const int gl = threadIdx.x % G;
    const int gj = threadIdx.x / G;                               // tile inside the block
    const int64_t tile = (int64_t) blockIdx.x * TPB + gj;
    const bool active = tile < a.n_tiles;
    int64_t s = 0, e = 0, h = 0;
    bool started = false, next_is_head = true;
    uint32_t u = 0;
    if (active) {
        const uint4 ti = a.tile_info[tile];
        s = (int64_t) ti.x;
        started = (ti.y & TILE_STARTS_AT_HEAD) != 0u;
        u = ti.z;
        e = a.m;
        if (tile + 1 < a.n_tiles) {
            const uint4 tn = a.tile_info[tile + 1];
            e = (int64_t) tn.x;
            next_is_head = (tn.y & TILE_STARTS_AT_HEAD) != 0u;
        }
        h = (int64_t) ti.w < e ? (int64_t) ti.w : e;              // first head inside the tile, else its end
    }
    // no head inside; the last tile of the block also vouches for the run going on into the next block
    const bool inside = active && h >= e && (gj < TPB - 1 || !next_is_head);
    const bool merged = MERGE ? (__syncthreads_and(inside ? 1 : 0) != 0) : false;

    int piece[C];
    bool live[C];
    size_t piece_off[C];
#pragma unroll
    for (int c = 0; c < C; ++c) {
        piece[c] = (int) blockIdx.y * (G * C) + c * G + gl;
        live[c] = piece[c] < a.pieces;
        piece_off[c] = (size_t) (live[c] ? piece[c] : 0) * (E * sizeof(T));
    }

    seg_acc_t acc[C][E];
    auto clear = [&]() {
#pragma unroll
        for (int c = 0; c < C; ++c)
#pragma unroll
            for (int x = 0; x < E; ++x) acc[c][x] = (seg_acc_t) 0;
    };
    clear();

    auto store_partial = [&](double* dst) {
#pragma unroll
        for (int c = 0; c < C; ++c) {
            const size_t sc = (size_t) blockIdx.y * C + c;
            if (VEC) {
#pragma unroll
                for (int x = 0; x < E; x += 2)
                    *(double2*) (dst + ((sc * (E / 2) + x / 2) * G + gl) * 2) =
                        make_double2((double) acc[c][x], (double) acc[c][x + 1]);
            } else {
                dst[sc * G + gl] = (double) acc[c][0];
            }
        }
    };

    // Rows [from, to), from < to, are added to acc, BB rows per batch.  With TAILS, a row whose
    // reference carries the tail bit finishes run u: its sum is written (or applied) and acc starts
    // again.  Only the fused modes' stretch with tails holds table (and accumulator) pieces, so only
    // that stretch needs the smaller batches; a stretch without heads streams at the full depth.
    auto walk = [&](int64_t from, int64_t to, auto tails_tag, auto batch_tag) {
        constexpr bool TAILS = decltype(tails_tag)::value;
        constexpr bool STATE = TAILS && FUSED;
        constexpr int BB = decltype(batch_tag)::value;
        constexpr int FBB = STATE ? BB : 1, ABB = (STATE && MODE == MODE_ADAGRAD) ? BB : 1;
        const int64_t lastrow = to - 1;
        uint64_t wn[BB], wf[BB];                                  // references of the next batch and the one after
        uint32_t kc[FBB], kn[FBB], kf[FBB];                       // fused modes: the rows' ids
        Raw rc[BB][C], rn[BB][C];
        uint32_t tc = 0, tn = 0;                                  // tail bits of the current and the next batch
        StateV wsc[FBB][C][SV], wsn[FBB][C][SV];
        StateV asc[ABB][C][SV], asn[ABB][C][SV];
        float* dst = a.out_rows + (size_t) u * a.dim + (size_t) piece[0] * E;   // MODE_ROWS: lane's place in row u

        auto load_refs = [&](int64_t r0, uint64_t (&w)[BB], uint32_t (&k)[FBB]) {
#pragma unroll
            for (int j = 0; j < BB; ++j) {
                const int64_t i = r0 + j < to ? r0 + j : lastrow;
                w[j] = a.rowref[i];
                if (STATE) k[STATE ? j : 0] = ((const uint32_t*) a.sorted)[2 * i + 1];
            }
        };
        auto load_rows = [&](const uint64_t (&w)[BB], Raw (&raw)[BB][C]) {
#pragma unroll
            for (int j = 0; j < BB; ++j) {
                const char* row = (const char*) (w[j] & ~1ull);
#pragma unroll
                for (int c = 0; c < C; ++c) raw[j][c] = L::load(row + piece_off[c]);
            }
        };
        auto tails_of = [&](int64_t r0, const uint64_t (&w)[BB]) -> uint32_t {
            if (!TAILS) return 0u;
            uint32_t t = 0;
#pragma unroll
            for (int j = 0; j < BB; ++j) t |= ((uint32_t) w[j] & 1u) << j;
            const int64_t left = to - r0;
            return left >= BB ? t : (left > 0 ? t & ((1u << (int) left) - 1u) : 0u);
        };
        auto load_state = [&](uint32_t t, const uint32_t (&k)[FBB], StateV (&ws)[FBB][C][SV], StateV (&as)[ABB][C][SV]) {
            if (!STATE) return;
#pragma unroll
            for (int j = 0; j < BB; ++j)
                if ((t >> j) & 1u) {
                    const size_t off = (size_t) k[STATE ? j : 0] * a.dim;
#pragma unroll
                    for (int c = 0; c < C; ++c)
                        if (live[c]) {
#pragma unroll
                            for (int v = 0; v < SV; ++v) {
                                ws[STATE ? j : 0][c][v] = ((const StateV*) (a.table + off + (size_t) piece[c] * E))[v];
                                if (MODE == MODE_ADAGRAD)
                                    as[ABB > 1 ? j : 0][c][v] = ((const StateV*) (a.accum + off + (size_t) piece[c] * E))[v];
                            }
                        }
                }
        };
        // row j of the current batch is the last of run u
        auto finish = [&](int j) {
            if (!FUSED) {
#ifndef PX_SEG_NO_EXCHANGE
                if (VEC && E == 8) {
                    // A piece of 8 bfloat16 becomes 32 bytes of output.  Lanes trade halves so that each
                    // store instruction writes one contiguous block of G*16 bytes: in store h lane l
                    // writes half (l & 1) of piece h*G/2 + l/2 of the lane group's block.
#pragma unroll
                    for (int c = 0; c < C; ++c) {
                        float o[8];
#pragma unroll
                        for (int x = 0; x < 8; ++x) o[x] = (float) ((double) acc[c][x < E ? x : 0] * a.scale);
#pragma unroll
                        for (int hh = 0; hh < 2; ++hh) {
                            const int src = hh * (G / 2) + (gl >> 1);
                            float lo[4], hi[4];
#pragma unroll
                            for (int x = 0; x < 4; ++x) {
                                lo[x] = __shfl(o[x], src, G);
                                hi[x] = __shfl(o[4 + x], src, G);
                            }
                            const bool odd = (gl & 1) != 0;
                            const float4 v = make_float4(odd ? hi[0] : lo[0], odd ? hi[1] : lo[1], odd ? hi[2] : lo[2],
                                                         odd ? hi[3] : lo[3]);
                            if ((int) blockIdx.y * (G * C) + c * G + src < a.pieces)
                                seg_store16(dst + (size_t) c * (G * 8) + hh * (G * 4) - gl * 4, v);
                        }
                    }
                } else
#endif
#pragma unroll
                for (int c = 0; c < C; ++c)
                    if (live[c]) {
                        if (VEC) {
#pragma unroll
                            for (int x = 0; x < E; x += 4) {
                                float4 o = make_float4((float) ((double) acc[c][x] * a.scale), (float) ((double) acc[c][x + 1] * a.scale),
                                                       (float) ((double) acc[c][x + 2] * a.scale), (float) ((double) acc[c][x + 3] * a.scale));
                                seg_store16(dst + (size_t) c * (G * E) + x, o);
                            }
                        } else {
                            dst[(size_t) c * G] = (float) ((double) acc[c][0] * a.scale);
                        }
                    }
                dst += a.dim;
            } else {
                const size_t off = (size_t) kc[STATE ? j : 0] * a.dim;
#pragma unroll
                for (int c = 0; c < C; ++c)
                    if (live[c]) {
                        float* wf32 = (float*) &wsc[STATE ? j : 0][c][0];
                        float* af32 = (float*) &asc[ABB > 1 ? j : 0][c][0];
#pragma unroll
                        for (int x = 0; x < E; ++x) {
                            const float g = (float) ((double) acc[c][x] * a.scale);
                            if (MODE == MODE_ADAGRAD) pxu::adagrad(wf32[x], af32[x], g, a.lr, a.eps);
                            else pxu::sgd(wf32[x], g, a.lr);
                        }
#pragma unroll
                        for (int v = 0; v < SV; ++v) {
                            ((StateV*) (a.table + off + (size_t) piece[c] * E))[v] = wsc[STATE ? j : 0][c][v];
                            if (MODE == MODE_ADAGRAD)
                                ((StateV*) (a.accum + off + (size_t) piece[c] * E))[v] = asc[ABB > 1 ? j : 0][c][v];
                        }
                    }
            }
            ++u;
            clear();
        };

        {
            uint64_t w0[BB];
            load_refs(from, w0, kc);
            load_refs(from + BB, wn, kn);
            load_rows(w0, rc);
            tc = tails_of(from, w0);
            load_state(tc, kc, wsc, asc);
        }
        for (int64_t r = from; r < to; r += BB) {
            // Loads come back in the order they were issued, so the references of batch k + 2 go out
            // before the rows of batch k + 1: the next iteration then finds them without having to
            // wait for those rows, and two batches of rows really are in flight.
            load_refs(r + 2 * BB, wf, kf);
            load_rows(wn, rn);
            tn = tails_of(r + BB, wn);
            load_state(tn, kn, wsn, asn);
            if (r + BB <= to) {
#pragma unroll
                for (int j = 0; j < BB; ++j) {
#pragma unroll
                    for (int c = 0; c < C; ++c)
                        if (live[c]) L::add(acc[c], rc[j][c]);
                    if (TAILS && ((tc >> j) & 1u)) finish(j);
                }
            } else {
#pragma unroll
                for (int j = 0; j < BB; ++j)
                    if (r + j < to) {
#pragma unroll
                        for (int c = 0; c < C; ++c)
                            if (live[c]) L::add(acc[c], rc[j][c]);
                        if (TAILS && ((tc >> j) & 1u)) finish(j);
                    }
            }
            tc = tn;
#pragma unroll
            for (int j = 0; j < BB; ++j) {
                wn[j] = wf[j];
#pragma unroll
                for (int c = 0; c < C; ++c) rc[j][c] = rn[j][c];
            }
            if (STATE) {
#pragma unroll
                for (int j = 0; j < FBB; ++j) {
                    kc[j] = kn[j];
                    kn[j] = kf[j];
#pragma unroll
                    for (int c = 0; c < C; ++c)
#pragma unroll
                        for (int v = 0; v < SV; ++v) {
                            wsc[j][c][v] = wsn[j][c][v];
                            if (MODE == MODE_ADAGRAD) asc[ABB > 1 ? j : 0][c][v] = asn[ABB > 1 ? j : 0][c][v];
                        }
                }
            }
        }
    };

    if (active) {
        if (!started) {
            // the run that entered from the tile before
            walk(s, h, std::false_type(), std::integral_constant<int, BH>());
            if (h < e) {
                store_partial(a.pfirst + (size_t) tile * a.pstride);
                clear();
                ++u;
            } else if (!merged) {
                store_partial(a.pfirst + (size_t) tile * a.pstride);
            }
        }
        if (h < e) {
            walk(h, e, std::true_type(), std::integral_constant<int, B>());
            if (!next_is_head) {
                // the tile's last run goes on into the next tile
                store_partial(a.plast + (size_t) tile * a.pstride);
                if (gl == 0 && blockIdx.y == 0) {
                    // record where the run ends
                    const uint32_t last_row = a.run_start[u + 1] - 1u;
                    uint32_t last_tile = last_row / (uint32_t) a.tile_rows;
                    if (a.tile_info[last_tile].x > last_row) --last_tile;
                    const bool is_long = last_tile - (uint32_t) tile > (uint32_t) SPAN_LONG_TILES;
                    const uint32_t slot = atomicAdd(a.counters + (is_long ? 0 : 1), 1u);
                    (is_long ? a.span_long : a.span_short)[slot] = make_uint4(u, (uint32_t) tile, last_tile, 0u);
                }
            }
        }
    }

    if (MERGE && merged) {                                    // uniform over the block
        // every tile of the block is a continuation of one run with no head inside: add in tile order
#pragma unroll
        for (int c = 0; c < C; ++c)
#pragma unroll
            for (int x = 0; x < E; ++x) s_part[((gj * C + c) * E + x) * G + gl] = (double) acc[c][x];
        __syncthreads();
        if (gj == 0) {
#pragma unroll
            for (int c = 0; c < C; ++c)
#pragma unroll
                for (int x = 0; x < E; ++x) {
                    double t = s_part[((0 * C + c) * E + x) * G + gl];
                    for (int j = 1; j < TPB; ++j) t += s_part[((j * C + c) * E + x) * G + gl];
                    acc[c][x] = (seg_acc_t) t;
                }
            store_partial(a.pfirst + (size_t) tile * a.pstride);
        }
    }
}

// -------------------------------------------------------------------- fix-up
// A run split over tiles first..last left partial rows plast[first], then pfirst[t] for the tiles
// after it -- except that a block of tiles_per_block tiles lying strictly inside the run left a
// single row, at its first tile.  Rows are added in double, rounded once and written to the
// column each slot of the lane-interleaved partial row stands for.
//   long runs   one workgroup of 16 waves per run and 64-slot slab: wave w adds parts w, w+16, ...,
//               the 16 sums are added in wave order
//   other runs  one wave per run and slab
enum { FIX_SPLITS = 16 };
#ifndef PX_FIXUP_DEPTH
#define PX_FIXUP_DEPTH 8         // partial rows a wave of a long run's workgroup requests at a time
#endif
#ifndef PX_FIXUP_RESIDENT
#define PX_FIXUP_RESIDENT 256    // workgroups of 16 waves in one fix-up launch (measured: 128 and 512 are slower)
#endif

struct FixupArgs {
    int mode;                     // MODE_ROWS, MODE_SGD or MODE_ADAGRAD
    float* table;
    float* accum;
    const int64_t* out_ids;
    const uint32_t* flags;
    float lr, eps;
    const uint4* span_long;
    const uint4* span_short;
    const uint32_t* counters;
    const uint32_t* run_start;
    const double* pfirst;
    const double* plast;
    float* out_rows;
    int32_t* out_run_len;
    const int64_t* num_unique;
    int64_t dim;
    int64_t pstride;
    int tiles_per_block;          // 0: the segsum kernel never merges
    int G, C, E, pieces;
    float scale;
};

// The q-th partial row (q = 0 .. parts-1) of a run over tiles first..last.
struct PartList {
    uint32_t first, heads, merged, g0, g1, tpb, parts;
    __device__ PartList(uint32_t first_tile, uint32_t last_tile, uint32_t tiles_per_block) {
        first = first_tile;
        tpb = tiles_per_block;
        heads = last_tile - first_tile;        // no merged block: every later tile is its own part
        merged = 0;
        g0 = g1 = 0;
        if (tpb > 0) {
            const uint32_t lo = (first_tile + 1u + tpb - 1u) / tpb;      // first block starting after `first`
            const uint32_t hi = last_tile / tpb;                         // blocks below hi end before `last`
            if (lo < hi) {
                g0 = lo;
                g1 = hi;
                heads = g0 * tpb - (first_tile + 1u);
                merged = g1 - g0;
            }
        }
        const uint32_t tail = merged ? last_tile - g1 * tpb + 1u : 0u;
        parts = 1u + heads + merged + tail;
    }
    __device__ const double* row(uint32_t q, const double* pfirst, const double* plast, int64_t pstride) const {
        if (q == 0) return plast + (size_t) first * pstride;
        uint32_t t;
        if (q <= heads) t = first + q;
        else if (q <= heads + merged) t = (g0 + (q - heads - 1u)) * tpb;
        else t = g1 * tpb + (q - heads - merged - 1u);
        return pfirst + (size_t) t * pstride;
    }
};

// What becomes of a split run's column once its sum is known.
__device__ __forceinline__ void fixup_finish(const FixupArgs& a, uint32_t u, int64_t col, double sum) {
    const float g = (float) (sum * a.scale);
    if (a.mode == MODE_ROWS) {
        a.out_rows[(size_t) u * a.dim + col] = g;
        return;
    }
    const size_t at = (size_t) a.out_ids[u] * a.dim + col;
    float w = a.table[at];
    if (a.mode == MODE_ADAGRAD) {
        float acc = a.accum[at];
        pxu::adagrad(w, acc, g, a.lr, a.eps);
        a.accum[at] = acc;
    } else {
        pxu::sgd(w, g, a.lr);
    }
    a.table[at] = w;
}

__global__ __launch_bounds__(64 * FIX_SPLITS) void k_fixup(FixupArgs a) {
    __shared__ double s_red[FIX_SPLITS][64];
    if ((a.flags[0] & PXF_INTERNAL) || (a.mode != MODE_ROWS && a.flags[0])) return;   // uniform, as in the segmented sum
    const int lane = threadIdx.x & 63, split = threadIdx.x >> 6;
    const int64_t pe = (int64_t) blockIdx.y * 64 + lane;          // slot in the partial row
    // which column does slot pe hold?
    const int pair = a.E >= 2 ? 2 : 1, halves = a.E >= 2 ? a.E / 2 : 1;
    const int64_t idx2 = pe / pair;
    const int l = (int) (idx2 % a.G);
    const int64_t t = idx2 / a.G;
    const int64_t sc = t / halves;
    const int64_t piece = (sc / a.C) * a.G * a.C + (sc % a.C) * a.G + l;
    const int64_t col = piece * a.E + (t % halves) * pair + pe % pair;
    const bool live = pe < a.pstride && piece < a.pieces;

    const uint32_t n_long = a.counters[0], n_short = a.counters[1];
    for (uint32_t i = blockIdx.x; i < n_long; i += gridDim.x) {
        const uint4 rec = a.span_long[i];
        const PartList pl(rec.y, rec.z, (uint32_t) a.tiles_per_block);
        double acc = 0.0;
        if (live) {
            uint32_t q = split;
            for (; q + (PX_FIXUP_DEPTH - 1) * FIX_SPLITS < pl.parts; q += PX_FIXUP_DEPTH * FIX_SPLITS) {
                double v[PX_FIXUP_DEPTH];
#pragma unroll
                for (int j = 0; j < PX_FIXUP_DEPTH; ++j) v[j] = pl.row(q + j * FIX_SPLITS, a.pfirst, a.plast, a.pstride)[pe];
#pragma unroll
                for (int j = 0; j < PX_FIXUP_DEPTH; ++j) acc += v[j];
            }
            {
                // fewer than a full batch is left for this wave: request them together, add them in order
                double v[PX_FIXUP_DEPTH - 1];
#pragma unroll
                for (int j = 0; j < PX_FIXUP_DEPTH - 1; ++j)
                    v[j] = q + j * FIX_SPLITS < pl.parts ? pl.row(q + j * FIX_SPLITS, a.pfirst, a.plast, a.pstride)[pe] : 0.0;
#pragma unroll
                for (int j = 0; j < PX_FIXUP_DEPTH - 1; ++j)
                    if (q + j * FIX_SPLITS < pl.parts) acc += v[j];
            }
        }
        s_red[split][lane] = acc;
        __syncthreads();
        if (split == 0 && live) {
            double tsum = 0.0;
#pragma unroll
            for (int w = 0; w < FIX_SPLITS; ++w) tsum += s_red[w][lane];
            fixup_finish(a, rec.x, col, tsum);
        }
        __syncthreads();
    }
    // the short spans are dealt out from the far end of the grid: the workgroups that had a long
    // run to add up get theirs last
    for (uint32_t i = (gridDim.x - 1u - blockIdx.x) * FIX_SPLITS + split; i < n_short; i += gridDim.x * FIX_SPLITS) {
        const uint4 rec = a.span_short[i];
        const PartList pl(rec.y, rec.z, (uint32_t) a.tiles_per_block);
        if (live) {
            double acc = 0.0;
            uint32_t q = 0;
            for (; q + 7 < pl.parts; q += 8) {
                double v[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) v[j] = pl.row(q + j, a.pfirst, a.plast, a.pstride)[pe];
#pragma unroll
                for (int j = 0; j < 8; ++j) acc += v[j];
            }
            if (q + 3 < pl.parts) {
                double v[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) v[j] = pl.row(q + j, a.pfirst, a.plast, a.pstride)[pe];
#pragma unroll
                for (int j = 0; j < 4; ++j) acc += v[j];
                q += 4;
            }
            {
                // at most three parts are left: request them together, add them in order
                double v[3];
#pragma unroll
                for (int j = 0; j < 3; ++j) v[j] = q + j < pl.parts ? pl.row(q + j, a.pfirst, a.plast, a.pstride)[pe] : 0.0;
#pragma unroll
                for (int j = 0; j < 3; ++j)
                    if (q + j < pl.parts) acc += v[j];
            }
            fixup_finish(a, rec.x, col, acc);
        }
    }
    if (a.out_run_len != nullptr) {                               // every workgroup of the grid takes its share
        const int64_t n = a.num_unique[0];
        const int64_t stride = (int64_t) gridDim.x * gridDim.y * blockDim.x;
        for (int64_t u = ((int64_t) blockIdx.y * gridDim.x + blockIdx.x) * blockDim.x + threadIdx.x; u < n; u += stride)
            a.out_run_len[u] = (int32_t) (a.run_start[u + 1] - a.run_start[u]);
    }
}

int bits_for(uint64_t max_value) {   // bits needed to write max_value
    int b = 0;
    while (max_value) {
        ++b;
        max_value >>= 1;
    }
    return b;
}

// Rows in flight per lane group.  The fused modes also hold the table (and accumulator) pieces of
// every row of a batch that may finish a run, so their batches shrink as rows get wider.
constexpr int batch_rows(int mode, int c, int state_vectors) {
    if (mode == MODE_ROWS) return c == 1 ? PX_SEG_ROWS : c == 2 ? PX_SEG_ROWS_2 : PX_SEG_ROWS_WIDE;
    const int per_row = c * state_vectors * (mode == MODE_ADAGRAD ? 2 : 1);
    return per_row >= PX_FUSED_STATE_PIECES ? 1 : PX_FUSED_STATE_PIECES / per_row;
}

template <typename T, bool VEC, int MODE>
void launch_segsum(const SegsumArgs& a, const RowShape& sh, hipStream_t stream) {
    constexpr int SV = VEC ? RowLoad<T, VEC>::E / 4 : 1;
    const dim3 grid((unsigned) ((a.n_tiles + (256 / sh.G) - 1) / (256 / sh.G)), (unsigned) sh.slabs, 1);
    // batch depth of a stretch with tails, and of a stretch without heads (never holds table pieces)
#define PX_SEG_LAUNCH(G_, C_) \
    k_segsum<T, VEC, G_, C_, batch_rows(MODE, C_, SV), batch_rows(MODE_ROWS, C_, SV), MODE><<<grid, 256, 0, stream>>>(a)
    if (sh.G == 16) PX_SEG_LAUNCH(16, 1);
    else if (sh.G == 32) PX_SEG_LAUNCH(32, 1);
    else if (sh.C == 1) PX_SEG_LAUNCH(64, 1);
    else if (sh.C == 2) PX_SEG_LAUNCH(64, 2);
    else PX_SEG_LAUNCH(64, 4);
#undef PX_SEG_LAUNCH
}

template <int MODE>
void launch_segsum_mode(const SegsumArgs& a, const RowShape& sh, bool vec, px_dtype val_dtype, hipStream_t stream) {
    if (vec) {
        if (val_dtype == PX_F32) launch_segsum<float, true, MODE>(a, sh, stream);
        else launch_segsum<uint16_t, true, MODE>(a, sh, stream);
    } else {
        if (val_dtype == PX_F32) launch_segsum<float, false, MODE>(a, sh, stream);
        else launch_segsum<uint16_t, false, MODE>(a, sh, stream);
    }
}

}  // namespace

extern "C" size_t px_coalesce_scratch_bytes(int64_t total_rows, int64_t dim) {
    if (total_rows < 0 || dim < 1) return 0;
    if (total_rows == 0) return 256;
    return carve(nullptr, total_rows, dim).bytes;
}

static px_status coalesce_common(px_ctx* ctx, int mode, int n_workers, const int64_t* const* idx,
                                 const void* const* val, const int64_t* counts, int64_t dim,
                                 px_dtype val_dtype, int64_t vocab, float scale, int64_t* out_ids,
                                 float* out_rows, float* table, float* accum, float lr, float eps,
                                 int64_t* out_num_unique, int32_t* out_run_len, void* scratch,
                                 size_t scratch_bytes, void* hip_stream) {
    if (!ctx) return PX_ERR_INVALID_ARG;
    hipStream_t stream = (hipStream_t) hip_stream;
    if (n_workers < 1 || n_workers > PX_MAX_SOURCES)
        return px_fail(ctx, PX_ERR_INVALID_ARG, "n_workers %d outside [1, %d]", n_workers, (int) PX_MAX_SOURCES);
    if (!idx || !val || !counts || !out_num_unique)
        return px_fail(ctx, PX_ERR_INVALID_ARG, "null argument");
    if (dim < 1 || vocab < 1 || vocab > (1ll << 32))
        return px_fail(ctx, PX_ERR_INVALID_ARG, "dim %lld or vocab %lld unsupported", (long long) dim, (long long) vocab);
    if (val_dtype != PX_F32 && val_dtype != PX_BF16)
        return px_fail(ctx, PX_ERR_INVALID_ARG, "value dtype %d unknown", (int) val_dtype);
    const size_t es = val_dtype == PX_F32 ? 4 : 2;
    int64_t m = 0, max_count = 0;
    bool vec = (((size_t) dim * es) % 16) == 0;
    uint64_t host_words[3 * PX_MAX_SOURCES + 1];
    for (int w = 0; w < n_workers; ++w) {
        if (counts[w] < 0) return px_fail(ctx, PX_ERR_INVALID_ARG, "counts[%d] negative", w);
        if (counts[w] > 0 && (!idx[w] || !val[w]))
            return px_fail(ctx, PX_ERR_INVALID_ARG, "worker %d has rows but a null pointer", w);
        if (((uintptr_t) val[w]) % es || ((uintptr_t) idx[w]) % 8)
            return px_fail(ctx, PX_ERR_INVALID_ARG, "worker %d pointers misaligned", w);
        if (((uintptr_t) val[w]) % 16) vec = false;
        if (counts[w] > max_count) max_count = counts[w];
        m += counts[w];
        if (m >= (1ll << 31)) return px_fail(ctx, PX_ERR_INVALID_ARG, "more than 2^31-1 input rows");
    }
    if (m == 0) {
        k_write_zero_count<<<1, 64, 0, stream>>>(out_num_unique);
        return px_check_hip(ctx, hipGetLastError(), "launch");
    }
    if (!out_ids || !scratch) return px_fail(ctx, PX_ERR_INVALID_ARG, "null output or scratch");
    if (((uintptr_t) scratch) % 256) return px_fail(ctx, PX_ERR_INVALID_ARG, "scratch needs 256-byte alignment");
    if (mode == MODE_ROWS) {
        if (!out_rows || ((uintptr_t) out_rows) % 16)
            return px_fail(ctx, PX_ERR_INVALID_ARG, "out_rows null or not 16-byte aligned");
    } else {
        if (!table || (mode == MODE_ADAGRAD && !accum)) return px_fail(ctx, PX_ERR_INVALID_ARG, "null table or accumulator");
        if (((uintptr_t) table) % 4 || (accum && ((uintptr_t) accum) % 4))
            return px_fail(ctx, PX_ERR_INVALID_ARG, "float pointers misaligned");
        // the 128-bit path also reads and writes the variable in 16-byte pieces
        if (dim % 4 || ((uintptr_t) table) % 16 || (accum && ((uintptr_t) accum) % 16)) vec = false;
    }
    const int local_bits = bits_for((uint64_t) (max_count - 1));
    if (bits_for((uint64_t) (n_workers - 1)) + local_bits > 32)
        return px_fail(ctx, PX_ERR_INVALID_ARG, "bits(n_workers-1) + bits(max count-1) exceeds 32");
    const Scratch sc = carve(scratch, m, dim);
    if (scratch_bytes < sc.bytes)
        return px_fail(ctx, PX_ERR_SCRATCH_TOO_SMALL, "scratch %zu < %zu bytes", scratch_bytes, sc.bytes);

    // Pointer and offset tables travel to the device inside kernel arguments.
    int64_t run = 0;
    for (int w = 0; w < n_workers; ++w) {
        host_words[w] = (uint64_t) (uintptr_t) idx[w];
        host_words[n_workers + w] = (uint64_t) (uintptr_t) val[w];
        host_words[2 * n_workers + w] = (uint64_t) run;
        run += counts[w];
    }
    host_words[3 * n_workers] = (uint64_t) run;
    const px_sort_geom g = px_sort_geometry(m);
    // Digits of up to PX_RADIX_MAX_BITS bits: as few passes as that allows, all of the same width
    // (at least 8 bits).
    // Wide digits only while a pass is bound by its launches (few blocks): at 512 blocks the 2,048-bin
    // histogram matrix makes a pass cost twice an 8-bit one.
    const int key_bits = bits_for((uint64_t) (vocab - 1));
    const int widest = g.n_blocks <= PX_WIDE_DIGIT_BLOCKS ? PX_RADIX_MAX_BITS : 8;
    int passes = (key_bits + widest - 1) / widest;
    if (passes < 1) passes = 1;
    int digit_bits = (key_bits + passes - 1) / passes;
    if (digit_bits < 8) digit_bits = 8;
    uint64_t* sorted_words = nullptr;
    uint64_t* other_words = nullptr;
    px_status sort_status = PX_OK;
    auto sort = [&](auto bits_tag) {
        constexpr int BITS = decltype(bits_tag)::value;
        if (3 * n_workers + 1 <= PX_UPLOAD_WORDS) {
            // up to 85 workers: the tables ride in the pack kernel's own arguments
            px_word_pack pack;
            memcpy(pack.w, host_words, (size_t) (3 * n_workers + 1) * sizeof(uint64_t));
            k_pack<true, BITS><<<g.n_blocks, PX_SORT_THREADS, 0, stream>>>(ctx->d_words, pack, sc.counters, 64, n_workers, m,
                                                                           vocab, local_bits, sc.keys_a, sc.hist, g.chunk,
                                                                           ctx->d_flags, sc.hcount);
        } else {
            sort_status = px_upload_words(ctx, ctx->d_words, host_words, 3 * n_workers + 1, sc.counters, 64, stream);
            if (sort_status != PX_OK) return;
            px_word_pack unused;
            unused.w[0] = 0;
            k_pack<false, BITS><<<g.n_blocks, PX_SORT_THREADS, 0, stream>>>(ctx->d_words, unused, sc.counters, 64, n_workers, m,
                                                                            vocab, local_bits, sc.keys_a, sc.hist, g.chunk,
                                                                            ctx->d_flags, sc.hcount);
        }
        uint64_t* src = sc.keys_a;
        uint64_t* dst = sc.keys_b;
        for (int p = 0; p < passes; ++p) {
            SortWords pol{src, dst, m, BITS * p, (uint32_t) ((1 << BITS) - 1)};
            if (p > 0) pxr::k_radix_hist<SortWords, BITS><<<g.n_blocks, PX_SORT_THREADS, 0, stream>>>(pol, sc.hist, g.chunk);
            const int own = g.n_blocks <= PX_OWN_PREFIX_BLOCKS ? g.n_blocks : 0;
            if (!own) pxr::k_radix_prefix<<<(1 << BITS) / 4, 256, 0, stream>>>(sc.hist, g.n_blocks, 1 << BITS, sc.totals);
            pxr::k_radix_scatter<SortWords, BITS><<<g.n_blocks, PX_SORT_THREADS, 0, stream>>>(pol, sc.hist, sc.totals, g.chunk, own, 0);
            uint64_t* t = src;
            src = dst;
            dst = t;
        }
        sorted_words = src;
        other_words = dst;
    };
    if (digit_bits <= 8) sort(std::integral_constant<int, 8>());
    else if (digit_bits == 9) sort(std::integral_constant<int, 9>());
    else if (digit_bits == 10) sort(std::integral_constant<int, 10>());
    else sort(std::integral_constant<int, 11>());
    if (sort_status != PX_OK) return sort_status;
    uint64_t* dst = other_words;
    const uint64_t* sorted = sorted_words;

    const int tile_rows = tile_rows_for(m, mode != MODE_ROWS);
    const int64_t n_tiles = (m + tile_rows - 1) / tile_rows;
    const int n_hblocks = (int) ((m + PX_SORT_TILE - 1) / PX_SORT_TILE);
    uint64_t* rowref = dst;               // the sort's other buffer is free now
    k_heads_emit<<<n_hblocks, 256, 0, stream>>>(sorted, m, sc.hcount, tile_rows, ctx->d_words, n_workers, local_bits,
                                                dim * (int64_t) es, rowref, out_ids, sc.run_start, sc.tile_info,
                                                out_num_unique, ctx->d_flags, ctx->wait_polls);

    const RowShape sh = row_shape(dim, (int) es, vec);
    SegsumArgs a;
    a.rowref = rowref;
    a.sorted = sorted;
    a.tile_info = sc.tile_info;
    a.run_start = sc.run_start;
    a.pfirst = sc.pfirst;
    a.plast = sc.plast;
    a.span_long = sc.span_long;
    a.span_short = sc.span_short;
    a.counters = sc.counters;
    a.out_rows = out_rows;
    a.m = m;
    a.n_tiles = n_tiles;
    a.dim = dim;
    a.pstride = sh.pstride;
    a.tile_rows = tile_rows;
    a.pieces = sh.pieces;
    a.scale = scale;
    a.table = table;
    a.accum = accum;
    a.flags = ctx->d_flags;
    a.lr = lr;
    a.eps = eps;
    if (mode == MODE_ROWS) launch_segsum_mode<MODE_ROWS>(a, sh, vec, val_dtype, stream);
    else if (mode == MODE_SGD) launch_segsum_mode<MODE_SGD>(a, sh, vec, val_dtype, stream);
    else launch_segsum_mode<MODE_ADAGRAD>(a, sh, vec, val_dtype, stream);
    FixupArgs f;
    f.mode = mode;
    f.table = table;
    f.accum = accum;
    f.out_ids = out_ids;
    f.flags = ctx->d_flags;
    f.lr = lr;
    f.eps = eps;
    f.span_long = sc.span_long;
    f.span_short = sc.span_short;
    f.counters = sc.counters;
    f.run_start = sc.run_start;
    f.pfirst = sc.pfirst;
    f.plast = sc.plast;
    f.out_rows = out_rows;
    f.out_run_len = out_run_len;
    f.num_unique = out_num_unique;
    f.dim = dim;
    f.pstride = sh.pstride;
    f.tiles_per_block = (sh.C * sh.E <= 16) ? 256 / sh.G : 0;      // the segsum kernel's MERGE rule
    f.G = sh.G;
    f.C = sh.C;
    f.E = sh.E;
    f.pieces = sh.pieces;
    f.scale = scale;
    // 1,024-thread workgroups: the grid stays at one per compute unit, so that all of them are resident
    // at once (a second round of workgroups would only start after the first one's long runs)
    const unsigned fy = (unsigned) ((sh.pstride + 63) / 64);
    unsigned fx = PX_FIXUP_RESIDENT / fy;
    if (fx > 64u) fx = 64u;
    if (fx < 8u) fx = 8u;
    if ((int64_t) fx > n_tiles) fx = (unsigned) n_tiles;
    k_fixup<<<dim3(fx, fy, 1), 64 * FIX_SPLITS, 0, stream>>>(f);
    return px_check_hip(ctx, hipGetLastError(), "coalesce launch");
}

extern "C" px_status px_sparse_coalesce(px_ctx* ctx, int n_workers, const int64_t* const* idx,
                                        const void* const* val, const int64_t* counts, int64_t dim,
                                        px_dtype val_dtype, int64_t vocab, float scale,
                                        int64_t* out_ids, float* out_rows, int64_t* out_num_unique,
                                        int32_t* out_run_len, void* scratch, size_t scratch_bytes,
                                        void* hip_stream) {
    return coalesce_common(ctx, MODE_ROWS, n_workers, idx, val, counts, dim, val_dtype, vocab, scale, out_ids,
                           out_rows, nullptr, nullptr, 0.f, 0.f, out_num_unique, out_run_len, scratch,
                           scratch_bytes, hip_stream);
}

extern "C" px_status px_sparse_coalesce_apply_sgd(px_ctx* ctx, int n_workers, const int64_t* const* idx,
                                                  const void* const* val, const int64_t* counts, int64_t dim,
                                                  px_dtype val_dtype, int64_t vocab, float scale, float* table,
                                                  float lr, int64_t* out_ids, int64_t* out_num_unique,
                                                  int32_t* out_run_len, void* scratch, size_t scratch_bytes,
                                                  void* hip_stream) {
    return coalesce_common(ctx, MODE_SGD, n_workers, idx, val, counts, dim, val_dtype, vocab, scale, out_ids,
                           nullptr, table, nullptr, lr, 0.f, out_num_unique, out_run_len, scratch, scratch_bytes,
                           hip_stream);
}

extern "C" px_status px_sparse_coalesce_apply_adagrad(px_ctx* ctx, int n_workers, const int64_t* const* idx,
                                                      const void* const* val, const int64_t* counts,
                                                      int64_t dim, px_dtype val_dtype, int64_t vocab,
                                                      float scale, float* table, float* accum, float lr,
                                                      float eps, int64_t* out_ids, int64_t* out_num_unique,
                                                      int32_t* out_run_len, void* scratch, size_t scratch_bytes,
                                                      void* hip_stream) {
    return coalesce_common(ctx, MODE_ADAGRAD, n_workers, idx, val, counts, dim, val_dtype, vocab, scale, out_ids,
                           nullptr, table, accum, lr, eps, out_num_unique, out_run_len, scratch, scratch_bytes,
                           hip_stream);
}
