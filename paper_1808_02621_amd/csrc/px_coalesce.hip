// px_sparse_coalesce: aggregate N workers' sparse gradients of one variable.
//
// Parallax Fig. 3 / Sec. 3.2: the workers' (indices, values) arrays are
// concatenated and values carrying the same index are accumulated.  On the GPU:
//   1. pack    every input row becomes one 64-bit word  id << 32 | worker << LB | local row
//   2. sort    stable least-significant-digit radix sort of the words on the id bits only
//              (ceil(log2 vocab) bits, 8 per pass); value rows never move
//   3. heads   a row is a run head if its id differs from its predecessor's; counting and
//              ranking the heads yields U, the distinct ids and every run's start
//   4. segsum  the sorted order is cut into fixed tiles of rows; a lane group walks its tile,
//              gathers each value row with 128-bit loads and accumulates in double.  Runs
//              inside one tile are written out at once; a run that crosses a tile border
//              leaves one double-precision partial row per tile
//   5. fixup   each border-crossing run adds up its partial rows, rounds once, writes its row
// Nothing waits on another workgroup and global atomics only append to the list of
// border-crossing runs, so the sums are deterministic.
#include "px_radix.h"

namespace {

// ------------------------------------------------------------------ geometry

// Rows per segsum tile: enough tiles to fill the chip, few enough partial rows.
inline int tile_rows_for(int64_t m) {
    int64_t t = (m + 8191) / 8192;
    t = (t + 7) / 8 * 8;
    if (t < 32) t = 32;
    if (t > 256) t = 256;
    return (int) t;
}

struct Scratch {
    uint64_t* keys_a;
    uint64_t* keys_b;
    uint32_t* hist;        // [PX_SORT_MAX_BLOCKS][256]
    uint32_t* hcount;      // heads per 2048-row block
    uint32_t* run_start;   // [M + 1]
    uint32_t* tile_u0;     // run index of each tile's first row
    uint32_t* span_list;   // runs that cross a tile border
    uint32_t* counters;    // [0] = length of span_list
    double* pfirst;        // [n_tiles][dim] partial of the run entering a tile
    double* plast;         // [n_tiles][dim] partial of the run leaving a tile
    size_t bytes;
};

inline Scratch carve(void* base, int64_t m, int64_t dim) {
    Scratch s;
    const int t = tile_rows_for(m);
    const size_t n_tiles = (size_t) ((m + t - 1) / t);
    const size_t n_hblocks = (size_t) ((m + PX_SORT_TILE - 1) / PX_SORT_TILE);
    size_t off = 0;
    char* b = (char*) base;
    auto take = [&](size_t bytes) {
        char* p = b + off;
        off += px_align_up(bytes, 256);
        return p;
    };
    s.keys_a = (uint64_t*) take((size_t) m * 8);
    s.keys_b = (uint64_t*) take((size_t) m * 8);
    s.hist = (uint32_t*) take((size_t) PX_SORT_MAX_BLOCKS * PX_RADIX * 4);
    s.hcount = (uint32_t*) take((n_hblocks + 1) * 4);
    s.run_start = (uint32_t*) take(((size_t) m + 1) * 4);
    s.tile_u0 = (uint32_t*) take((n_tiles + 1) * 4);
    s.span_list = (uint32_t*) take((n_tiles + 1) * 4);
    s.counters = (uint32_t*) take(64 * 4);
    s.pfirst = (double*) take(n_tiles * (size_t) dim * 8);
    s.plast = (double*) take(n_tiles * (size_t) dim * 8);
    s.bytes = off;
    return s;
}

__device__ __forceinline__ uint32_t key_of(uint64_t w) { return (uint32_t) (w >> 32); }

// ---------------------------------------------------------------------- pack

__global__ __launch_bounds__(PX_SORT_THREADS) void k_pack(const uint64_t* __restrict__ words,
                                                          int n_workers, int64_t m, int64_t vocab,
                                                          int local_bits, uint64_t* __restrict__ keys,
                                                          uint32_t* __restrict__ hist, int64_t chunk,
                                                          uint32_t* __restrict__ flags) {
    __shared__ uint32_t s_prefix[PX_MAX_SOURCES + 1];
    __shared__ uint32_t s_hist[PX_RADIX];
    const int tid = threadIdx.x;
    for (int i = tid; i <= n_workers; i += PX_SORT_THREADS) s_prefix[i] = (uint32_t) words[PXW_PREFIX + i];
    s_hist[tid] = 0u;
    __syncthreads();
    const int64_t* const* idx = (const int64_t* const*) (words + PXW_IDX_PTR);
    const int64_t begin = (int64_t) blockIdx.x * chunk;
    int64_t end = begin + chunk;
    if (end > m) end = m;
    for (int64_t p = begin + tid; p < end; p += PX_SORT_THREADS) {
        int lo = 0, hi = n_workers;                 // s_prefix[lo] <= p < s_prefix[hi]
        while (hi - lo > 1) {
            int mid = (lo + hi) >> 1;
            if ((int64_t) s_prefix[mid] <= p) lo = mid; else hi = mid;
        }
        const uint32_t local = (uint32_t) (p - (int64_t) s_prefix[lo]);
        int64_t id = idx[lo][local];
        if (id < 0 || id >= vocab) {
            atomicOr(flags, (uint32_t) PXF_BAD_ID);
            id = 0;
        }
        keys[p] = ((uint64_t) (uint32_t) id << 32) | (uint64_t) (((uint32_t) lo << local_bits) | local);
        atomicAdd(&s_hist[(uint32_t) id & 255u], 1u);
    }
    __syncthreads();
    hist[(size_t) blockIdx.x * PX_RADIX + tid] = s_hist[tid];
}

struct SortWords {
    typedef uint64_t Item;
    const uint64_t* in;
    uint64_t* out;
    int64_t n;
    int shift;                                      // bit offset inside the id
    __device__ int64_t count() const { return n; }
    __device__ Item load(int64_t i) const { return in[i]; }
    __device__ uint32_t digit(Item v, int64_t) const { return (uint32_t) (v >> (32 + shift)) & 255u; }
    __device__ void note(int64_t, uint32_t) const {}
    __device__ void store(uint32_t dst, Item v) const { out[dst] = v; }
};

// --------------------------------------------------------------------- heads

__global__ __launch_bounds__(256) void k_heads_count(const uint64_t* __restrict__ sorted, int64_t m,
                                                     uint32_t* __restrict__ hcount) {
    __shared__ uint32_t s_cnt;
    if (threadIdx.x == 0) s_cnt = 0u;
    __syncthreads();
    const int64_t base = (int64_t) blockIdx.x * PX_SORT_TILE;
    uint32_t c = 0;
#pragma unroll
    for (int j = 0; j < PX_SORT_ITEMS; ++j) {
        const int64_t i = base + j * 256 + threadIdx.x;
        if (i < m) c += (i == 0 || key_of(sorted[i]) != key_of(sorted[i - 1])) ? 1u : 0u;
    }
    for (int o = 32; o > 0; o >>= 1) c += __shfl_down(c, o);
    if (pxr::lane_id() == 0) atomicAdd(&s_cnt, c);
    __syncthreads();
    if (threadIdx.x == 0) hcount[blockIdx.x] = s_cnt;
}

__global__ __launch_bounds__(256) void k_heads_emit(const uint64_t* __restrict__ sorted, int64_t m,
                                                    const uint32_t* __restrict__ hcount, int tile_rows,
                                                    int64_t* __restrict__ out_ids,
                                                    uint32_t* __restrict__ run_start,
                                                    uint32_t* __restrict__ tile_u0,
                                                    int64_t* __restrict__ out_num_unique,
                                                    const uint32_t* __restrict__ flags) {
    __shared__ uint32_t s_wave[4];
    const int tid = threadIdx.x;
    // heads in all blocks before this one
    uint32_t part = 0;
    for (int b = tid; b < (int) blockIdx.x; b += 256) part += hcount[b];
    uint32_t before;
    pxr::block_exclusive_scan_256(part, s_wave, &before);

    const int64_t base = (int64_t) blockIdx.x * PX_SORT_TILE + (int64_t) tid * PX_SORT_ITEMS;
    uint32_t keys[PX_SORT_ITEMS];
    uint32_t flag[PX_SORT_ITEMS];
    uint32_t prev = 0;
    if (base > 0 && base - 1 < m) prev = key_of(sorted[base - 1]);
    uint32_t cnt = 0;
#pragma unroll
    for (int j = 0; j < PX_SORT_ITEMS; ++j) {
        const int64_t i = base + j;
        keys[j] = 0;
        flag[j] = 0;
        if (i < m) {
            keys[j] = key_of(sorted[i]);
            flag[j] = (i == 0 || keys[j] != prev) ? 1u : 0u;
            prev = keys[j];
        }
        cnt += flag[j];
    }
    uint32_t block_total;
    uint32_t rank = before + pxr::block_exclusive_scan_256(cnt, s_wave, &block_total);
#pragma unroll
    for (int j = 0; j < PX_SORT_ITEMS; ++j) {
        const int64_t i = base + j;
        if (i < m) {
            if (flag[j]) {
                out_ids[rank] = (int64_t) keys[j];
                run_start[rank] = (uint32_t) i;
                ++rank;
            }
            if ((uint32_t) i % (uint32_t) tile_rows == 0u)
                tile_u0[(uint32_t) i / (uint32_t) tile_rows] = rank - 1u;   // run that row i belongs to
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

template <typename T, bool VEC> struct RowLoad;

template <> struct RowLoad<float, true> {
    typedef uint4 Raw;
    enum { E = 4 };
    static __device__ __forceinline__ Raw load(const char* p) { return *(const uint4*) p; }
    static __device__ __forceinline__ void add(double* acc, const Raw& r) {
        acc[0] += (double) __uint_as_float(r.x);
        acc[1] += (double) __uint_as_float(r.y);
        acc[2] += (double) __uint_as_float(r.z);
        acc[3] += (double) __uint_as_float(r.w);
    }
};
template <> struct RowLoad<float, false> {
    typedef float Raw;
    enum { E = 1 };
    static __device__ __forceinline__ Raw load(const char* p) { return *(const float*) p; }
    static __device__ __forceinline__ void add(double* acc, const Raw& r) { acc[0] += (double) r; }
};
// bfloat16 is the upper half of a float32: widening is a shift.
template <> struct RowLoad<uint16_t, true> {
    typedef uint4 Raw;
    enum { E = 8 };
    static __device__ __forceinline__ Raw load(const char* p) { return *(const uint4*) p; }
    static __device__ __forceinline__ void add(double* acc, const Raw& r) {
        acc[0] += (double) __uint_as_float(r.x << 16);
        acc[1] += (double) __uint_as_float(r.x & 0xffff0000u);
        acc[2] += (double) __uint_as_float(r.y << 16);
        acc[3] += (double) __uint_as_float(r.y & 0xffff0000u);
        acc[4] += (double) __uint_as_float(r.z << 16);
        acc[5] += (double) __uint_as_float(r.z & 0xffff0000u);
        acc[6] += (double) __uint_as_float(r.w << 16);
        acc[7] += (double) __uint_as_float(r.w & 0xffff0000u);
    }
};
template <> struct RowLoad<uint16_t, false> {
    typedef uint16_t Raw;
    enum { E = 1 };
    static __device__ __forceinline__ Raw load(const char* p) { return *(const uint16_t*) p; }
    static __device__ __forceinline__ void add(double* acc, const Raw& r) {
        acc[0] += (double) __uint_as_float((uint32_t) r << 16);
    }
};

struct SegsumArgs {
    const uint64_t* sorted;       // packed words in id order
    const uint64_t* words;        // context table: value base pointers
    const uint32_t* tile_u0;
    double* pfirst;
    double* plast;
    uint32_t* span_list;
    uint32_t* span_count;
    float* out_rows;
    int64_t m;
    int64_t dim;                  // elements per row
    int64_t row_bytes;            // bytes per input row
    int n_workers;
    int local_bits;
    int tile_rows;
    int pieces;                   // row pieces (E elements each) per row
    float scale;
};

// G lanes walk one tile; lane l owns pieces slab*G*C + c*G + l, c < C, E elements each.
// B rows are in flight at once.
template <typename T, bool VEC, int G, int C, int B>
__global__ __launch_bounds__(256) void k_segsum(SegsumArgs a) {
    typedef RowLoad<T, VEC> L;
    enum { E = L::E };
    __shared__ uint64_t s_base[PX_MAX_SOURCES];
    for (int i = threadIdx.x; i < a.n_workers; i += 256) s_base[i] = a.words[PXW_VAL_PTR + i];
    __syncthreads();

    const int gl = threadIdx.x % G;
    const int64_t tile = (int64_t) blockIdx.x * (256 / G) + threadIdx.x / G;
    const int64_t s = tile * a.tile_rows;
    if (s >= a.m) return;
    int64_t e = s + a.tile_rows;
    if (e > a.m) e = a.m;

    int piece[C];
    bool live[C];
#pragma unroll
    for (int c = 0; c < C; ++c) {
        piece[c] = (int) blockIdx.y * (G * C) + c * G + gl;
        live[c] = piece[c] < a.pieces;
    }
    const uint32_t local_mask = (a.local_bits >= 32) ? 0xffffffffu : ((1u << a.local_bits) - 1u);

    double acc[C][E];
#pragma unroll
    for (int c = 0; c < C; ++c)
#pragma unroll
        for (int x = 0; x < E; ++x) acc[c][x] = 0.0;

    uint32_t u = a.tile_u0[tile];
    uint32_t cur = key_of(a.sorted[s]);
    bool started = (s == 0) || key_of(a.sorted[s - 1]) != cur;

    auto flush = [&](bool ended) {
        if (started && ended) {
            float* dst = a.out_rows + (size_t) u * a.dim;
#pragma unroll
            for (int c = 0; c < C; ++c)
                if (live[c]) {
                    if (VEC) {
#pragma unroll
                        for (int x = 0; x < E; x += 4) {
                            float4 o = make_float4((float) (acc[c][x] * a.scale), (float) (acc[c][x + 1] * a.scale),
                                                   (float) (acc[c][x + 2] * a.scale), (float) (acc[c][x + 3] * a.scale));
                            *(float4*) (dst + (size_t) piece[c] * E + x) = o;
                        }
                    } else {
#pragma unroll
                        for (int x = 0; x < E; ++x) dst[(size_t) piece[c] * E + x] = (float) (acc[c][x] * a.scale);
                    }
                }
        } else {
            double* dst = (started ? a.plast : a.pfirst) + (size_t) tile * a.dim;
#pragma unroll
            for (int c = 0; c < C; ++c)
                if (live[c]) {
#pragma unroll
                    for (int x = 0; x < E; ++x) dst[(size_t) piece[c] * E + x] = acc[c][x];
                }
            if (started && gl == 0 && blockIdx.y == 0) {
                uint32_t slot = atomicAdd(a.span_count, 1u);
                a.span_list[slot] = u;
            }
        }
#pragma unroll
        for (int c = 0; c < C; ++c)
#pragma unroll
            for (int x = 0; x < E; ++x) acc[c][x] = 0.0;
    };

    for (int64_t r = s; r < e; r += B) {
        uint64_t w[B];
        typename L::Raw raw[B][C];
#pragma unroll
        for (int j = 0; j < B; ++j) w[j] = (r + j < e) ? a.sorted[r + j] : 0ull;
#pragma unroll
        for (int j = 0; j < B; ++j) {
            if (r + j < e) {
                const uint32_t payload = (uint32_t) w[j];
                const uint32_t worker = (a.local_bits >= 32) ? 0u : (payload >> a.local_bits);
                const char* row = (const char*) s_base[worker] + (size_t) (payload & local_mask) * a.row_bytes;
#pragma unroll
                for (int c = 0; c < C; ++c)
                    if (live[c]) raw[j][c] = L::load(row + (size_t) piece[c] * (E * sizeof(T)));
            }
        }
#pragma unroll
        for (int j = 0; j < B; ++j) {
            if (r + j < e) {
                const uint32_t k = key_of(w[j]);
                if (k != cur) {
                    flush(true);
                    ++u;
                    cur = k;
                    started = true;
                }
#pragma unroll
                for (int c = 0; c < C; ++c)
                    if (live[c]) L::add(acc[c], raw[j][c]);
            }
        }
    }
    const bool ended = (e == a.m) || key_of(a.sorted[e]) != cur;
    flush(ended);
}

// -------------------------------------------------------------------- fix-up

__global__ __launch_bounds__(256) void k_fixup(const uint32_t* __restrict__ span_list,
                                               const uint32_t* __restrict__ span_count,
                                               const uint32_t* __restrict__ run_start, int tile_rows,
                                               int64_t dim, const double* __restrict__ pfirst,
                                               const double* __restrict__ plast, float* __restrict__ out_rows,
                                               float scale, int32_t* __restrict__ out_run_len,
                                               const int64_t* __restrict__ num_unique) {
    __shared__ double s_red[4][64];
    const int lane = threadIdx.x & 63, split = threadIdx.x >> 6;
    const int64_t col = (int64_t) blockIdx.y * 64 + lane;
    const uint32_t count = span_count[0];
    for (uint32_t i = blockIdx.x; i < count; i += gridDim.x) {
        const uint32_t u = span_list[i];
        const uint32_t first_tile = run_start[u] / (uint32_t) tile_rows;
        const uint32_t last_tile = (run_start[u + 1] - 1u) / (uint32_t) tile_rows;
        const uint32_t parts = last_tile - first_tile + 1u;
        double acc = 0.0;
        if (col < dim) {
#pragma unroll 4
            for (uint32_t q = split; q < parts; q += 4) {
                const double* src = (q == 0) ? plast + (size_t) first_tile * dim
                                             : pfirst + (size_t) (first_tile + q) * dim;
                acc += src[col];
            }
        }
        s_red[split][lane] = acc;
        __syncthreads();
        if (split == 0 && col < dim) {
            const double t = ((s_red[0][lane] + s_red[1][lane]) + s_red[2][lane]) + s_red[3][lane];
            out_rows[(size_t) u * dim + col] = (float) (t * scale);
        }
        __syncthreads();
    }
    if (out_run_len != nullptr && blockIdx.y == 0) {
        const int64_t n = num_unique[0];
        for (int64_t u = (int64_t) blockIdx.x * 256 + threadIdx.x; u < n; u += (int64_t) gridDim.x * 256)
            out_run_len[u] = (int32_t) (run_start[u + 1] - run_start[u]);
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

template <typename T, bool VEC>
void launch_segsum(const SegsumArgs& a, int64_t n_tiles, hipStream_t stream) {
    const int pieces = a.pieces;
    auto grid = [&](int g, int c) {
        return dim3((unsigned) ((n_tiles + (256 / g) - 1) / (256 / g)), (unsigned) ((pieces + g * c - 1) / (g * c)), 1);
    };
    if (pieces <= 16) k_segsum<T, VEC, 16, 1, 8><<<grid(16, 1), 256, 0, stream>>>(a);
    else if (pieces <= 32) k_segsum<T, VEC, 32, 1, 8><<<grid(32, 1), 256, 0, stream>>>(a);
    else if (pieces <= 64) k_segsum<T, VEC, 64, 1, 8><<<grid(64, 1), 256, 0, stream>>>(a);
    else if (pieces <= 128) k_segsum<T, VEC, 64, 2, 8><<<grid(64, 2), 256, 0, stream>>>(a);
    else k_segsum<T, VEC, 64, 4, 4><<<grid(64, 4), 256, 0, stream>>>(a);
}

}  // namespace

extern "C" size_t px_coalesce_scratch_bytes(int64_t total_rows, int64_t dim) {
    if (total_rows < 0 || dim < 1) return 0;
    if (total_rows == 0) return 256;
    return carve(nullptr, total_rows, dim).bytes;
}

extern "C" px_status px_sparse_coalesce(px_ctx* ctx, int n_workers, const int64_t* const* idx,
                                        const void* const* val, const int64_t* counts, int64_t dim,
                                        px_dtype val_dtype, int64_t vocab, float scale,
                                        int64_t* out_ids, float* out_rows, int64_t* out_num_unique,
                                        int32_t* out_run_len, void* scratch, size_t scratch_bytes,
                                        void* hip_stream) {
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
    if (!out_ids || !out_rows || !scratch) return px_fail(ctx, PX_ERR_INVALID_ARG, "null output or scratch");
    if (((uintptr_t) scratch) % 256 || ((uintptr_t) out_rows) % 16)
        return px_fail(ctx, PX_ERR_INVALID_ARG, "scratch needs 256-byte and out_rows 16-byte alignment");
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
    px_status st;
    st = px_upload_words(ctx, ctx->d_words + PXW_IDX_PTR, host_words, n_workers, sc.counters, 64, stream);
    if (st != PX_OK) return st;
    st = px_upload_words(ctx, ctx->d_words + PXW_VAL_PTR, host_words + n_workers, n_workers, nullptr, 0, stream);
    if (st != PX_OK) return st;
    st = px_upload_words(ctx, ctx->d_words + PXW_PREFIX, host_words + 2 * n_workers, n_workers + 1, nullptr, 0, stream);
    if (st != PX_OK) return st;

    const px_sort_geom g = px_sort_geometry(m);
    k_pack<<<g.n_blocks, PX_SORT_THREADS, 0, stream>>>(ctx->d_words, n_workers, m, vocab, local_bits,
                                                       sc.keys_a, sc.hist, g.chunk, ctx->d_flags);
    int key_bits = bits_for((uint64_t) (vocab - 1));
    int passes = (key_bits + 7) / 8;
    if (passes < 1) passes = 1;
    uint64_t* src = sc.keys_a;
    uint64_t* dst = sc.keys_b;
    for (int p = 0; p < passes; ++p) {
        SortWords pol{src, dst, m, 8 * p};
        if (p > 0) pxr::k_radix_hist<SortWords><<<g.n_blocks, PX_SORT_THREADS, 0, stream>>>(pol, sc.hist, g.chunk);
        pxr::k_radix_scatter<SortWords><<<g.n_blocks, PX_SORT_THREADS, 0, stream>>>(pol, sc.hist, g.n_blocks, g.chunk);
        uint64_t* t = src;
        src = dst;
        dst = t;
    }
    const uint64_t* sorted = src;

    const int tile_rows = tile_rows_for(m);
    const int64_t n_tiles = (m + tile_rows - 1) / tile_rows;
    const int n_hblocks = (int) ((m + PX_SORT_TILE - 1) / PX_SORT_TILE);
    k_heads_count<<<n_hblocks, 256, 0, stream>>>(sorted, m, sc.hcount);
    k_heads_emit<<<n_hblocks, 256, 0, stream>>>(sorted, m, sc.hcount, tile_rows, out_ids, sc.run_start,
                                                sc.tile_u0, out_num_unique, ctx->d_flags);

    SegsumArgs a;
    a.sorted = sorted;
    a.words = ctx->d_words;
    a.tile_u0 = sc.tile_u0;
    a.pfirst = sc.pfirst;
    a.plast = sc.plast;
    a.span_list = sc.span_list;
    a.span_count = sc.counters;
    a.out_rows = out_rows;
    a.m = m;
    a.dim = dim;
    a.row_bytes = dim * (int64_t) es;
    a.n_workers = n_workers;
    a.local_bits = local_bits;
    a.tile_rows = tile_rows;
    a.scale = scale;
    if (vec) {
        a.pieces = (int) (dim * es / 16);
        if (val_dtype == PX_F32) launch_segsum<float, true>(a, n_tiles, stream);
        else launch_segsum<uint16_t, true>(a, n_tiles, stream);
    } else {
        a.pieces = (int) dim;
        if (val_dtype == PX_F32) launch_segsum<float, false>(a, n_tiles, stream);
        else launch_segsum<uint16_t, false>(a, n_tiles, stream);
    }
    const unsigned fx = (unsigned) (n_tiles < 1024 ? n_tiles : 1024);
    k_fixup<<<dim3(fx, (unsigned) ((dim + 63) / 64), 1), 256, 0, stream>>>(
        sc.span_list, sc.counters, sc.run_start, tile_rows, dim, sc.pfirst, sc.plast, out_rows, scale,
        out_run_len, out_num_unique);
    return px_check_hip(ctx, hipGetLastError(), "coalesce launch");
}
