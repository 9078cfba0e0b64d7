// px_dense_average: element-wise reduction of N workers' dense gradient buffers.
//
// Parallax Sec. 2.1: AllReduce computes the sum over the workers of their
// gradients (Sec. 4.1: or the average); this is the reduction one GPU performs
// on the slice it owns.  One streaming pass: each thread owns four 16-byte pieces of
// every input buffer (4 floats or 8 bfloat16 each), reads them buffer by buffer,
// adds in worker order and writes once.  Pure HBM streaming: N*C*es bytes in, C*4 (or C*2) out.
#include <string.h>

#include "px_internal.h"

namespace {

#ifdef PX_DENSE_ACC_FLOAT
typedef float acc_t;
#else
typedef double acc_t;
#endif

#ifndef PX_DENSE_BATCH
#define PX_DENSE_BATCH 1        // buffers a thread reads from at a time (with 4 pieces each: 4 loads in flight; two
                                // buffers at a time, 8 loads, are 2-3 % slower on 48 bfloat16 buffers and the same elsewhere)
#endif
enum { DENSE_BATCH = PX_DENSE_BATCH };
#ifndef PX_DENSE_PIECES
#define PX_DENSE_PIECES 4       // 16-byte pieces of every buffer per thread, 4 KB apart (measured: 4 x 2 >= 2 x 2 >= 1 x 4 > 1 x 8)
#endif

typedef uint32_t v4u __attribute__((ext_vector_type(4)));

// Every input byte is read exactly once: non-temporal loads keep the stream out of the caches.
__device__ __forceinline__ uint4 load16(const uint4* p) {
#ifdef PX_DENSE_TEMPORAL
    return *p;
#else
    v4u v = __builtin_nontemporal_load((const v4u*) p);
    return make_uint4(v.x, v.y, v.z, v.w);
#endif
}

__device__ __forceinline__ uint16_t to_bf16(float f) {   // round to nearest, ties to even
    uint32_t u = __float_as_uint(f);
    // a NaN stays a NaN (quiet bit set): the rounding bias would carry it into infinity or zero
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t) ((u >> 16) | 0x0040u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t) (u >> 16);
}

template <typename TIN> struct In;
template <> struct In<float> {
    enum { E = 4 };
    static __device__ __forceinline__ void add(acc_t* acc, const uint4& r) {
        acc[0] += (acc_t) __uint_as_float(r.x);
        acc[1] += (acc_t) __uint_as_float(r.y);
        acc[2] += (acc_t) __uint_as_float(r.z);
        acc[3] += (acc_t) __uint_as_float(r.w);
    }
    static __device__ __forceinline__ float widen(float v) { return v; }
};
template <> struct In<uint16_t> {
    enum { E = 8 };
    static __device__ __forceinline__ void add(acc_t* acc, const uint4& r) {
        acc[0] += (acc_t) __uint_as_float(r.x << 16);
        acc[1] += (acc_t) __uint_as_float(r.x & 0xffff0000u);
        acc[2] += (acc_t) __uint_as_float(r.y << 16);
        acc[3] += (acc_t) __uint_as_float(r.y & 0xffff0000u);
        acc[4] += (acc_t) __uint_as_float(r.z << 16);
        acc[5] += (acc_t) __uint_as_float(r.z & 0xffff0000u);
        acc[6] += (acc_t) __uint_as_float(r.w << 16);
        acc[7] += (acc_t) __uint_as_float(r.w & 0xffff0000u);
    }
    static __device__ __forceinline__ float widen(uint16_t v) { return __uint_as_float((uint32_t) v << 16); }
};

#ifndef PX_DENSE_THREADS
#define PX_DENSE_THREADS 256    // threads of a k_dense_vec workgroup
#endif
// A workgroup owns 4 consecutive kilobyte-rows of 256 pieces (16 bytes each) of every buffer; a thread
// owns one piece of each row.
#ifndef PX_DENSE_LAUNCH_PIECES
#define PX_DENSE_LAUNCH_PIECES (1 << 19)    // pieces per launch (0: one launch for everything)
#endif
#ifndef PX_DENSE_LAUNCH_OUT_MB
#define PX_DENSE_LAUNCH_OUT_MB 16           // most output bytes per launch, in MiB
#endif

// The buffer pointers come from the context's device table (words) or, for up to PX_UPLOAD_WORDS
// buffers, inside the launch arguments (pack, CARRIED), which saves the upload launch.
// One launch covers pieces [first, pieces).
template <typename TIN, bool OUT_BF16, bool CARRIED>
__global__ __launch_bounds__(PX_DENSE_THREADS) void k_dense_vec(const uint64_t* __restrict__ words, px_word_pack pack,
                                                   int n_buffers, int64_t first, int64_t pieces,
                                                   void* __restrict__ out, float scale) {
    enum { E = In<TIN>::E };
#ifndef PX_DENSE_PLAIN_BLOCKS
    const unsigned lb = px_die_contiguous_block(blockIdx.x, gridDim.x);    // the grid is a multiple of 8
#else
    const unsigned lb = blockIdx.x;
#endif
    const uint4* const* bufs = (const uint4* const*) (CARRIED ? pack.w : words);
    enum { P = PX_DENSE_PIECES };
    int64_t ip[P];
    bool okp[P];
#pragma unroll
    for (int q = 0; q < P; ++q) {
        ip[q] = first + ((int64_t) lb * P + q) * PX_DENSE_THREADS + threadIdx.x;
        okp[q] = ip[q] < pieces;
        if (!okp[q]) ip[q] = pieces - 1;
    }
    if (!okp[0]) return;
    acc_t acc[P][E];
#pragma unroll
    for (int q = 0; q < P; ++q)
#pragma unroll
        for (int x = 0; x < E; ++x) acc[q][x] = (acc_t) 0;
    for (int w0 = 0; w0 < n_buffers; w0 += DENSE_BATCH) {
        uint4 r[DENSE_BATCH][P];
#pragma unroll
        for (int j = 0; j < DENSE_BATCH; ++j)
            if (w0 + j < n_buffers) {
#pragma unroll
                for (int q = 0; q < P; ++q) r[j][q] = load16(bufs[w0 + j] + ip[q]);
            }
#pragma unroll
        for (int j = 0; j < DENSE_BATCH; ++j)
            if (w0 + j < n_buffers) {
#pragma unroll
                for (int q = 0; q < P; ++q) In<TIN>::add(acc[q], r[j][q]);
            }
    }
#pragma unroll
    for (int q = 0; q < P; ++q) {
        if (!okp[q]) continue;
        const int64_t i = ip[q];
        float o[E];
#pragma unroll
        for (int x = 0; x < E; ++x) o[x] = (float) (acc[q][x] * (acc_t) scale);
        if (OUT_BF16) {
            uint16_t* dst = (uint16_t*) out + i * E;
            if constexpr (E == 8) {
                uint4 v;
                v.x = to_bf16(o[0]) | ((uint32_t) to_bf16(o[1]) << 16);
                v.y = to_bf16(o[2]) | ((uint32_t) to_bf16(o[3]) << 16);
                v.z = to_bf16(o[4]) | ((uint32_t) to_bf16(o[5]) << 16);
                v.w = to_bf16(o[6]) | ((uint32_t) to_bf16(o[7]) << 16);
                *(uint4*) dst = v;
            } else {
                uint2 v;
                v.x = to_bf16(o[0]) | ((uint32_t) to_bf16(o[1]) << 16);
                v.y = to_bf16(o[2]) | ((uint32_t) to_bf16(o[3]) << 16);
                *(uint2*) dst = v;
            }
        } else {
            float4* dst = (float4*) ((float*) out + i * E);
#pragma unroll
            for (int x = 0; x < E; x += 4) dst[x / 4] = make_float4(o[x], o[x + 1], o[x + 2], o[x + 3]);
        }
    }
}

// One element per thread, for unaligned buffers and for the tail behind the last full piece.
template <typename TIN, bool OUT_BF16, bool CARRIED>
__global__ __launch_bounds__(256) void k_dense_scalar(const uint64_t* __restrict__ words, px_word_pack pack,
                                                      int n_buffers, int64_t first, int64_t count,
                                                      void* __restrict__ out, float scale) {
    const int64_t i = first + (int64_t) blockIdx.x * 256 + threadIdx.x;
    if (i >= count) return;
    const TIN* const* bufs = (const TIN* const*) (CARRIED ? pack.w : words);
    acc_t acc = (acc_t) 0;
    for (int w = 0; w < n_buffers; ++w) acc += (acc_t) In<TIN>::widen(bufs[w][i]);
    const float o = (float) (acc * (acc_t) scale);
    if (OUT_BF16) ((uint16_t*) out)[i] = to_bf16(o);
    else ((float*) out)[i] = o;
}

// Pieces (16 bytes of every input buffer) one launch covers.  A long output is produced by several
// launches in a row, each small enough for its output to stay in the L2 caches until the launch
// ends and is written back in one burst: a steady trickle of writes between the reads costs this
// machine more than the extra launches do.
//   - 2^19 pieces (two workgroups of 1,024 pieces per compute unit): the measured optimum for 48 buffers;
//   - more when there are few buffers, so that a launch still reads about 256 MiB;
//   - never more than 16 MiB of output, half of what the L2 caches hold together.
int64_t pieces_per_launch(int n_buffers, int64_t out_piece_bytes) {
    if (PX_DENSE_LAUNCH_PIECES <= 0) return (int64_t) 1 << 62;         // one launch for everything
    int64_t per = PX_DENSE_LAUNCH_PIECES;
    const int64_t for_bytes = ((int64_t) 256 << 20) / ((int64_t) (n_buffers > 0 ? n_buffers : 1) * 16);
    if (per < for_bytes) per = for_bytes;
    const int64_t cap = ((int64_t) PX_DENSE_LAUNCH_OUT_MB << 20) / out_piece_bytes;
    if (per > cap) per = cap;
    return per;
}

template <typename TIN, bool OUT_BF16, bool CARRIED>
void launch(px_ctx* ctx, const px_word_pack& pack, int n, int64_t count, bool vec, void* out, float scale,
            hipStream_t stream) {
    enum { E = In<TIN>::E };
    int64_t done = 0;
    if (vec) {
        const int64_t pieces = count / E;
        const int64_t per_launch = pieces_per_launch(n, E * (OUT_BF16 ? 2 : 4));
        for (int64_t first = 0; first < pieces; first += per_launch) {
            const int64_t last = first + per_launch < pieces ? first + per_launch : pieces;
            k_dense_vec<TIN, OUT_BF16, CARRIED><<<px_round_up_8((unsigned) ((last - first + PX_DENSE_THREADS * PX_DENSE_PIECES - 1) / (PX_DENSE_THREADS * PX_DENSE_PIECES))), PX_DENSE_THREADS, 0, stream>>>(
                ctx->d_words, pack, n, first, last, out, scale);
        }
        done = pieces * E;
    }
    // element-wise: unaligned buffers, or the tail behind the last full piece; at most 2^30 elements a launch
    const int64_t scalar_chunk = (int64_t) 1 << 30;
    for (; done < count; done += scalar_chunk) {
        const int64_t last = done + scalar_chunk < count ? done + scalar_chunk : count;
        k_dense_scalar<TIN, OUT_BF16, CARRIED><<<(unsigned) ((last - done + 255) / 256), 256, 0, stream>>>(
            ctx->d_words, pack, n, done, last, out, scale);
    }
}

template <bool CARRIED>
void launch_dtype(px_ctx* ctx, const px_word_pack& pack, int n, int64_t count, bool vec, px_dtype in_dtype,
                  void* out, px_dtype out_dtype, float scale, hipStream_t stream) {
    if (in_dtype == PX_F32) {
        if (out_dtype == PX_F32) launch<float, false, CARRIED>(ctx, pack, n, count, vec, out, scale, stream);
        else launch<float, true, CARRIED>(ctx, pack, n, count, vec, out, scale, stream);
    } else {
        if (out_dtype == PX_F32) launch<uint16_t, false, CARRIED>(ctx, pack, n, count, vec, out, scale, stream);
        else launch<uint16_t, true, CARRIED>(ctx, pack, n, count, vec, out, scale, stream);
    }
}

}  // namespace

extern "C" int64_t px_dense_average_launches(int n_buffers, int64_t count, px_dtype in_dtype, px_dtype out_dtype) {
    if (n_buffers < 1 || count < 1) return 0;
    const int64_t e = in_dtype == PX_F32 ? 4 : 8;
    const int64_t pieces = count / e;
    if (pieces == 0) return 0;
    const int64_t per = pieces_per_launch(n_buffers, e * (out_dtype == PX_F32 ? 4 : 2));
    return (pieces + per - 1) / per;
}

extern "C" px_status px_dense_average(px_ctx* ctx, int n_buffers, const void* const* bufs, int64_t count,
                                      px_dtype in_dtype, void* out, px_dtype out_dtype, float scale,
                                      void* hip_stream) {
    if (!ctx) return PX_ERR_INVALID_ARG;
    hipStream_t stream = (hipStream_t) hip_stream;
    if (n_buffers < 1 || n_buffers > PX_MAX_SOURCES)
        return px_fail(ctx, PX_ERR_INVALID_ARG, "n_buffers %d outside [1, %d]", n_buffers, (int) PX_MAX_SOURCES);
    if ((in_dtype != PX_F32 && in_dtype != PX_BF16) || (out_dtype != PX_F32 && out_dtype != PX_BF16))
        return px_fail(ctx, PX_ERR_INVALID_ARG, "unknown dtype");
    if (count < 0 || count > (1ll << 40)) return px_fail(ctx, PX_ERR_INVALID_ARG, "count %lld unsupported", (long long) count);
    if (count == 0) return PX_OK;
    if (!bufs || !out) return px_fail(ctx, PX_ERR_INVALID_ARG, "null argument");
    const size_t es = in_dtype == PX_F32 ? 4 : 2, os = out_dtype == PX_F32 ? 4 : 2;
    bool vec = ((uintptr_t) out) % 16 == 0;
    if (((uintptr_t) out) % os) return px_fail(ctx, PX_ERR_INVALID_ARG, "out misaligned");
    uint64_t host_words[PX_MAX_SOURCES];
    for (int w = 0; w < n_buffers; ++w) {
        if (!bufs[w] || ((uintptr_t) bufs[w]) % es) return px_fail(ctx, PX_ERR_INVALID_ARG, "buffer %d null or misaligned", w);
        if (((uintptr_t) bufs[w]) % 16) vec = false;
        host_words[w] = (uint64_t) (uintptr_t) bufs[w];
    }
    px_word_pack pack;
    if (n_buffers <= PX_UPLOAD_WORDS) {
        memcpy(pack.w, host_words, (size_t) n_buffers * sizeof(uint64_t));
        launch_dtype<true>(ctx, pack, n_buffers, count, vec, in_dtype, out, out_dtype, scale, stream);
    } else {
        px_status st = px_upload_words(ctx, ctx->d_words, host_words, n_buffers, nullptr, 0, stream);
        if (st != PX_OK) return st;
        pack.w[0] = 0;
        launch_dtype<false>(ctx, pack, n_buffers, count, vec, in_dtype, out, out_dtype, scale, stream);
    }
    return px_check_hip(ctx, hipGetLastError(), "dense launch");
}
