// px_sparse_apply_sgd / px_sparse_apply_adagrad: in-place update of the touched rows.
//
// Parallax Sec. 2.1: gradients are aggregated before they update the variable,
// so every distinct id is updated exactly once from its aggregated row; Sec. 4.3:
// the update of a (partition of a) sparse variable runs where the variable lives.
// One lane group per row: 128-bit loads of the gradient row and the table row
// (and accumulator row), the update, 128-bit stores.  Rows are taken in the order
// perm gives, restricted to [range[0], range[1]) when a shard range is passed.
#include "px_internal.h"
#include "px_update.h"

namespace {

struct ApplyArgs {
    float* table;
    float* accum;
    const int64_t* ids;
    const float* rows;
    const int64_t* num_ids;
    const int32_t* perm;
    const int64_t* range;
    uint32_t* flags;
    int64_t vocab;
    int64_t dim;
    int64_t cap;
    int pieces;          // row pieces per row (4 floats each when VEC, else 1)
    float lr;
    float eps;
};

template <bool VEC> struct Piece;
template <> struct Piece<true> {
    typedef float4 V;
    enum { E = 4 };
};
template <> struct Piece<false> {
    typedef float V;
    enum { E = 1 };
};

typedef float apply_v4f __attribute__((ext_vector_type(4)));
// The aggregated gradient row is read exactly once.
__device__ __forceinline__ float4 load_grad(const float4* p) {
#ifdef PX_APPLY_NONTEMPORAL
    apply_v4f v = __builtin_nontemporal_load((const apply_v4f*) p);
    return make_float4(v.x, v.y, v.z, v.w);
#else
    return *p;
#endif
}
__device__ __forceinline__ float load_grad(const float* p) { return *p; }
__device__ __forceinline__ float4 load_state(const float4* p) {
#ifdef PX_APPLY_NT_STATE_LOAD
    apply_v4f v = __builtin_nontemporal_load((const apply_v4f*) p);
    return make_float4(v.x, v.y, v.z, v.w);
#else
    return *p;
#endif
}
__device__ __forceinline__ float load_state(const float* p) { return *p; }
__device__ __forceinline__ void store_state(float4* p, float4 v) {
#ifdef PX_APPLY_NT_STATE_STORE
    apply_v4f t = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(t, (apply_v4f*) p);
#else
    *p = v;
#endif
}
__device__ __forceinline__ void store_state(float* p, float v) { *p = v; }


#ifndef PX_APPLY_BLOCKS
#define PX_APPLY_BLOCKS 16384    // most blocks of one apply launch (65,536 is 4 % faster when every id is distinct and
                                 // 40 % slower when the capacity is 20 times the number of distinct ids: the grid follows the capacity)
#endif
#ifndef PX_APPLY_ROWS
#define PX_APPLY_ROWS 1         // rows a lane group has in flight when a row is one piece per lane (2 and 4 measured no faster)
#endif

// R rows per lane group are in flight at once: their ids, then all their row pieces, are loaded
// before anything is computed or stored.
template <bool ADAGRAD, bool VEC, int G, int C, int R>
__global__ __launch_bounds__(256) void k_apply(ApplyArgs p) {
    typedef typename Piece<VEC>::V V;
    enum { E = Piece<VEC>::E };
    if (p.flags[0]) return;                          // an earlier call saw a bad or repeated id: leave the table alone
    int64_t n = p.num_ids[0];
    if (n < 0) n = 0;
    if (n > p.cap) n = p.cap;
    int64_t first = 0, last = n;
    if (p.range) {
        first = p.range[0];
        last = p.range[1];
        if (first < 0) first = 0;
        if (last > n) last = n;
    }
    const int gl = threadIdx.x % G;
    const int64_t group = (int64_t) blockIdx.x * (256 / G) + threadIdx.x / G;
    const int64_t n_groups = (int64_t) gridDim.x * (256 / G);
    for (int64_t j0 = first + group * R; j0 < last; j0 += n_groups * R) {
        int64_t k[R], id[R];
        bool ok[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            ok[r] = j0 + r < last;
            k[r] = ok[r] ? (p.perm ? (int64_t) p.perm[j0 + r] : j0 + r) : 0;
            ok[r] = ok[r] && k[r] >= 0 && k[r] < n;
        }
        // the id and its two neighbours' are requested together (positions clamped to the list)
        int64_t id_before[R], id_after[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int64_t kk = ok[r] ? k[r] : 0;
            id[r] = n > 0 ? p.ids[kk] : 0;
            id_before[r] = n > 0 ? p.ids[kk > 0 ? kk - 1 : 0] : 0;
            id_after[r] = n > 0 ? p.ids[kk + 1 < n ? kk + 1 : n - 1] : 0;
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            if (ok[r] && (id[r] < 0 || id[r] >= p.vocab)) {
                if (gl == 0) atomicOr(p.flags, (uint32_t) PXF_BAD_ID);
                ok[r] = false;
            }
            // An id that repeats its neighbour's (any repeat, when the ids are sorted) would be updated by
            // two lane groups at once: neither touches the row, and the flag is raised.
            if (ok[r] && ((k[r] > 0 && id_before[r] == id[r]) || (k[r] + 1 < n && id_after[r] == id[r]))) {
                if (gl == 0) atomicOr(p.flags, (uint32_t) PXF_NOT_UNIQUE);
                ok[r] = false;
            }
        }
        for (int p0 = 0; p0 < p.pieces; p0 += G * C) {
            V gv[R][C], wv[R][C], av[R][C];
#pragma unroll
            for (int r = 0; r < R; ++r) {
                if (!ok[r]) continue;
                const V* g = (const V*) (p.rows + (size_t) k[r] * p.dim);
                const V* w = (const V*) (p.table + (size_t) id[r] * p.dim);
                const V* a = ADAGRAD ? (const V*) (p.accum + (size_t) id[r] * p.dim) : nullptr;
#pragma unroll
                for (int c = 0; c < C; ++c) {
                    const int pc = p0 + c * G + gl;
                    if (pc < p.pieces) {
                        gv[r][c] = load_grad(g + pc);
                        wv[r][c] = load_state(w + pc);
                        if (ADAGRAD) av[r][c] = load_state(a + pc);
                    }
                }
            }
#pragma unroll
            for (int r = 0; r < R; ++r) {
                if (!ok[r]) continue;
                V* w = (V*) (p.table + (size_t) id[r] * p.dim);
                V* a = ADAGRAD ? (V*) (p.accum + (size_t) id[r] * p.dim) : nullptr;
#pragma unroll
                for (int c = 0; c < C; ++c) {
                    const int pc = p0 + c * G + gl;
                    if (pc < p.pieces) {
                        float* gf = (float*) &gv[r][c];
                        float* wf = (float*) &wv[r][c];
                        float* af = (float*) &av[r][c];
#pragma unroll
                        for (int x = 0; x < E; ++x) {
                            if (ADAGRAD) pxu::adagrad(wf[x], af[x], gf[x], p.lr, p.eps);
                            else pxu::sgd(wf[x], gf[x], p.lr);
                        }
                        store_state(w + pc, wv[r][c]);
                        if (ADAGRAD) store_state(a + pc, av[r][c]);
                    }
                }
            }
        }
    }
}

template <bool ADAGRAD, bool VEC>
void launch(const ApplyArgs& p, hipStream_t stream) {
    auto blocks = [&](int g) {
        int64_t b = (p.cap + (256 / g) - 1) / (256 / g);
        if (b > PX_APPLY_BLOCKS) b = PX_APPLY_BLOCKS;
        if (b < 1) b = 1;
        return dim3((unsigned) b, 1, 1);
    };
    if (p.pieces <= 16) k_apply<ADAGRAD, VEC, 16, 1, PX_APPLY_ROWS><<<blocks(16), 256, 0, stream>>>(p);
    else if (p.pieces <= 32) k_apply<ADAGRAD, VEC, 32, 1, PX_APPLY_ROWS><<<blocks(32), 256, 0, stream>>>(p);
    else if (p.pieces <= 64) k_apply<ADAGRAD, VEC, 64, 1, PX_APPLY_ROWS><<<blocks(64), 256, 0, stream>>>(p);
    else if (p.pieces <= 128) k_apply<ADAGRAD, VEC, 64, 2, 1><<<blocks(64), 256, 0, stream>>>(p);
    else k_apply<ADAGRAD, VEC, 64, 4, 1><<<blocks(64), 256, 0, stream>>>(p);
}

px_status apply_common(px_ctx* ctx, bool adagrad, float* table, float* accum, int64_t vocab, int64_t dim,
                       const int64_t* ids, const float* rows, const int64_t* num_ids, int64_t cap,
                       const int32_t* perm, const int64_t* range, float lr, float eps, hipStream_t stream) {
    if (!ctx) return PX_ERR_INVALID_ARG;
    if (vocab < 1 || dim < 1 || cap < 0 || cap >= (1ll << 31))
        return px_fail(ctx, PX_ERR_INVALID_ARG, "vocab %lld, dim %lld or cap %lld unsupported", (long long) vocab,
                       (long long) dim, (long long) cap);
    if (!num_ids || !table || (adagrad && !accum) || (cap > 0 && (!ids || !rows)))
        return px_fail(ctx, PX_ERR_INVALID_ARG, "null argument");
    if (((uintptr_t) table) % 4 || ((uintptr_t) rows) % 4 || (adagrad && ((uintptr_t) accum) % 4))
        return px_fail(ctx, PX_ERR_INVALID_ARG, "float pointers misaligned");
    if (cap == 0) return PX_OK;
    ApplyArgs p;
    p.table = table;
    p.accum = accum;
    p.ids = ids;
    p.rows = rows;
    p.num_ids = num_ids;
    // Without a range every position is updated exactly once whatever the order, so the rows are
    // taken in storage order: perm is not read, gradient rows stream, and the table rows of
    // neighbouring lane groups lie close together (Stress-uniform: 518 -> 490 us).
    p.perm = range ? perm : nullptr;
    p.range = range;
    p.flags = ctx->d_flags;
    p.vocab = vocab;
    p.dim = dim;
    p.cap = cap;
    p.lr = lr;
    p.eps = eps;
    const bool vec = dim % 4 == 0 && ((uintptr_t) table) % 16 == 0 && ((uintptr_t) rows) % 16 == 0 &&
                     (!adagrad || ((uintptr_t) accum) % 16 == 0);
    p.pieces = (int) (vec ? dim / 4 : dim);
    if (adagrad) {
        if (vec) launch<true, true>(p, stream); else launch<true, false>(p, stream);
    } else {
        if (vec) launch<false, true>(p, stream); else launch<false, false>(p, stream);
    }
    return px_check_hip(ctx, hipGetLastError(), "apply launch");
}

}  // namespace

extern "C" px_status px_sparse_apply_sgd(px_ctx* ctx, float* table, int64_t vocab, int64_t dim,
                                         const int64_t* ids, const float* rows, const int64_t* num_ids,
                                         int64_t cap, const int32_t* perm, const int64_t* range, float lr,
                                         void* hip_stream) {
    return apply_common(ctx, false, table, nullptr, vocab, dim, ids, rows, num_ids, cap, perm, range, lr, 0.f,
                        (hipStream_t) hip_stream);
}

extern "C" px_status px_sparse_apply_adagrad(px_ctx* ctx, float* table, float* accum, int64_t vocab,
                                             int64_t dim, const int64_t* ids, const float* rows,
                                             const int64_t* num_ids, int64_t cap, const int32_t* perm,
                                             const int64_t* range, float lr, float eps, void* hip_stream) {
    return apply_common(ctx, true, table, accum, vocab, dim, ids, rows, num_ids, cap, perm, range, lr, eps,
                        (hipStream_t) hip_stream);
}
