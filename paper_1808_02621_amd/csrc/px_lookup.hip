// px_sparse_lookup: the pull side of a partitioned sparse variable.
//
// Parallax Sec. 3.1: each iteration a worker pulls the rows of a sparse variable
// that its mini-batch touches; Sec. 3.2: with the variable partitioned, the rows
// come from the partitions and are stitched back into one tensor in the order the
// batch asked for them (the cost that grows with the number of partitions).  Here
// the variable is one [vocab][dim] array whose shards are logical, so looking a
// row up in its shard and placing it at its batch position is one gather:
//   out[k][:] = table[ids[k]][:]      for k = perm[j], j in [first, last)
// With perm / range from px_partition_rows a call serves one shard's part of the
// batch; with both NULL it produces the whole stitched result.  One lane group per
// row, 128-bit loads and stores; ids may repeat.
#include <type_traits>

#include "px_internal.h"

namespace {

struct LookupArgs {
    const float* table;
    const int64_t* ids;
    const int64_t* num_ids;
    const int32_t* perm;
    const int64_t* range;
    float* out;
    uint32_t* flags;
    int64_t vocab;
    int64_t dim;
    int64_t cap;
    int pieces;
};

#ifndef PX_LOOKUP_WIDE_ROWS
#define PX_LOOKUP_WIDE_ROWS 1
#endif
#ifndef PX_LOOKUP_WIDE_DIE
#define PX_LOOKUP_WIDE_DIE true
#endif
#ifndef PX_LOOKUP_BLOCKS
#define PX_LOOKUP_BLOCKS 65536    // most workgroups of one lookup launch (measured: 2,048 ... 16,384 are 2-7 % slower)
#endif

// DIE: the hardware's workgroup number is mapped so that each of the 8 dies gathers one contiguous
// eighth of the requested rows (the grid is then a multiple of 8).
template <bool VEC, int G, int R, bool DIE>
__global__ __launch_bounds__(256) void k_lookup(LookupArgs p) {
    typedef typename std::conditional<VEC, float4, float>::type V;
    enum { E = VEC ? 4 : 1 };
    int64_t n = p.num_ids ? p.num_ids[0] : p.cap;
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
    const int64_t group = (int64_t) (DIE ? px_die_contiguous_block(blockIdx.x, gridDim.x) : blockIdx.x) * (256 / G) + threadIdx.x / G;
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
#pragma unroll
        for (int r = 0; r < R; ++r) {
            id[r] = ok[r] ? p.ids[k[r]] : 0;
            if (ok[r] && (id[r] < 0 || id[r] >= p.vocab)) {
                if (gl == 0) atomicOr(p.flags, (uint32_t) PXF_BAD_ID);
                ok[r] = false;
            }
        }
        for (int p0 = gl; p0 < p.pieces; p0 += G) {
            V v[R];
#pragma unroll
            for (int r = 0; r < R; ++r)
                if (ok[r]) v[r] = ((const V*) (p.table + (size_t) id[r] * p.dim))[p0];
#pragma unroll
            for (int r = 0; r < R; ++r)
                if (ok[r]) {
#ifndef PX_LOOKUP_PLAIN_STORE
                    // the gathered rows are written once and not read here again: storing them past the
                    // caches leaves the L2 to the table rows, which hot ids make it re-read
                    if constexpr (VEC) {
                        typedef float v4f __attribute__((ext_vector_type(4)));
                        v4f t = {v[r].x, v[r].y, v[r].z, v[r].w};
                        __builtin_nontemporal_store(t, (v4f*) (p.out + (size_t) k[r] * p.dim) + p0);
                    } else {
                        ((V*) (p.out + (size_t) k[r] * p.dim))[p0] = v[r];
                    }
#else
                    ((V*) (p.out + (size_t) k[r] * p.dim))[p0] = v[r];
#endif
                }
        }
    }
}

template <bool VEC>
void launch(const LookupArgs& p, hipStream_t stream) {
    auto blocks = [&](int g, int r) {
        int64_t b = (p.cap + (256 / g) * r - 1) / ((256 / g) * r);
        if (b > PX_LOOKUP_BLOCKS) b = PX_LOOKUP_BLOCKS;
        if (b < 1) b = 1;
        return dim3(px_round_up_8((unsigned) b), 1, 1);
    };
    // rows of more than 32 pieces (512 bytes): one row in flight per lane group and die-contiguous
    // numbering (measured: NMT-like 147 -> 132 us, Large-vocab LM 56 -> 54.5 us; for narrower rows the numbering costs up to 9 %)
    if (p.pieces <= 16) k_lookup<VEC, 16, 4, false><<<blocks(16, 4), 256, 0, stream>>>(p);
    else if (p.pieces <= 32) k_lookup<VEC, 32, 4, false><<<blocks(32, 4), 256, 0, stream>>>(p);
    else k_lookup<VEC, 64, PX_LOOKUP_WIDE_ROWS, PX_LOOKUP_WIDE_DIE><<<blocks(64, PX_LOOKUP_WIDE_ROWS), 256, 0, stream>>>(p);
}

}  // namespace

extern "C" px_status px_sparse_lookup(px_ctx* ctx, const float* table, int64_t vocab, int64_t dim,
                                      const int64_t* ids, const int64_t* num_ids, int64_t cap,
                                      const int32_t* perm, const int64_t* range, float* out_rows,
                                      void* hip_stream) {
    if (!ctx) return PX_ERR_INVALID_ARG;
    if (vocab < 1 || dim < 1 || cap < 0 || cap >= (1ll << 31))
        return px_fail(ctx, PX_ERR_INVALID_ARG, "vocab %lld, dim %lld or cap %lld unsupported", (long long) vocab,
                       (long long) dim, (long long) cap);
    if (cap == 0) return PX_OK;
    if (!table || !ids || !out_rows) return px_fail(ctx, PX_ERR_INVALID_ARG, "null argument");
    if (((uintptr_t) table) % 4 || ((uintptr_t) out_rows) % 4 || ((uintptr_t) ids) % 8)
        return px_fail(ctx, PX_ERR_INVALID_ARG, "pointers misaligned");
    LookupArgs p;
    p.table = table;
    p.ids = ids;
    p.num_ids = num_ids;
    p.perm = perm;
    p.range = range;
    p.out = out_rows;
    p.flags = ctx->d_flags;
    p.vocab = vocab;
    p.dim = dim;
    p.cap = cap;
    const bool vec = dim % 4 == 0 && ((uintptr_t) table) % 16 == 0 && ((uintptr_t) out_rows) % 16 == 0;
    p.pieces = (int) (vec ? dim / 4 : dim);
    if (vec) launch<true>(p, (hipStream_t) hip_stream);
    else launch<false>(p, (hipStream_t) hip_stream);
    return px_check_hip(ctx, hipGetLastError(), "lookup launch");
}
