// CPU oracle for the sparse/dense gradient aggregation path of Parallax
// (arXiv 1808.02621).  TEST INFRASTRUCTURE ONLY: tests, the smoke check and the
// benchmark's cpu_baseline leg may call it; the product path never does.
//
// Plain, slow and meant to be checked against the paper by eye: an ordered-map
// row accumulator in double precision, scalar optimizer updates, a scalar mean.
// It shares no code with the HIP library.  Host pointers everywhere.
//
// Every function is pinned by tests that do not go through this file
// (brute-force densification, invariants, closed forms, library routines).
//
// Build: g++ -O2 -std=c++17 -shared -fPIC -o libpx_oracle.so px_oracle.cpp

#include <cmath>
#include <cstdint>
#include <cstring>
#include <map>
#include <vector>

namespace {

enum { DT_F32 = 0, DT_BF16 = 1 };
enum { HASH_MOD = 0, HASH_MUL = 1 };
enum { AGG_SUM = 0, AGG_AVERAGE = 1 };

// bfloat16 is the upper half of a float32: widening is a 16-bit shift, exact.
double load_value(const void* base, int dtype, int64_t i) {
    if (dtype == DT_BF16) {
        uint32_t bits = (uint32_t) static_cast<const uint16_t*>(base)[i] << 16;
        float f;
        std::memcpy(&f, &bits, sizeof f);
        return (double) f;
    }
    return (double) static_cast<const float*>(base)[i];
}

int64_t shard_of(int64_t id, int n_shards, int hash) {
    uint64_t h = (uint64_t) id;
    if (hash == HASH_MUL) h *= 2654435761ULL;  // Knuth's multiplicative constant, wraps mod 2^64
    return (int64_t) (h % (uint64_t) n_shards);
}

}  // namespace

extern "C" {

// Sparse gradient aggregation (Fig. 3 caption; Sec. 3.2: gradients of a sparse
// variable from all workers are concatenated, then values carrying the same
// index are accumulated).  Workers are visited in order 0..N-1, rows in order.
// aggregation = AGG_AVERAGE divides by the number of workers (Sec. 4.1: the
// average of gradients over all GPUs), not by how often a row occurs.
// Output ids ascending; out_run_len[k] = how many input rows carried out_ids[k].
// Returns U, or -1 if an id is outside [0, vocab) (outputs then untouched).
int64_t pxo_sparse_coalesce(int n_workers, const int64_t* const* idx, const void* const* val,
                            const int64_t* counts, int64_t dim, int val_dtype, int64_t vocab,
                            int aggregation, int64_t* out_ids, float* out_rows,
                            int32_t* out_run_len) {
    for (int w = 0; w < n_workers; ++w)
        for (int64_t i = 0; i < counts[w]; ++i)
            if (idx[w][i] < 0 || idx[w][i] >= vocab) return -1;

    std::map<int64_t, std::vector<double>> acc;
    std::map<int64_t, int32_t> seen;
    for (int w = 0; w < n_workers; ++w) {
        for (int64_t i = 0; i < counts[w]; ++i) {
            std::vector<double>& row = acc[idx[w][i]];
            if (row.empty()) row.assign((size_t) dim, 0.0);
            for (int64_t d = 0; d < dim; ++d) row[(size_t) d] += load_value(val[w], val_dtype, i * dim + d);
            seen[idx[w][i]] += 1;
        }
    }
    int64_t k = 0;
    for (const auto& kv : acc) {
        out_ids[k] = kv.first;
        for (int64_t d = 0; d < dim; ++d) {
            double s = kv.second[(size_t) d];
            if (aggregation == AGG_AVERAGE) s /= (double) n_workers;
            out_rows[k * dim + d] = (float) s;  // the only rounding
        }
        if (out_run_len) out_run_len[k] = seen[kv.first];
        ++k;
    }
    return k;
}

// Partitioning of a sparse variable (Sec. 3.2: incoming indices and values are
// divided into disjoint sets, one per partition).  shard = H(id) mod P with
// H = identity (HASH_MOD) or multiplication by 2654435761 mod 2^64 (HASH_MUL).
// perm lists positions 0..n-1 grouped by shard, input order kept inside a shard;
// offsets[p]..offsets[p+1] is shard p's slice of perm.
int pxo_partition_rows(const int64_t* ids, int64_t n, int n_shards, int hash, int32_t* out_shard,
                       int32_t* out_perm, int64_t* out_offsets) {
    if (n_shards < 1) return 1;
    std::vector<int64_t> fill((size_t) n_shards, 0);
    for (int64_t k = 0; k < n; ++k) fill[(size_t) shard_of(ids[k], n_shards, hash)] += 1;
    out_offsets[0] = 0;
    for (int p = 0; p < n_shards; ++p) out_offsets[p + 1] = out_offsets[p] + fill[(size_t) p];
    std::vector<int64_t> next(out_offsets, out_offsets + n_shards);
    for (int64_t k = 0; k < n; ++k) {
        int64_t p = shard_of(ids[k], n_shards, hash);
        if (out_shard) out_shard[k] = (int32_t) p;
        out_perm[next[(size_t) p]++] = (int32_t) k;
    }
    return 0;
}

// Sparse variable update, plain gradient descent (Fig. 4 uses
// GradientDescentOptimizer; Sec. 2.1: gradients are aggregated before they
// update the variable, so each distinct id is updated exactly once).
// W[id] <- W[id] - lr * g, visiting rows in the order perm gives (NULL = 0..n-1).
// Returns 0, 2 for an id outside the table, 4 for a repeated id; the table is
// untouched on error.
int pxo_sparse_apply_sgd(float* table, int64_t vocab, int64_t dim, const int64_t* ids,
                         const float* rows, int64_t n, const int32_t* perm, double lr) {
    std::map<int64_t, int> once;
    for (int64_t k = 0; k < n; ++k) {
        if (ids[k] < 0 || ids[k] >= vocab) return 2;
        if (once[ids[k]]++) return 4;
    }
    for (int64_t j = 0; j < n; ++j) {
        int64_t k = perm ? perm[j] : j;
        float* w = table + ids[k] * dim;
        const float* g = rows + k * dim;
        for (int64_t d = 0; d < dim; ++d) w[d] = (float) ((double) w[d] - lr * (double) g[d]);
    }
    return 0;
}

// Sparse variable update, Adagrad (Duchi et al.): per element
//   A <- A + g^2 ;  W <- W - lr * g / (sqrt(A) + eps)      with the updated A.
// Arithmetic in double, each stored value rounded once.  Same preconditions
// and return codes as the gradient-descent update.
int pxo_sparse_apply_adagrad(float* table, float* accum, int64_t vocab, int64_t dim,
                             const int64_t* ids, const float* rows, int64_t n, const int32_t* perm,
                             double lr, double eps) {
    std::map<int64_t, int> once;
    for (int64_t k = 0; k < n; ++k) {
        if (ids[k] < 0 || ids[k] >= vocab) return 2;
        if (once[ids[k]]++) return 4;
    }
    for (int64_t j = 0; j < n; ++j) {
        int64_t k = perm ? perm[j] : j;
        float* w = table + ids[k] * dim;
        float* a = accum + ids[k] * dim;
        const float* g = rows + k * dim;
        for (int64_t d = 0; d < dim; ++d) {
            double gd = (double) g[d];
            double ad = (double) a[d] + gd * gd;
            a[d] = (float) ad;
            w[d] = (float) ((double) w[d] - lr * gd / (std::sqrt(ad) + eps));
        }
    }
    return 0;
}

// Dense gradient aggregation (Sec. 2.1: AllReduce computes the sum over the N
// workers of their gradients; Sec. 4.1: optionally the average over all GPUs).
int pxo_dense_average(int n_buffers, const void* const* bufs, int64_t count, int in_dtype,
                      int aggregation, float* out) {
    for (int64_t j = 0; j < count; ++j) {
        double s = 0.0;
        for (int w = 0; w < n_buffers; ++w) s += load_value(bufs[w], in_dtype, j);
        if (aggregation == AGG_AVERAGE) s /= (double) n_buffers;
        out[j] = (float) s;
    }
    return 0;
}

// The pull side of a partitioned sparse variable (Sec. 3.1: a worker pulls the rows its
// mini-batch touches; Sec. 3.2: rows looked up per partition are stitched into one tensor in
// the order of the request).  out[k] = table[ids[k]] for k = perm[j], j in [first, last);
// perm NULL = identity.  Rows outside the range are left as they are.  Returns 2 for a bad id.
int pxo_sparse_lookup(const float* table, int64_t vocab, int64_t dim, const int64_t* ids, int64_t n,
                      const int32_t* perm, int64_t first, int64_t last, float* out) {
    for (int64_t j = first; j < last && j < n; ++j) {
        int64_t k = perm ? perm[j] : j;
        if (ids[k] < 0 || ids[k] >= vocab) return 2;
    }
    for (int64_t j = first; j < last && j < n; ++j) {
        int64_t k = perm ? perm[j] : j;
        for (int64_t d = 0; d < dim; ++d) out[k * dim + d] = table[ids[k] * dim + d];
    }
    return 0;
}

}  // extern "C"
