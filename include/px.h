/*
 * px.h -- C ABI of the sparse/dense gradient aggregation hot path of Parallax
 * (Kim et al., "Parallax: Sparsity-aware Data Parallel Training of Deep Neural
 * Networks", EuroSys '19, arXiv 1808.02621) for AMD MI355X (gfx950).
 *
 * The paper routes the gradients of sparse variables (embedding tables; the
 * gradient is a pair of arrays, row indices and value rows, Sec. 2.2) through
 * parameter servers that aggregate them index by index and update the rows
 * they own, and the gradients of dense variables through AllReduce (Sec. 3.1,
 * Sec. 4.3).  This library is the arithmetic of that path on one GPU:
 *
 *   px_sparse_coalesce       aggregate N workers' sparse gradients of one variable
 *   px_partition_rows        split the aggregated rows into P disjoint shards
 *   px_sparse_apply_sgd      update the touched rows in place, gradient descent
 *   px_sparse_apply_adagrad  update the touched rows in place, Adagrad
 *   px_dense_average         reduce N workers' dense gradient buffers (sum or mean)
 * and, fused, the first and third of these without the aggregated rows ever being stored:
 *   px_sparse_coalesce_apply_sgd / px_sparse_coalesce_apply_adagrad
 * and the pull side, the rows of a (partitioned) variable a mini-batch asks for:
 *   px_sparse_lookup
 *
 * Conventions for every call
 *   - "dev" pointers are device (HBM) addresses on the context's GPU; "host"
 *     pointers are ordinary host memory.  The caller owns every buffer,
 *     scratch included; the library never frees or keeps caller memory.
 *   - Calls only enqueue work on `hip_stream` (a hipStream_t passed as void*,
 *     NULL = the default stream) and return; nothing synchronises.  Sizes that
 *     depend on the data stay on the device: the number of distinct ids is a
 *     device scalar, and outputs have worst-case capacity.
 *   - Host arrays (pointer tables, counts) are read before the call returns.
 *   - Argument errors are found on the host before anything is enqueued and
 *     leave all buffers untouched.  Errors that only the device can see (an id
 *     outside the table; an update handed a repeated id) raise a sticky flag in
 *     the context: the kernels stay in bounds, the coalesced count becomes 0
 *     for a bad id, the offending rows are not updated, and every later update
 *     on that context leaves its table untouched until px_device_status has
 *     reported and cleared the flag.  A caller that never polls therefore
 *     loses updates after the first error: poll once per step (it is the one
 *     call that blocks) or at whatever interval losing updates is acceptable.
 *   - One context per stream; calls on one context must not overlap.
 *   - Empty inputs (no rows, a worker with no rows, count 0) are valid no-ops.
 */
#ifndef PX_H_
#define PX_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct px_ctx px_ctx;

typedef enum {
    PX_OK = 0,
    PX_ERR_INVALID_ARG = 1,        /* bad pointer, size, dtype, alignment or unsupported shape */
    PX_ERR_INDEX_OUT_OF_RANGE = 2, /* an id outside [0, vocab) reached the device */
    PX_ERR_SCRATCH_TOO_SMALL = 3,
    PX_ERR_NOT_UNIQUE = 4,         /* an update was handed the same id in adjacent positions */
    PX_ERR_DEVICE = 5              /* a HIP runtime call failed */
} px_status;

typedef enum { PX_F32 = 0, PX_BF16 = 1 } px_dtype;

/* Shard function H(id) mod P.  PX_HASH_MOD: H(id) = id.  PX_HASH_MUL:
 * H(id) = id * 2654435761 taken modulo 2^64 (unsigned wrap-around). */
typedef enum { PX_HASH_MOD = 0, PX_HASH_MUL = 1 } px_hash;

enum {
    PX_MAX_SOURCES = 1024, /* most workers / dense buffers in one call */
    PX_MAX_SHARDS = 256,   /* most shards in one px_partition_rows call (Table 2 sweeps 8..256) */
    PX_PARTITION_NOALLOC_MAX_IDS = 1 << 22 /* largest cap px_partition_rows_noalloc accepts */
};

/* Create a context on GPU `device`.  Allocates a few hundred KB of device and
 * pinned host memory that live until px_destroy.  Not on the hot path. */
px_status px_create(px_ctx** out, int device);
px_status px_destroy(px_ctx* ctx);

const char* px_status_string(px_status s);
/* Message of the last failed call on this context ("" if none).  Host string owned by ctx. */
const char* px_last_error(const px_ctx* ctx);

/* Waits for `hip_stream`, then reports and clears the context's device-side
 * error flag: PX_OK, PX_ERR_INDEX_OUT_OF_RANGE, or PX_ERR_NOT_UNIQUE (in that
 * order of precedence when both were raised).  PX_ERR_DEVICE, ahead of both,
 * if a workgroup gave up one of the library's bounded waits for another
 * workgroup's published count (head ranking, small partitions): the outputs of
 * that call are then invalid.  The only call that blocks. */
px_status px_device_status(px_ctx* ctx, void* hip_stream);

/* Two kernels let a workgroup wait for a count another workgroup publishes (head ranking in the
 * coalesce calls; px_partition_rows when it runs as one launch).  Every such wait is bounded: after
 * `polls` polls (default 2^18, about a third of a second) the workgroup gives up, the call's outputs
 * are invalid, nothing is read or written out of bounds, later updates on the context leave their
 * tables alone, and px_device_status reports PX_ERR_DEVICE.  0 makes every wait give up at its first
 * unsuccessful poll, which is how the error path is tested; 0 <= polls <= 2^30. */
px_status px_set_wait_limit(px_ctx* ctx, int64_t polls);

/* Bytes of scratch px_sparse_coalesce needs for `total_rows` input rows (over
 * all workers) of width `dim` elements.  Depends on nothing else. */
size_t px_coalesce_scratch_bytes(int64_t total_rows, int64_t dim);

/* Bytes of scratch px_partition_rows needs for capacity `cap`. */
size_t px_partition_scratch_bytes(int64_t cap);

/*
 * Sparse gradient aggregation (Fig. 3: gradients of a sparse variable are
 * aggregated by concatenating the workers' arrays; Sec. 3.2: values with the
 * same index are then accumulated).
 *
 *   idx[w]   dev  int64[counts[w]]          row ids of worker w, each in [0, vocab)
 *   val[w]   dev  dtype[counts[w]][dim]     value rows of worker w, row-major, dense rows
 *   counts   host int64[n_workers]          rows per worker (>= 0)
 *   scale         1 for the sum, 1/n_workers for the average over workers (Sec. 4.1)
 *
 * Output, with M = sum of counts and U = number of distinct ids:
 *   out_ids        dev int64[M]       first U entries: the distinct ids, ascending
 *   out_rows       dev float[M][dim]  first U rows: scale * (sum of all value rows with that id)
 *   out_num_unique dev int64[1]       U
 *   out_run_len    dev int32[M]       first U entries: input rows per id; may be NULL
 * Entries past U are unspecified.  Rows are accumulated in double precision in
 * the order of the concatenation (worker 0's rows first) and rounded once, so
 * the result is deterministic.  bf16 values are widened exactly.
 *
 * Limits: 1 <= n_workers <= PX_MAX_SOURCES, M < 2^31, vocab <= 2^32, dim >= 1,
 * bits(n_workers - 1) + bits(max count - 1) <= 32.  Value pointers must be
 * aligned to their element size; 16-byte alignment with dim * sizeof(element)
 * a multiple of 16 selects the fast 128-bit path.  scratch: dev, 256-byte
 * aligned, at least px_coalesce_scratch_bytes(M, dim).  Inputs, outputs and
 * scratch must not overlap.
 */
px_status px_sparse_coalesce(px_ctx* ctx, int n_workers, const int64_t* const* idx,
                             const void* const* val, const int64_t* counts, int64_t dim,
                             px_dtype val_dtype, int64_t vocab, float scale, int64_t* out_ids,
                             float* out_rows, int64_t* out_num_unique, int32_t* out_run_len,
                             void* scratch, size_t scratch_bytes, void* hip_stream);

/*
 * Partitioning of a sparse variable (Sec. 3.2: incoming indices and values
 * are divided into disjoint sets so that aggregation and update run per
 * partition; Sec. 4.3: each piece has its own update).
 *
 *   ids      dev int64[cap]   only the first *num_ids are read
 *   num_ids  dev int64[1]     0 <= *num_ids <= cap
 * Output:
 *   out_shard   dev int32[cap]          shard of ids[k]; may be NULL
 *   out_perm    dev int32[cap]          positions 0..*num_ids-1 grouped by shard, input order
 *                                       kept inside a shard (ascending ids stay ascending)
 *   out_offsets dev int64[num_shards+1] shard p owns out_perm[out_offsets[p] .. out_offsets[p+1])
 * Limits: 1 <= num_shards <= PX_MAX_SHARDS, cap < 2^31.  scratch: dev,
 * 256-byte aligned, at least px_partition_scratch_bytes(cap).
 */
px_status px_partition_rows(px_ctx* ctx, const int64_t* ids, const int64_t* num_ids, int64_t cap,
                            int num_shards, px_hash hash, int32_t* out_shard, int32_t* out_perm,
                            int64_t* out_offsets, void* scratch, size_t scratch_bytes,
                            void* hip_stream);

/*
 * px_partition_rows for callers that can neither allocate device memory nor hand over a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments (without scratch), same kernels, same results bit for bit.  The workspace is
 * an array built into the library, 513 KiB on every GPU it runs on, held until the process
 * ends; its device address is looked up once per GPU, when px_create runs there.  The call
 * allocates and frees nothing.  Limits: cap <= PX_PARTITION_NOALLOC_MAX_IDS (4,194,304 ids; a
 * larger cap is refused with PX_ERR_INVALID_ARG before anything is enqueued: use
 * px_partition_rows).  All contexts on a GPU share that GPU's array: calls of this entry point
 * that overlap on one GPU (two streams, two contexts) race and must be ordered by the caller.
 */
px_status px_partition_rows_noalloc(px_ctx* ctx, const int64_t* ids, const int64_t* num_ids,
                                    int64_t cap, int num_shards, px_hash hash, int32_t* out_shard,
                                    int32_t* out_perm, int64_t* out_offsets, void* hip_stream);

/*
 * Sparse variable update by gradient descent (Fig. 4; Sec. 2.1: gradients are
 * aggregated before they update the variable, so each touched row is updated
 * exactly once; Sec. 4.3: the update runs where the variable lives).
 *   table[ids[k]][:] -= lr * rows[k][:]     for k = perm[j], j in [first, last)
 *
 *   table    dev float[vocab][dim], updated in place; other rows are not touched
 *   ids      dev int64[cap], rows dev float[cap][dim]: the output of px_sparse_coalesce
 *   num_ids  dev int64[1]
 *   perm     dev int32[cap] from px_partition_rows (a permutation of 0 .. *num_ids - 1), or NULL
 *            for the identity
 *   range    dev int64[2] = {first, last} positions of perm to apply (e.g. two
 *            consecutive entries of out_offsets: one shard), or NULL for all *num_ids; every
 *            position is then updated once whatever the order, and perm is not read
 * Precondition: the ids are distinct; rows and table do not overlap.  Two lane groups
 * updating one row would race, so every position whose id equals that of a neighbouring
 * position (k - 1 or k + 1; in a sorted list, such as px_sparse_coalesce's output, every
 * repeat is one) is skipped and raises the context's flag (PX_ERR_NOT_UNIQUE from
 * px_device_status).  The other rows of that call are updated unless their workgroup started
 * after the flag went up (a launch of one workgroup updates all of them).  Repeats that are
 * not adjacent are not detected: the result for those rows is then undefined.
 */
px_status px_sparse_apply_sgd(px_ctx* ctx, float* table, int64_t vocab, int64_t dim,
                              const int64_t* ids, const float* rows, const int64_t* num_ids,
                              int64_t cap, const int32_t* perm, const int64_t* range, float lr,
                              void* hip_stream);

/*
 * Sparse variable update by Adagrad, element-wise on the touched rows:
 *   accum[id] += g*g ;  table[id] -= lr * g / (sqrt(accum[id]) + eps)   (updated accum)
 * The paper's own example uses plain gradient descent (Fig. 4) and leaves the optimizer to the
 * single-GPU graph it transforms (Sec. 4.1); what it fixes is where and when the update runs:
 * once per touched row, from the aggregated gradient, on the partition that owns the row
 * (Sec. 2.1, Sec. 4.3).  The rule itself is Adagrad as published (Duchi et al., 2011) in the
 * form the sparse language-model workloads use: a per-element accumulator of the same shape as
 * the variable, read after it has been increased by g*g, eps added outside the square root.
 * accum: dev float[vocab][dim], same layout as table, updated in place.
 * Other arguments, the precondition and the error behaviour as px_sparse_apply_sgd.
 */
px_status px_sparse_apply_adagrad(px_ctx* ctx, float* table, float* accum, int64_t vocab,
                                  int64_t dim, const int64_t* ids, const float* rows,
                                  const int64_t* num_ids, int64_t cap, const int32_t* perm,
                                  const int64_t* range, float lr, float eps, void* hip_stream);

/*
 * Aggregate and update in one go (Sec. 4.3: the global aggregation is placed on the server that
 * holds the variable, so the aggregated gradient never travels; here it is never written to
 * memory).  Same result as px_sparse_coalesce followed by px_sparse_apply_sgd /
 * px_sparse_apply_adagrad over all rows (perm = NULL, range = NULL), bit for bit: the sum of a
 * run is rounded to float, scaled, and fed to the same update arithmetic.
 * Arguments as in those two calls; there is no out_rows.  out_ids, out_num_unique and
 * out_run_len are still produced (px_partition_rows can run on them afterwards).
 * An id outside [0, vocab) raises the context's flag and leaves table and accum untouched.
 */
px_status px_sparse_coalesce_apply_sgd(px_ctx* ctx, int n_workers, const int64_t* const* idx,
                                       const void* const* val, const int64_t* counts, int64_t dim,
                                       px_dtype val_dtype, int64_t vocab, float scale, float* table,
                                       float lr, int64_t* out_ids, int64_t* out_num_unique,
                                       int32_t* out_run_len, void* scratch, size_t scratch_bytes,
                                       void* hip_stream);

px_status px_sparse_coalesce_apply_adagrad(px_ctx* ctx, int n_workers, const int64_t* const* idx,
                                           const void* const* val, const int64_t* counts, int64_t dim,
                                           px_dtype val_dtype, int64_t vocab, float scale, float* table,
                                           float* accum, float lr, float eps, int64_t* out_ids,
                                           int64_t* out_num_unique, int32_t* out_run_len, void* scratch,
                                           size_t scratch_bytes, void* hip_stream);

/*
 * Dense gradient aggregation (Sec. 2.1: AllReduce computes the sum over the N
 * workers of their gradients; Sec. 4.1: or their average).  This is the
 * reduction one GPU performs on its slice:
 *   out[j] = scale * sum_w bufs[w][j],   j in [0, count)
 *   bufs   host array of n_buffers dev pointers, each in_dtype[count]
 *   out    dev out_dtype[count]; may alias none of the inputs
 * Accumulation is in worker order, in double precision, rounded once.
 * A long output is produced by several kernel launches in a row (px_dense_average_launches says
 * how many): each covers 2^19 16-byte pieces of every buffer, more when there are few buffers,
 * and at most 16 MiB of output.
 * Limits: 1 <= n_buffers <= PX_MAX_SOURCES.  Pointers aligned to the element
 * size; 16-byte alignment selects the 128-bit path.
 */
px_status px_dense_average(px_ctx* ctx, int n_buffers, const void* const* bufs, int64_t count,
                           px_dtype in_dtype, void* out, px_dtype out_dtype, float scale,
                           void* hip_stream);

/* Host only: the number of kernel launches of the 128-bit path px_dense_average makes for these
 * arguments (what a profile of the call shows, and what a per-launch figure divides by); the
 * element-wise kernel for a ragged tail or unaligned buffers is not counted.  0 for an empty call. */
int64_t px_dense_average_launches(int n_buffers, int64_t count, px_dtype in_dtype, px_dtype out_dtype);

/*
 * The pull side of a partitioned sparse variable (Sec. 3.1: workers pull the rows their
 * mini-batch touches; Sec. 3.2: the rows looked up in the partitions are stitched back into
 * one tensor in the order of the request):
 *   out_rows[k][:] = table[ids[k]][:]     for k = perm[j], j in [first, last)
 *   table    dev float[vocab][dim], read only
 *   ids      dev int64[cap], any order, may repeat; num_ids dev int64[1] or NULL (= cap)
 *   perm     dev int32[cap] from px_partition_rows on these ids, or NULL for the identity
 *   range    dev int64[2] = {first, last} (one shard's slice of perm), or NULL for everything
 *   out_rows dev float[cap][dim]; only the rows selected by perm / range are written
 * An id outside [0, vocab) raises the context's flag; its output row is left untouched.
 */
px_status px_sparse_lookup(px_ctx* ctx, const float* table, int64_t vocab, int64_t dim,
                           const int64_t* ids, const int64_t* num_ids, int64_t cap,
                           const int32_t* perm, const int64_t* range, float* out_rows,
                           void* hip_stream);

/*
 * Partition-count cost model (Sec. 3.2, Eq. 1):  iter_time(P) = theta0 + theta1 / P + theta2 * P.
 * Host-only arithmetic in double; all pointers are host pointers; no context, nothing enqueued.
 *
 * px_partition_cost_fit      least-squares fit of theta[3] to n >= 3 samples (p[i] > 0, at least three
 *                            distinct values; PX_ERR_INVALID_ARG otherwise).
 * px_partition_cost_argmin   the integer P in [p_lo, p_hi] with the smallest fitted time (Eq. 1 is
 *                            convex for theta1, theta2 > 0 with critical point sqrt(theta1/theta2));
 *                            best_time may be NULL.
 * px_partition_search_next   the paper's sampling rule: start at p_start, double while the time does
 *                            not go up (never beyond p_max), then halve from p_start while it does not
 *                            go up.  Given the samples taken so far it returns the next P to measure
 *                            in *next_p, or 0 once sampling is complete.
 */
px_status px_partition_cost_fit(const double* p, const double* t, int n, double* theta);
px_status px_partition_cost_argmin(const double* theta, int64_t p_lo, int64_t p_hi, int64_t* best_p,
                                   double* best_time);
px_status px_partition_search_next(const double* p, const double* t, int n, int64_t p_start,
                                   int64_t p_max, int64_t* next_p);

#ifdef __cplusplus
}
#endif
#endif /* PX_H_ */
