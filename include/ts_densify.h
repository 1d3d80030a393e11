/*
 * ts_densify -- densify an assumed-sparse gradient on one MI355X (gfx950).
 *
 * The operation (arXiv 1905.04035): a transformer whose embedding matrix is shared
 * with the pre-softmax projection receives, for that one [V, d] weight, sparse
 * gradients from the encoder and decoder embedding lookups (one (id, row) slice
 * per looked-up token, ids repeat) and one dense [V, d] gradient from the
 * projection (Section 3).  Section 4, Listing 1 converts each sparse gradient to a
 * dense tensor so that a fixed-size reduce replaces an ever-growing gather;
 * Section 6, Algorithm 2 (the added branch) converts every gradient to dense and
 * sums them.  These entry points compute exactly that sum:
 *
 *     dense_out[v, :] = dense_in[v, :] + sum over pairs t with ids[t] == v of rows[t, :]
 *
 * Conventions common to all calls
 *   - Pointers named ids, rows, dense_in, dense_out and the workspace are DEVICE
 *     pointers owned by the caller.  The library never frees them and does not
 *     keep them after the work it enqueued on `stream` has run.  Arrays named *_k
 *     and every out-parameter of a query are HOST pointers.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Work
 *     is enqueued; no call synchronises the host or allocates device memory.
 *   - Layout: ids int32 [n]; rows [n, d] row-major, fp32 or bf16 bit patterns;
 *     dense_in / dense_out fp32 [V, d] row-major.  rows, dense_in and dense_out
 *     must be 16-byte aligned and d must be a multiple of 4.
 *   - dense_in == NULL means "no dense operand" (Listing 1 alone): rows that
 *     receive no pair are +0.0.  dense_out == dense_in (the same pointer) is
 *     allowed and updates in place; any other overlap is undefined.
 *   - Rows that receive no pair are copied from dense_in bit for bit.
 *   - A pair whose id is outside [0, V) is skipped, never dereferenced, and
 *     counted; the count is visible through ts_last_views (n_bad_ids).
 *   - Sums are fp32.  Within one output row the pairs are added in input order
 *     inside fixed-size pieces, the pieces are combined in a fixed order and
 *     dense_in is added last; no floating-point atomics are used, so the same
 *     inputs give the same bits on every run.
 *   - Return value: TS_OK or a ts_status; it covers only what the host can check
 *     (arguments, workspace, launch errors).
 *   - One call at a time per process: calls share the bound workspace, and the library
 *     remembers which workspace and shapes the most recent call used (for ts_last_views and
 *     ts_unique_ids).  The calls declared in ts_densify_tools.h (tests, benchmarks, tuning)
 *     change process-wide settings; none of them is needed to use the library.
 */
#ifndef TS_DENSIFY_H
#define TS_DENSIFY_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    TS_OK = 0,
    TS_ERR_NULL = 1,      /* a required pointer is NULL */
    TS_ERR_SHAPE = 2,     /* n < 0, V <= 0, d <= 0, d % 4 != 0, k out of range, unknown dtype */
    TS_ERR_ALIGN = 3,     /* rows / dense_in / dense_out not 16-byte aligned */
    TS_ERR_WORKSPACE = 4, /* no workspace bound, or it is too small for this call */
    TS_ERR_HIP = 5,       /* the HIP runtime reported an error (launch, event) */
    TS_ERR_OVERFLOW = 6,  /* a size does not fit (n_total >= 2^31, byte count overflow) */
    TS_ERR_CAPACITY = 7   /* an output buffer is too small for what the call would write */
} ts_status;

enum { TS_ROW_FP32 = 0, TS_ROW_BF16 = 1 };

/* Largest k accepted by ts_densify_multi (shard descriptors travel as kernel arguments). */
#define TS_MAX_SHARDS 64

/*
 * Densify one sparse gradient with fp32 value rows and add the dense one
 * (Section 4, Listing 1; Section 6, Algorithm 2, added branch).
 * n may be 0 (then dense_out = dense_in, or zeros).
 */
int ts_densify(const int32_t* ids, const float* rows, int64_t n, int32_t d, int32_t V,
               const float* dense_in, float* dense_out, void* stream);

/*
 * ts_densify for callers that cannot allocate device memory or bind a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, same kernels, same bits as ts_densify; the workspace is an array built into
 * the library's device image, TS_STATIC_SCRATCH_BYTES per GPU, held by every GPU the
 * library is loaded on until the process ends.  The call allocates and frees nothing and
 * ignores the bound workspace.  It serves the calls whose own workspace fits the array
 * (V = 32768, d = 1024: up to about 150 thousand pairs; ts_workspace_bytes(n, d, V) <=
 * TS_STATIC_SCRATCH_BYTES is sufficient); a larger call returns TS_ERR_CAPACITY before
 * anything is enqueued.  Every call on a GPU uses that GPU's one array: two such calls that
 * overlap in time on one GPU (two streams, two threads) race; calls on one stream do not.
 * Nothing in the array has to survive from call to call, and each call clears what it
 * needs cleared.  ts_last_views afterwards describes this call.
 */
#define TS_STATIC_SCRATCH_BYTES (16 << 20)
int ts_densify_static(const int32_t* ids, const float* rows, int64_t n, int32_t d, int32_t V,
                      const float* dense_in, float* dense_out, void* stream);

/* Same as ts_densify, value rows stored as bf16 bit patterns; they are widened exactly and summed in fp32. */
int ts_densify_bf16(const int32_t* ids, const uint16_t* rows, int64_t n, int32_t d, int32_t V,
                    const float* dense_in, float* dense_out, void* stream);

/*
 * Densify k contributions at once: the result is that of ts_densify on their
 * concatenation in shard order (Section 3: under the gather strategy the
 * accumulate buffer is the concatenation of every worker's slices).
 * ids_k[j], rows_k[j] (device pointers) and n_k[j] describe shard j; the three
 * arrays themselves are host arrays of length k, read before the call returns.
 * 1 <= k <= TS_MAX_SHARDS; shards may be empty and of different lengths; a
 * contiguous gathered buffer is the case k = 1.  row_dtype is TS_ROW_FP32 or
 * TS_ROW_BF16 for all shards.
 */
int ts_densify_multi(const int32_t* const* ids_k, const void* const* rows_k, const int64_t* n_k,
                     int32_t k, int32_t row_dtype, int32_t d, int32_t V,
                     const float* dense_in, float* dense_out, void* stream);

enum { TS_OUT_FP32 = 0, TS_OUT_BF16 = 1 };

/*
 * ts_densify_multi with a write-back epilogue, for a result that goes straight into the
 * buffer a dense reduction will read (Section 4: after the conversion the gradient is
 * accumulated by reduction; Section 5, runtime settings: the experiments give the
 * reduction a fusion buffer of 134217728 bytes, the size of a [32768, 1024] fp32 tensor;
 * Section 1 names reduced precision as the other way to cut the exchange):
 *
 *     out[v,:] = cast( scale * (dense_in[v,:] + sum of the value rows with id v) )
 *
 * scale is one finite fp32 factor (1/k turns the sum over k workers into their average;
 * infinite or NaN: TS_ERR_SHAPE).  The sum is formed in fp32 exactly as by
 * ts_densify_multi, multiplied once in fp32, then stored as fp32 (TS_OUT_FP32) or rounded
 * to bf16, nearest with ties to even (TS_OUT_BF16: out holds V*d uint16 bit patterns and
 * half the bytes are written).  Untouched rows are scale * dense_in, rounded the same way.
 * With TS_OUT_FP32 and scale == 1 the call is ts_densify_multi, bit for bit.
 * out is a device pointer, 16-byte aligned, e.g. fusion buffer + the offset that
 * ts_fusion_place returns.  out == dense_in is allowed for TS_OUT_FP32 only (TS_OUT_BF16:
 * TS_ERR_SHAPE); other overlaps are undefined.  Everything else as for ts_densify_multi.
 */
int ts_densify_scaled(const int32_t* const* ids_k, const void* const* rows_k, const int64_t* n_k,
                      int32_t k, int32_t row_dtype, int32_t d, int32_t V,
                      const float* dense_in, void* out, int32_t out_dtype, float scale, void* stream);

/*
 * The share of one owner when the vocabulary is split among owners: only rows
 * [v_begin, v_end) of the [V, d] result are produced (Section 3: under the gather strategy
 * every worker receives every worker's slices; an owner of a range of rows then needs only
 * the pairs that name its rows.  Section 6, Algorithm 2: those are converted and summed
 * onto its slice of the dense gradient).  dense_in (or NULL) and dense_out point to that
 * slice, [v_end - v_begin, d] fp32; row v of the vocabulary is row v - v_begin of the slice.
 * Pairs with an id in [0, V) outside the range are skipped without being counted as bad;
 * ids outside [0, V) are skipped and counted.  After the call ts_last_views describes the
 * slice: count and row_start have v_end - v_begin (+ 1) entries, n_valid is the number of
 * pairs inside the range, so n_total - n_valid - n_bad_ids pairs belonged to other owners.
 * 0 <= v_begin < v_end <= V, else TS_ERR_SHAPE.  The workspace is sized for
 * ts_workspace_bytes(n_total, d, v_end - v_begin).  Everything else as for
 * ts_densify_multi, which is the case v_begin = 0, v_end = V.
 */
int ts_densify_range(const int32_t* const* ids_k, const void* const* rows_k, const int64_t* n_k,
                     int32_t k, int32_t row_dtype, int32_t d, int32_t V, int32_t v_begin, int32_t v_end,
                     const float* dense_in, float* dense_out, void* stream);

/*
 * Host arithmetic, no GPU: where a [V, d] result of out_dtype goes in a fusion buffer of
 * capacity_bytes of which used_bytes are taken.  *offset_bytes = used_bytes rounded up to
 * 256; *used_after_bytes = offset + 4*V*d (2*V*d for bf16).  TS_ERR_CAPACITY if that
 * exceeds the capacity (nothing is written then), TS_ERR_OVERFLOW if a size overflows.
 */
int ts_fusion_place(int64_t capacity_bytes, int64_t used_bytes, int32_t d, int32_t V, int32_t out_dtype,
                    int64_t* offset_bytes, int64_t* used_after_bytes);

/*
 * The two accumulation rules of the paper, for the gradients that one variable receives.
 *
 * Section 3, Algorithm 1 (TensorFlow's rule, TS_RULE_TF): fewer than two gradients pass
 * through; if all are dense tensors they are summed (reduce); otherwise all are turned
 * into indexed slices and concatenated (gather) -- a dense [V, d] tensor becomes V
 * slices with ids 0 .. V-1.  Section 6, Algorithm 2 (TS_RULE_PROPOSED) adds a branch
 * before the gather: if any gradient is a dense tensor, all are converted to dense
 * tensors and summed, which is ts_densify_multi onto the (sum of the) dense one(s).
 *
 * ts_accumulate_strategy only tells which branch the rule takes (host logic).
 * ts_accumulate runs it on `stream`:
 *   - TS_ACC_REDUCE, TS_ACC_DENSIFY_REDUCE and a passed-through dense gradient write
 *     dense_out fp32 [V, d] (device; fp32 sums, dense gradients added in list order,
 *     converted slices as in ts_densify).  TS_ACC_DENSIFY_REDUCE needs the workspace
 *     bound for the total number of pairs and at most TS_MAX_SHARDS slice gradients.
 *   - TS_ACC_GATHER and a passed-through slices gradient write ids_out int32 [total]
 *     and rows_out fp32 [total, d] (device), the gradients' slices in list order, and
 *     total to *n_slices_out (host); total > slice_capacity gives TS_ERR_CAPACITY
 *     before anything is written.
 * Outputs the taken branch does not write may be NULL.  *strategy_out (host, may be
 * NULL) receives the branch.  grads is a host array of m >= 1 descriptors; value rows
 * and dense tensors are fp32, 16-byte aligned, and must not overlap the outputs
 * (except that a single dense gradient may be dense_out itself).
 */
typedef struct {
    int32_t kind;          /* TS_GRAD_DENSE or TS_GRAD_SLICES */
    int32_t reserved;
    const int32_t* ids;    /* slices: device int32 [n]; dense: ignored */
    const float* values;   /* slices: device rows [n, d]; dense: device [V, d] */
    int64_t n;             /* slices: number of pairs; dense: ignored */
} ts_grad;

enum { TS_GRAD_DENSE = 0, TS_GRAD_SLICES = 1 };
enum { TS_RULE_TF = 1, TS_RULE_PROPOSED = 2 };
enum { TS_ACC_PASS_THROUGH = 0, TS_ACC_REDUCE = 1, TS_ACC_DENSIFY_REDUCE = 2, TS_ACC_GATHER = 3 };

int ts_accumulate_strategy(const ts_grad* grads, int32_t m, int32_t rule, int32_t* strategy_out);
int ts_accumulate(const ts_grad* grads, int32_t m, int32_t rule, int32_t d, int32_t V,
                  float* dense_out, int32_t* ids_out, float* rows_out, int64_t slice_capacity,
                  int64_t* n_slices_out, int32_t* strategy_out, void* stream);

/*
 * Bytes of the two accumulate buffers the paper compares (Section 4, Fig. 5a):
 * gathered = k * N * (4 + elem * d) for k workers of N slices each (int32 id plus
 * d values of elem bytes), dense = 4 * V * d whatever k is.  Pure host arithmetic.
 */
int ts_buffer_bytes(int64_t k, int64_t N, int32_t d, int32_t V, int32_t row_dtype,
                    int64_t* gathered_bytes, int64_t* dense_bytes);

/*
 * Workspace.  The caller allocates device memory (256-byte aligned) of at least
 * ts_workspace_bytes(n_total, d, V) and binds it once; every later call with
 * n <= n_total and d, V no larger reuses it.  Its contents need no initialisation.
 * The library holds the pointer until another workspace is bound (ws == NULL
 * unbinds); a call that needs more than the bound bytes returns TS_ERR_WORKSPACE.
 */
int ts_workspace_bytes(int64_t n_total, int32_t d, int32_t V, int64_t* bytes);
int ts_bind_workspace(void* ws, int64_t bytes);

/*
 * Views into the bound workspace describing the most recent densify call, valid
 * (in stream order) until the next one: count int32 [V] pairs per row,
 * row_start int32 [V + 1] exclusive prefix of count, sorted [n_valid] records of
 * TS_SORTED_PAIR_BYTES bytes each, in (id, input position) order, whose int32 words
 * 2 and 3 are the pair's id and its position in the input, n_valid and n_bad_ids
 * int32 scalars.  Any out-pointer may be NULL.  All returned pointers are device
 * pointers.
 */
#define TS_SORTED_PAIR_BYTES 32
int ts_last_views(const int32_t** count, const int32_t** row_start, const void** sorted,
                  const int32_t** n_valid, const int32_t** n_bad_ids);

/*
 * Ascending list of the rows that received at least one pair in the most recent
 * call: writes unique_ids_out[0 .. n_unique) (device, capacity >= min(n, V)
 * int32) and *n_unique_out (device int32).  Enqueues one small kernel.
 */
int ts_unique_ids(int32_t* unique_ids_out, int32_t* n_unique_out, void* stream);

const char* ts_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* TS_DENSIFY_H */
