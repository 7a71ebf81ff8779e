/*
 * weld_nested.h -- a `for` nested inside a `for` (Sec. 3.2: loops nest arbitrarily, which is how
 * the IR expresses irregular parallelism such as graph algorithms; the loop's optional start and
 * end index per input vector), run on the GPU by UN-NESTING (Sec. 5, "Partial GPU Backend": a
 * nested parallel program is turned into a regular one) -- the shape of the paper's PageRank
 * workload (Sec. 7.4, 7.5) and of a sparse matrix-vector product over CSR.
 *
 * The program is
 *
 *   result(for(zip(outer...), builders, (bs, i, x) =>
 *       let r = result(for(iter(zip(inner...), x.start, x.end), merger[T, func],
 *                          (b, j, e) => if (p(e, x)) merge(b, f(e, x, lookup(...))) else b));
 *       ... merges of g(x, r, i) into bs ...))
 *
 * i.e. outer element i owns the inner elements [start[i], end[i]) and reduces a function of
 * them with a merger; the outer body then uses that result like any other value.
 *
 * How it runs: the inner loops of all outer elements are flattened into ONE parallel loop over
 * the inner elements (balanced by inner elements, not by outer elements, so one outer element
 * with a million inner elements costs what a million outer elements with one each cost), with a
 * segmented merger that keeps one cell per outer element; a second, ordinary fused loop over the
 * outer elements evaluates the outer body with the cell as one more value.
 *
 * Two kinds of ranges (weld_nested_t.range_kind):
 *   WELD_RANGES_CSR  the ranges are CONSECUTIVE with stride 1: start[0] == 0, end[i] == start[i+1],
 *                    end[n_outer-1] == n_inner (CSR row pointers: pass the pointer array as `start`
 *                    and the same array shifted by one element as `end`).  The flattened loop then
 *                    streams the inner vectors front to back; nothing waits for the host.  Ranges
 *                    that are not of this form make the call fail with WELD_ERR_INVALID_ARG at the
 *                    evaluation point.
 *   WELD_RANGES_ANY  the loop's start, end and STRIDE per vector (Sec. 3.2: how the IR iterates over
 *                    a column of a row-major matrix): outer element i visits start[i], start[i] +
 *                    stride[i], ... below end[i]; ranges may overlap, leave gaps and be empty.  A
 *                    small kernel turns the ranges into element counts and their prefix sums, the
 *                    flattened loop runs over those positions and reads inner element
 *                    start[i] + k * stride[i] for the k-th of them (a gather instead of a stream).
 *                    Its size is the total count, so the call waits for that kernel before it
 *                    enqueues the rest; start < 0, end < start, end > n_inner or stride < 1 make it
 *                    fail with WELD_ERR_INVALID_ARG there and then.
 * In an inner body WELD_OP_INDEX is the position of the element in the inner vectors.
 */
#ifndef WELD_NESTED_H
#define WELD_NESTED_H

#include "weld_hip.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Extra operators of the two bodies (values continue weld_opcode_t). */
enum {
    WELD_OP_LOOKUP = 26, /* inner body: lookup(gather[a], t_b): element t_b (an integer value) of
                            gather vector a; an index outside the vector fails the call          */
    WELD_OP_OUTER = 27,  /* inner body: a = outer column: the CURRENT OUTER element of that vector */
    WELD_OP_INNER = 28   /* outer body: the result of this outer element's inner loop            */
};

enum { WELD_RANGES_CSR = 0, WELD_RANGES_ANY = 1 };

typedef struct {
    int64_t n_outer;            /* outer elements, >= 0                                           */
    weld_cols_t outer;          /* zipped outer vectors: device pointers to n_outer elements      */
    int32_t start_col, end_col; /* outer columns (WELD_I32 or WELD_I64, same type) holding each
                                   outer element's inner range [start, end)                      */
    int64_t n_inner;            /* inner elements, >= 0                                           */
    weld_cols_t inner;          /* zipped inner vectors: device pointers to n_inner elements      */
    int32_t ngather;            /* vectors readable at computed positions (WELD_OP_LOOKUP), <= 8  */
    const weld_col_t* gather;   /* host array; device pointers, never written                     */
    const int64_t* gather_len;  /* host array: elements of each gather vector                     */
    weld_body_t inner_body;     /* WELD_OP_COL reads inner column a; exactly one merge, into
                                   builder 0 = the inner merger                                  */
    int32_t inner_type;         /* T of the inner merger: WELD_I64 or WELD_F64                    */
    int32_t inner_func;         /* weld_func_t                                                    */
    weld_body_t outer_body;     /* WELD_OP_COL reads outer column a; merges go to `builders`      */
    int32_t range_kind;         /* WELD_RANGES_CSR (0) or WELD_RANGES_ANY                         */
    int32_t stride_col;         /* WELD_RANGES_ANY: outer column (type of start / end) holding each
                                   range's stride, or -1 for stride 1; ignored for WELD_RANGES_CSR */
} weld_nested_t;

/* Runs the nested loop above.  `builders` are the OUTER loop's builders (any kind
 * weld_fused_for takes) and carry the configuration; `out` is a handle like weld_fused_for's,
 * with one result per outer builder.  Enqueues on conf.stream and returns; every vector must
 * stay alive and unmodified until weld_result_status() has returned.  Errors found on the
 * device (WELD_RANGES_CSR ranges that are not consecutive, a lookup outside its vector) are
 * reported by weld_result_status() as WELD_ERR_INVALID_ARG.  weld_result_kernel_ms() times the flattened
 * inner loop; weld_result_elapsed_ms() the whole call. */
weld_status_t weld_nested_for(const weld_nested_t* loop, const weld_builder_t* builders, weld_result_t** out);

/* Validation only (no GPU needed); err/errlen: optional buffer for the message. */
weld_status_t weld_nested_validate(const weld_nested_t* loop, const weld_builder_t* builders, char* err, size_t errlen);

/* Compile (or load from the on-disk cache) the two kernels of this nested loop without running
 * them and without touching a GPU.  Device pointers inside `loop` are ignored. */
weld_status_t weld_nested_precompile(const weld_nested_t* loop, const weld_builder_t* builders);

#ifdef __cplusplus
}
#endif
#endif /* WELD_NESTED_H */
