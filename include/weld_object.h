/*
 * weld_object.h -- the lazy half of the runtime API (paper Sec. 4.1, Table 2) on top of
 * weld_fused_for: libraries wrap their data and their operators in objects that form a
 * DAG; nothing runs until an object is evaluated; evaluation first FUSES the DAG into one
 * loop over the leaves (loop fusion of Table 3: vertical = a map or filter feeding the
 * next operator, horizontal = several results over the same vectors) and then hands that
 * loop to weld_fused_for.  With conf.mode = WELD_MODE_UNFUSED the same program is run one
 * operator at a time instead.
 *
 * A scalar (a reduce object) may be a dependency of a map (Sec. 4.1: objects depend on other
 * objects; this is how a library normalises a column by its mean).  A loop cannot read what it is
 * still reducing, so evaluation then takes STAGES: the scalars that maps read are computed by
 * earlier fused loops (all scalars of a stage over vectors of one length share one loop; a
 * reduction written twice is computed once), and the loops that read them take them from device
 * memory (WELD_OP_SCALAR), in stream order, with no host wait and no host copy in between.
 *
 *   NewWeldObject(data, type, encoder)  -> weld_object_new_data
 *   NewWeldObject(deps, expr, encoder)  -> weld_object_new_map / _filter / _reduce / _groupby
 *                                          (the macros of Sec. 3.3; encoders are the caller's
 *                                           business: objects deal in raw device pointers)
 *   GetObjectType                       -> weld_object_kind / weld_object_elem_type
 *   Evaluate                            -> weld_object_evaluate (returns a weld_result_t)
 *   FreeWeldObject                      -> weld_object_free (frees this node, not its
 *                                          dependencies, which are reference counted)
 *
 * Objects are host-side values; all functions are thread-compatible, not thread-safe.
 */
#ifndef WELD_OBJECT_H
#define WELD_OBJECT_H

#include "weld_hip.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct weld_object weld_object_t;

typedef enum { WELD_OBJ_VEC = 0, WELD_OBJ_SCALAR = 1, WELD_OBJ_DICT = 2 } weld_object_kind_t;

/* A vector of `len` elements of `type` at DEVICE pointer `data`, owned by the caller, never
 * written, and alive until every evaluation that reaches it has finished. */
weld_status_t weld_object_new_data(const void* data, int32_t type, int64_t len, weld_object_t** out);

/* map(zip(deps), f): f is an SSA list as in weld_body_t.ops (operators up to WELD_OP_SELECT), in
 * which WELD_OP_COL with a = k reads the current element of deps[k] and the LAST op is the value
 * of the new element.  The vector deps must have the same length and have gone through the same
 * filters; a dep may also be a scalar (a reduce object), which WELD_OP_COL then reads as the
 * same value for every element; at least one dep must be a vector. */
weld_status_t weld_object_new_map(weld_object_t* const* deps, int32_t ndeps, const weld_op_t* ops,
                                  int32_t nops, weld_object_t** out);

/* filter(vec, mask): the elements of vec at which the bool vector mask is true, in order. */
weld_status_t weld_object_new_filter(weld_object_t* vec, weld_object_t* mask, weld_object_t** out);

/* reduce(vec, id, func) with func in weld_func_t and id its identity: a scalar. */
weld_status_t weld_object_new_reduce(weld_object_t* vec, int32_t func, weld_object_t** out);

/* group vals by keys and combine with func (a dictmerger): keys integer vectors (<= 64 bits in
 * total), vals numeric vectors, capacity = upper bound on the number of distinct keys. */
weld_status_t weld_object_new_groupby(weld_object_t* const* keys, int32_t nkeys, weld_object_t* const* vals,
                                      int32_t nvals, int32_t func, int64_t capacity, weld_object_t** out);

int32_t weld_object_kind(const weld_object_t* o);      /* weld_object_kind_t, -1 for NULL            */
int32_t weld_object_elem_type(const weld_object_t* o); /* element / scalar type; -1 for dictionaries */

/* Evaluate `nroots` objects together: they must iterate over vectors of one common length.
 * Result i of the handle belongs to roots[i]: a vector root is materialised by a vecbuilder, a
 * scalar root is a merger, a dictionary root a dictmerger.  Returns like weld_fused_for.
 * With stages (see above) every loop is enqueued before the call returns; the handle owns the
 * earlier loops' results, reports the first error among them, counts their kernels and adds
 * their time to weld_result_elapsed_ms(); weld_result_kernel_ms() and _kernel_name() are those
 * of the last loop.  A root that an earlier stage has computed is returned from there. */
weld_status_t weld_object_evaluate(weld_object_t* const* roots, int32_t nroots, const weld_conf_t* conf,
                                   weld_result_t** out);

/* The fused loop that weld_object_evaluate would run, written in the notation of the paper's
 * listings; with stages, the earlier loops first, each as `let {s0, s1} = <loop>`, then the
 * roots' loop, in which s0, s1 are parameters beside the zipped vectors.  Returns the bytes needed including the terminator (negative on error), copies at
 * most buflen.  Needs no GPU. */
int64_t weld_object_describe(weld_object_t* const* roots, int32_t nroots, char* buf, int64_t buflen);

/* Drops the caller's reference; dependencies stay alive while other objects use them. */
void weld_object_free(weld_object_t* o);

#ifdef __cplusplus
}
#endif
#endif /* WELD_OBJECT_H */
