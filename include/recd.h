/*
 * recd.h — C ABI of the MI355X (gfx950) deduplicated-embedding hot path of RecD.
 *
 * The path (paper Sec. 4.2 "Tensor Encoding for Deduplication", Sec. 5 "RecD in Training"):
 *   1. KJT -> IKJT        deduplicate identical per-sample lists of every sparse feature of a batch
 *   2. pooled lookup      sum-pooled embedding-bag lookup on the unique lists only
 *   3. expand             index_select of the pooled rows through the per-sample inverse index
 *   4. backward           gradient of 3 and 2 (+ optional row-wise Adagrad on the touched rows)
 *   5. KJT pooled lookup  the non-deduplicated comparison path
 * and, for sequence (unpooled) features (Sec. 5 "EMB Inputs and Activations", "Jagged Index Select"):
 *   6. sequence lookup    one activation row per id of the unique lists
 *   7. jagged expand      index select of whole unique lists back into the KJT's jagged layout
 *   8. KJT sequence lookup, the non-deduplicated comparison path
 * and for feature groups that share one inverse index (Sec. 4.2 "Grouped IKJTs"):
 *   9. grouped builder    10. element-wise sum over a group's features on the unique rows
 * other pooling functions (11), and partial IKJTs whose lists share storage when one continues
 * another (Sec. 7): 12. partial builder   13. pooled lookup on the windows
 *   14. backward of the sequence path   15. backward of the averaged pooled lookup
 *   16-19. per-id weights: builder, unique and KJT lookups, backward
 *   20. backward of the max-pooled lookup   21, 22. the backward in two halves (plan / apply)
 *   23, 24. run index of a batch (adjacent rows holding one list)   25. lookup and expand in one pass
 *   26. the backward's plan from the run index
 *
 * General rules
 *   - Every array argument marked "device" is a pointer into GPU memory owned by the caller and
 *     valid on the context's device; "host" arguments are ordinary host memory read during the
 *     call.  The library never allocates anything the caller sees and never frees caller memory.
 *   - Calls enqueue kernels on the context's HIP stream and return without synchronising, except
 *     where stated (host result requested, validation enabled).  Inputs are never modified;
 *     embedding tables and optimizer state are modified only by the optimizer branch of
 *     recd_backward_dedup.
 *   - Every call returns a recd_status; nothing throws or aborts.  On failure
 *     recd_last_error(ctx) holds a message.  F = 0, B = 0 and N = 0 are valid (no-op) sizes.
 *   - Preconditions (offsets[0] = 0, offsets non-decreasing, offsets[F*B] = N, ids within the
 *     table, inverse entries within [0, U_f)) are checked on the device only when RECD_OPT_VALIDATE is set (the call then
 *     synchronises and returns RECD_EBOUNDS without running the operation); otherwise behaviour
 *     for inputs that violate them is undefined.
 *   - One context serves one stream; calls on one context must not overlap (they share its
 *     workspace).  Use one context per stream.
 *
 * Data layout
 *   KJT (Sec. 4.2):   values  int64 [N], feature-major (all rows of feature 0, then feature 1, ...)
 *                     offsets int64 [F*B+1]; offsets[f*B+b] = start of row b of feature f in
 *                     values; one trailing sentinel offsets[F*B] = N (the paper's offsets slice is
 *                     the first F*B entries; it derives the last length from |values|).
 *   IKJT (Sec. 4.2):  u_values  int64 [M]    unique lists, feature-major, within a feature in order of
 *                                            first occurrence in the batch
 *                     u_offsets int64 [U+1]  start of unique list u in u_values, sentinel u_offsets[U] = M
 *                     inverse   int32 [F*B]  inverse[f*B+b] in [0, U_f): slot of row b among feature
 *                                            f's unique lists (the paper's inverse_lookup)
 *                     feat_uoff int64 [F+1]  prefix sum of U_f; unique list of (f,b) is
 *                                            feat_uoff[f] + inverse[f*B+b]; feat_uoff[F] = U
 *   Every feature is its own deduplication group.  Ids are stored as int64 and must lie in [0, 2^31).
 *   Tables: row-major [rows_f, D]; pooled / expanded outputs: row-major [lists, D].
 */
#ifndef RECD_H
#define RECD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct recd_ctx recd_ctx; /* opaque: stream, device workspace, error text */

typedef enum {
    RECD_OK = 0,
    RECD_EINVAL = -1,    /* bad argument (null pointer, negative size, unsupported D or dtype)  */
    RECD_ENOMEM = -2,    /* workspace allocation failed                                        */
    RECD_EHIP = -3,      /* a HIP runtime call failed; message holds the HIP error string       */
    RECD_EBOUNDS = -4,   /* validation found an id outside its table or a malformed index        */
    RECD_ECAPACITY = -5  /* a caller-provided capacity is too small for the result               */
} recd_status;

typedef enum { RECD_F32 = 0, RECD_F16 = 1, RECD_BF16 = 2 } recd_dtype;

/* Pooling functions of an embedding bag (Sec. 2.2 names average, sum and max). */
typedef enum { RECD_POOL_SUM = 0, RECD_POOL_MEAN = 1, RECD_POOL_MAX = 2 } recd_pooling;

typedef enum {
    RECD_OPT_VALIDATE = 1,  /* value != 0: check preconditions on the device before each operation  */
    RECD_OPT_WEAK_HASH = 2, /* test hook, value != 0: the builder hashes a list to its length only,
                               so that unequal lists collide constantly and only the exact list
                               comparison keeps them apart.  Results must not change.            */
    RECD_OPT_LONG_SEGMENT_CUT = 4 /* backward, step "sum per table row": a table row named by more
                               than this many entries of the unique lists is summed in chunks by
                               whole blocks instead of by one lane group.  16, 32 (default), 64 or
                               128.  The cut is part of how such a row's sum is associated, so the
                               low bits of its gradient depend on this option (and on nothing else
                               the caller passes); larger values suit batches without duplication,
                               where most of the work is in long rows.                            */
} recd_option;

/* Largest number of features per call and largest row size in bytes (D * element size). */
#define RECD_MAX_FEATURES 1024
#define RECD_MAX_ROW_BYTES 4096

/* Create a context bound to `device` and to `hip_stream` (a hipStream_t passed as void*; NULL =
 * the default stream).  `workspace_hint_bytes` pre-allocates the device workspace (0 = grow on
 * demand; growth synchronises the stream and reallocates).  Besides the workspace a context keeps
 * the hash tables of calls 1 and 16 (8 bytes for each of F * cap slots, cap = the power of two that
 * holds 2 * B): allocated by the first such call of a size, which synchronises the stream, and
 * held until recd_destroy.  The context is owned by the caller and released with recd_destroy. */
recd_status recd_create(recd_ctx **out, int device, void *hip_stream, size_t workspace_hint_bytes);
recd_status recd_destroy(recd_ctx *ctx);
recd_status recd_set_option(recd_ctx *ctx, recd_option opt, int64_t value);
/* Message of the last failing call on this context ("" if none). Valid until the next call. */
const char *recd_last_error(const recd_ctx *ctx);
const char *recd_status_string(recd_status s);
/* Upper bound of the workspace any call needs for these sizes (N = ids in the KJT). */
recd_status recd_workspace_bytes(int F, int64_t B, int64_t N, int D, size_t *out_bytes);

/* 1. KJT -> IKJT (Sec. 4.2 "InverseKeyedJaggedTensor": rows holding exactly the same list — same
 *    length, same ids, same order — share one stored copy; inverse_lookup[i] points at the entry
 *    of the deduplicated offsets for row i).  Duplicates are searched over the whole batch, per
 *    feature.  Unique lists are numbered in order of first occurrence, which makes the result
 *    canonical: independent of hashing and of thread scheduling.
 *    values [N], offsets [F*B+1]: device, read-only.
 *    u_values: device, capacity N.  u_offsets: device, capacity F*B+1.  inverse: device [F*B].
 *    feat_uoff: device [F+1].  Entries of u_values / u_offsets beyond M / U+1 are left untouched.
 *    host_U_M: optional host int64[2]; if non-NULL the call waits for the build and stores U and M
 *    there.  If NULL the build publishes them when it finishes on the GPU and
 *    recd_last_ikjt_counts returns them later.
 *    A batch of at most 1024 rows per feature, 256 features and 2^20 ids is built by one kernel
 *    launch (same outputs).  Its blocks exchange their counts once, with a bounded wait; should a
 *    wait ever expire, the outputs are unspecified and the error is reported as RECD_EHIP where U
 *    and M are handed over: by this call if host_U_M is given, else by recd_last_ikjt_counts. */
recd_status recd_build_ikjt(recd_ctx *ctx, int F, int64_t B, int64_t N,
                            const int64_t *values, const int64_t *offsets,
                            int64_t *u_values, int64_t *u_offsets, int32_t *inverse,
                            int64_t *feat_uoff, int64_t *host_U_M);

/* 2. Sum-pooled lookup on the unique lists (Sec. 5 "EMB Lookups", "Deduplicated Pooling"):
 *    pooled[u,:] = sum over the ids j of unique list u of table_f[u_values[j],:], fp32 accumulation,
 *    rounded once to out_dt.  An empty list pools to zero.
 *    tables: HOST array of F device pointers, table f is [rows[f], D] of table_dt.
 *    rows: HOST int64 [F] (used by validation only, may be NULL when validation is off).
 *    u_values, u_offsets, feat_uoff: device (outputs of recd_build_ikjt).
 *    max_lists: the host's bound or estimate of U (F*B always bounds it).  It sizes the launch only:
 *    the kernel reads U on the device and every block strides until all lists are done, so any
 *    positive value gives the same result (an estimate near U gives the best launch shape); with
 *    validation on it is also checked as the capacity of pooled.  pooled: device [U, D] of out_dt;
 *    the caller provides room for U rows (F*B when U is not known yet).
 *    D*sizeof(element) must be a multiple of 16 and at most RECD_MAX_ROW_BYTES for both dtypes.
 *    out_dt must be table_dt or RECD_F32. */
recd_status recd_pooled_lookup_unique(recd_ctx *ctx, int F, int D, recd_dtype table_dt,
                                      recd_dtype out_dt, const void *const *tables,
                                      const int64_t *rows, const int64_t *u_values,
                                      const int64_t *u_offsets, const int64_t *feat_uoff,
                                      int64_t max_lists, void *pooled);

/* 3. Expand through the inverse index (Sec. 5 "Jagged Index Select", dense pooled case):
 *    out[f,b,:] = pooled[feat_uoff[f] + inverse[f*B+b], :].  A pure copy (bit-exact).
 *    pooled: device [U, D] of dt; out: device [F, B, D] of dt. */
recd_status recd_expand_inverse(recd_ctx *ctx, int F, int64_t B, int D, recd_dtype dt,
                                const void *pooled, const int64_t *feat_uoff,
                                const int32_t *inverse, void *out);

/* 4. Comparison path: the same pooled lookup over every row of the KJT, no deduplication
 *    (Sec. 5 "EMB Lookups", the pre-RecD behaviour).  out: device [F, B, D] of out_dt.
 *    The summation order of a list depends on the list alone, so out equals the result of calls
 *    1-3 bit for bit.  values may be NULL when every list is empty. */
recd_status recd_kjt_pooled_lookup(recd_ctx *ctx, int F, int64_t B, int D, recd_dtype table_dt,
                                   recd_dtype out_dt, const void *const *tables,
                                   const int64_t *rows, const int64_t *values,
                                   const int64_t *offsets, void *out);

/* 5. Backward of calls 3 and 2 (chain rule; Sec. 2.2 names the EMB update of the backward pass,
 *    Sec. 6.2 "Accuracy" states that an IKJT carries the same logical data as the KJT):
 *      g_u[u,:] = sum over rows b (ascending) with inverse[f*B+b] = u of grad_out[f,b,:]
 *      G_f[r,:] = sum over the positions j (ascending) of feature f's unique ids with
 *                 u_values[j] = r of g_u[list of j, :]
 *    computed as stable radix sorts followed by segment sums in sorted order: no floating-point
 *    atomics, bit-identical from run to run.  (How the sum of a table row with many entries is
 *    associated depends on its number of entries and on RECD_OPT_LONG_SEGMENT_CUT; on nothing
 *    else: in particular not on the bounds U_cap and M_cap.)
 *    grad_out: device fp32 [F, B, D].  rows: HOST int64 [F] table sizes (bounds the sort key).
 *    U_cap, M_cap: host upper bounds of U and M (F*B and N always are; the exact values, as
 *    returned by recd_build_ikjt, avoid idle work).
 *    touched_rows: device int64, capacity M_cap: per feature the ascending distinct ids.
 *    feat_roff: device int64 [F+1] prefix sum of the per-feature distinct counts R_f.
 *    grad_rows: device fp32 [R, D], capacity M_cap rows, aligned with touched_rows.  May be NULL
 *    when the optimizer is on and F <= 128: the gradient rows are then consumed by the update
 *    from registers and never stored.
 *    Optimizer (this build's reading, not in the paper): if tables != NULL, row-wise Adagrad is
 *    applied once per touched row with the aggregated gradient:
 *      m[r] += mean_d G[r,d]^2 ;  W[r,d] -= lr * G[r,d] / (sqrt(m[r]) + eps)
 *    tables: HOST array of F device pointers to fp32 [rows_f, D], updated in place;
 *    adagrad_state: HOST array of F device pointers to fp32 [rows_f], updated in place.
 *    Each feature needs a table and an accumulator array of its own: repeated pointers in either
 *    array are refused (RECD_EINVAL), since the rows of different features are updated at the
 *    same time.
 *    host_R: optional host int64[1]; if non-NULL the call synchronises and stores R. */
recd_status recd_backward_dedup(recd_ctx *ctx, int F, int64_t B, int D, const float *grad_out,
                                const int32_t *inverse, const int64_t *feat_uoff,
                                const int64_t *u_values, const int64_t *u_offsets,
                                const int64_t *rows, int64_t U_cap, int64_t M_cap,
                                int64_t *touched_rows,
                                int64_t *feat_roff, float *grad_rows, void *const *tables,
                                float *const *adagrad_state, float lr, float eps,
                                int64_t *host_R);

/* 6. Unpooled lookup on the unique lists (Sec. 2.2: an EMB yields one activation vector per list
 *    element; Sec. 5 "EMB Inputs and Activations": with an IKJT only the unique values are looked
 *    up, which shrinks the activations by the deduplication factor):
 *      emb[j,:] = table_f[u_values[j],:]   for every position j of feature f's unique lists,
 *    i.e. j in [u_offsets[feat_uoff[f]], u_offsets[feat_uoff[f+1]]).  A copy (exact, also when a
 *    16-bit table is widened to out_dt = RECD_F32).
 *    tables, rows, u_values, u_offsets, feat_uoff, max_lists: as in call 2.
 *    M_cap: host upper bound of M (N always is).  emb: device [M, D] of out_dt, capacity M_cap
 *    rows; rows at and beyond M are left untouched, positions at and beyond M_cap are not written.
 *    D*sizeof(table element) must be a multiple of 16 and at most RECD_MAX_ROW_BYTES. */
recd_status recd_sequence_lookup_unique(recd_ctx *ctx, int F, int D, recd_dtype table_dt,
                                        recd_dtype out_dt, const void *const *tables,
                                        const int64_t *rows, const int64_t *u_values,
                                        const int64_t *u_offsets, const int64_t *feat_uoff,
                                        int64_t max_lists, int64_t M_cap, void *emb);

/* 7. Jagged index select (Sec. 5 "Jagged Index Select": IKJT -> KJT for unpooled activations, on
 *    the jagged data itself instead of padding it to dense for index_select):
 *      out[offsets[f*B+b] + t, :] = emb[u_offsets[feat_uoff[f] + inverse[f*B+b]] + t, :]
 *    for t in [0, offsets[f*B+b+1] - offsets[f*B+b]).  A pure copy (bit-exact).
 *    emb: device [M, D] of dt, M_cap = its capacity in rows (reads are clamped to it).
 *    u_offsets, feat_uoff, inverse: device, the IKJT; offsets: device [F*B+1], the KJT's offsets.
 *    out: device [N, D] of dt, the KJT's own jagged layout.  F*B and N must stay below 2^31.
 *    Precondition (checked under RECD_OPT_VALIDATE): the slot of every row holds a list of the
 *    row's length. */
recd_status recd_jagged_expand_inverse(recd_ctx *ctx, int F, int64_t B, int64_t N, int D,
                                       recd_dtype dt, const void *emb, int64_t M_cap,
                                       const int64_t *u_offsets, const int64_t *feat_uoff,
                                       const int32_t *inverse, const int64_t *offsets, void *out);

/* 8. Comparison path: the unpooled lookup over every id of the KJT, no deduplication
 *    (Sec. 2.2; the pre-RecD behaviour): out[j,:] = table_f[values[j],:] for the positions j of
 *    feature f's rows.  out: device [N, D] of out_dt.  Equals the result of calls 1, 6, 7 bit for
 *    bit. */
recd_status recd_kjt_sequence_lookup(recd_ctx *ctx, int F, int64_t B, int64_t N, int D,
                                     recd_dtype table_dt, recd_dtype out_dt,
                                     const void *const *tables, const int64_t *rows,
                                     const int64_t *values, const int64_t *offsets, void *out);

/* 9. KJT -> grouped IKJT (Sec. 4.2 "Grouped IKJTs": several features deduplicated within one
 *    IKJT share one inverse_lookup; rows whose features are not all duplicates together are not
 *    deduplicated, so that the shared inverse stays valid).
 *    group_off: HOST int32 [G+1], 0 = group_off[0] < ... < group_off[G] = F: group g holds the
 *    consecutive features [group_off[g], group_off[g+1]) of the KJT.
 *    Rows b, b' of group g share a slot iff they hold the same list in every feature of g.  Slots
 *    are numbered in first-occurrence order.  Every feature of g stores one list per slot (its
 *    own list of the slot's first row), in slot order; the unique arrays are feature-major.
 *    values [N], offsets [F*B+1]: device, read-only.
 *    u_values: device, capacity N.  u_offsets: device, capacity F*B+1.
 *    inverse_g: device int32 [G*B], inverse_g[g*B+b] in [0, U_g).
 *    group_uoff: device int64 [G+1], prefix sum of U_g.
 *    feat_uoff: device int64 [F+1], prefix sum of the per-feature list counts (U_g of f's group):
 *    with it calls 2 and 6 work on the result unchanged.
 *    inverse_per_feature: optional device int32 [F*B]: the group's inverse repeated for each of
 *    its features, in the layout calls 3, 5 and 7 expect; NULL to skip.
 *    host_counts: optional host int64[3]; if non-NULL the call synchronises and stores the number
 *    of stored lists (feat_uoff[F]), the number of stored ids M, and the sum of U_g.
 *    Singleton groups give exactly the result of call 1. */
recd_status recd_build_ikjt_grouped(recd_ctx *ctx, int F, int64_t B, int64_t N, int G,
                                    const int32_t *group_off, const int64_t *values,
                                    const int64_t *offsets, int64_t *u_values, int64_t *u_offsets,
                                    int32_t *inverse_g, int64_t *group_uoff, int64_t *feat_uoff,
                                    int32_t *inverse_per_feature, int64_t *host_counts);

/* 10. A compute module run on the deduplicated rows of a grouped IKJT (Sec. 5 "Deduplicated
 *    Pooling": the element-wise sum over the features of a group, computed once per unique row
 *    and expanded through the shared inverse_lookup):
 *      combined[group_uoff[g] + k, :] = sum over f in group g (feature order) of
 *                                       pooled[feat_uoff[f] + k, :],  k in [0, U_g)
 *    fp32 accumulation, rounded once to dt.  pooled: device [U, D] of dt (output of call 2 on a
 *    grouped IKJT); combined: device [sum of U_g, D] of dt, capacity max_rows rows (G*B always
 *    suffices).  recd_expand_inverse(ctx, G, B, D, dt, combined, group_uoff, inverse_g, out) then
 *    yields the [G, B, D] result.  group_off: HOST int32 [G+1] as in call 9. */
recd_status recd_group_sum_unique(recd_ctx *ctx, int F, int G, int D, recd_dtype dt,
                                  const int32_t *group_off, const void *pooled,
                                  const int64_t *feat_uoff, const int64_t *group_uoff,
                                  int64_t max_rows, void *combined);

/* 11. Calls 2 and 4 with another pooling function (Sec. 2.2 names average, sum and max; forward
 *    only).  RECD_POOL_SUM is exactly call 2 / call 4.  RECD_POOL_MEAN: the sum (fp32, same order
 *    of additions) divided by the number of ids of the list.  RECD_POOL_MAX: element-wise maximum
 *    over the list's rows.  An empty list pools to zero in every mode.  As for the sum, the
 *    order of operations depends on the list alone, so the expanded result of the deduplicated
 *    lookup equals the KJT lookup bit for bit.  Arguments as in calls 2 and 4. */
recd_status recd_pooled_lookup_unique_mode(recd_ctx *ctx, recd_pooling mode, int F, int D,
                                           recd_dtype table_dt, recd_dtype out_dt,
                                           const void *const *tables, const int64_t *rows,
                                           const int64_t *u_values, const int64_t *u_offsets,
                                           const int64_t *feat_uoff, int64_t max_lists, void *pooled);
recd_status recd_kjt_pooled_lookup_mode(recd_ctx *ctx, recd_pooling mode, int F, int64_t B, int D,
                                        recd_dtype table_dt, recd_dtype out_dt,
                                        const void *const *tables, const int64_t *rows,
                                        const int64_t *values, const int64_t *offsets, void *out);

/* 12. KJT -> partial IKJT (Sec. 7 "Supporting Partial IKJTs": no offsets slice; every row is an
 *    [offset, length] window into the values slice, so that lists which are shifts of one another
 *    share storage; the paper's example stores feature b as values [3,4,5,6] with the windows
 *    [0,3], [1,3], [0,3]).  The paper prints no construction; this library's: the slots are those
 *    of call 1 (same duplicates, same first-occurrence numbering, same inverse and feat_uoff).
 *    A slot whose first row directly follows a row holding the previous slot's list continues
 *    that list: with k >= 1 the largest overlap of the previous list's tail with the new list's
 *    head, only the other ids are stored and the window starts k ids before the old end.  Every
 *    other slot stores its whole list.
 *    values [N], offsets [F*B+1]: device, read-only.  N must stay below 2^31.
 *    p_values: device, capacity N: the stored ids, feature-major.
 *    win_start, win_len: device int64, capacity F*B: window of slot u (position in p_values,
 *    length); list u = p_values[win_start[u] .. win_start[u] + win_len[u]).
 *    inverse [F*B], feat_uoff [F+1]: as in call 1.  feat_poff: device int64 [F+1], prefix sum of
 *    the ids stored per feature; windows never leave their feature's range.
 *    row_window: optional device int64 [F*B*2]: the paper's per-row inverse_lookup,
 *    row_window[2*(f*B+b)] = offset, [.. + 1] = length; NULL to skip.
 *    host_counts: optional host int64[3]; if non-NULL the call synchronises and stores U, the
 *    number of stored ids P, and M (what call 1 would store). */
recd_status recd_build_partial_ikjt(recd_ctx *ctx, int F, int64_t B, int64_t N,
                                    const int64_t *values, const int64_t *offsets, int64_t *p_values,
                                    int64_t *win_start, int64_t *win_len, int32_t *inverse,
                                    int64_t *feat_uoff, int64_t *feat_poff, int64_t *row_window,
                                    int64_t *host_counts);

/* 13. Call 2 on a partial IKJT: pooled[u,:] = sum over the ids of window u.  The windows hold the
 *    lists of call 1's slots in the same order, and the order of additions depends on the list
 *    alone, so the result equals call 2 on the IKJT of the same batch bit for bit; call 3 expands
 *    it.  P_cap: host upper bound of the number of stored ids (used by validation only).
 *    Other arguments as in call 2. */
recd_status recd_pooled_lookup_partial(recd_ctx *ctx, int F, int D, recd_dtype table_dt,
                                       recd_dtype out_dt, const void *const *tables,
                                       const int64_t *rows, const int64_t *p_values, int64_t P_cap,
                                       const int64_t *win_start, const int64_t *win_len,
                                       const int64_t *feat_uoff, int64_t max_lists, void *pooled);

/* 14. Backward of calls 7 and 6, the sequence path (chain rule; the paper describes the forward
 *    side only, Sec. 5):
 *      grad_emb[u_offsets[u] + t, :] = sum over rows b (ascending) with inverse[f*B+b] = u of
 *                                      grad_out[offsets[f*B+b] + t, :]
 *      G_f[r,:] = sum over the positions j (ascending) of feature f's unique ids with
 *                 u_values[j] = r of grad_emb[j, :]
 *    Same machinery and guarantees as call 5 (stable sorts, fixed summation order, no
 *    floating-point atomics, optional fused row-wise Adagrad).
 *    grad_out: device fp32 [N, D], one gradient row per KJT position (the layout of call 7's
 *    output).  offsets: device [F*B+1], the KJT's offsets.  N must stay below 2^31.
 *    grad_emb: device fp32 [M, D], capacity M_cap rows: OUTPUT, the gradient with respect to the
 *    unique activations of call 6 (what a module between calls 6 and 7 would receive).
 *    All other arguments as in call 5. */
recd_status recd_backward_sequence_dedup(recd_ctx *ctx, int F, int64_t B, int64_t N, int D,
                                         const float *grad_out, const int64_t *offsets,
                                         const int32_t *inverse, const int64_t *feat_uoff,
                                         const int64_t *u_values, const int64_t *u_offsets,
                                         const int64_t *rows, int64_t U_cap, int64_t M_cap,
                                         float *grad_emb, int64_t *touched_rows, int64_t *feat_roff,
                                         float *grad_rows, void *const *tables,
                                         float *const *adagrad_state, float lr, float eps,
                                         int64_t *host_R);

/* 15. Call 5 for a pooled lookup made with another pooling function (Sec. 2.2 names sum, average
 *    and max).  RECD_POOL_SUM is exactly call 5.  RECD_POOL_MEAN: the backward of the averaged
 *    lookup of call 11: every position of unique list u receives g_u[u,:] / len(u), i.e.
 *      G_f[r,:] = sum over positions j (ascending) with u_values[j] = r of g_u[list of j, :] / len
 *    (g_u is divided once, in fp32, when it is formed).  RECD_POOL_MAX needs the looked-up tables:
 *    call 20; here it returns RECD_EINVAL.  All arguments as in call 5. */
recd_status recd_backward_dedup_mode(recd_ctx *ctx, recd_pooling mode, int F, int64_t B, int D,
                                     const float *grad_out, const int32_t *inverse,
                                     const int64_t *feat_uoff, const int64_t *u_values,
                                     const int64_t *u_offsets, const int64_t *rows, int64_t U_cap,
                                     int64_t M_cap, int64_t *touched_rows, int64_t *feat_roff,
                                     float *grad_rows, void *const *tables,
                                     float *const *adagrad_state, float lr, float eps,
                                     int64_t *host_R);

/* 16-19. Per-id weights (this build's reading; the paper's KJT carries ids only, Sec. 4.2): a
 *    weighted KJT holds one fp32 weight beside every id, `weights` device fp32 [N] aligned with
 *    `values`, and the pooled output of a list is the weighted sum
 *      out = sum over the ids j of the list, in list order, of weights[j] * W_f[values[j], :]
 *    (fp32, one fused multiply-add per element and id).  Two rows hold the same list only when ids
 *    AND weights agree position by position; weights are compared as bit patterns (+0 and -0
 *    differ, a NaN equals itself), which is what makes the pooled outputs equal whatever the table
 *    holds.
 *
 * 16. Call 1 for a weighted KJT.  u_weights: device fp32, capacity N: the weights of the unique
 *    lists, aligned with u_values.  All else as in call 1 (same slot numbering; with all weights
 *    equal the result is call 1's).  weights / u_weights may be NULL when N = 0. */
recd_status recd_build_ikjt_weighted(recd_ctx *ctx, int F, int64_t B, int64_t N,
                                     const int64_t *values, const float *weights,
                                     const int64_t *offsets, int64_t *u_values, float *u_weights,
                                     int64_t *u_offsets, int32_t *inverse, int64_t *feat_uoff,
                                     int64_t *host_U_M);

/* 17. Call 2 with weights: pooled[u,:] = weighted sum over unique list u.  The order of operations
 *    depends on the list alone, so call 3 on the result equals call 18 on the KJT bit for bit.
 *    u_weights may be NULL only when u_values is (no id anywhere). */
recd_status recd_pooled_lookup_unique_weighted(recd_ctx *ctx, int F, int D, recd_dtype table_dt,
                                               recd_dtype out_dt, const void *const *tables,
                                               const int64_t *rows, const int64_t *u_values,
                                               const float *u_weights, const int64_t *u_offsets,
                                               const int64_t *feat_uoff, int64_t max_lists,
                                               void *pooled);

/* 18. Call 4 with weights: the comparison path over every row of the weighted KJT. */
recd_status recd_kjt_pooled_lookup_weighted(recd_ctx *ctx, int F, int64_t B, int D,
                                            recd_dtype table_dt, recd_dtype out_dt,
                                            const void *const *tables, const int64_t *rows,
                                            const int64_t *values, const float *weights,
                                            const int64_t *offsets, void *out);

/* 19. Call 5 for the weighted lookup: position j of unique list u hands u_weights[j] * g_u[u,:] to
 *    table row u_values[j]:
 *      G_f[r,:] = sum over positions j (ascending) with u_values[j] = r of
 *                 u_weights[j] * g_u[list of j, :]      (fp32 fused multiply-adds)
 *    Same machinery and guarantees as call 5; all other arguments as there. */
recd_status recd_backward_dedup_weighted(recd_ctx *ctx, int F, int64_t B, int D,
                                         const float *grad_out, const int32_t *inverse,
                                         const int64_t *feat_uoff, const int64_t *u_values,
                                         const float *u_weights, const int64_t *u_offsets,
                                         const int64_t *rows, int64_t U_cap, int64_t M_cap,
                                         int64_t *touched_rows, int64_t *feat_roff, float *grad_rows,
                                         void *const *tables, float *const *adagrad_state, float lr,
                                         float eps, int64_t *host_R);

/* Counts of the most recent call 1 / call 16 on this context: host_U_M[0] = U, host_U_M[1] = M.
 *    A builder called with host_U_M = NULL publishes its counts to the host by itself as soon as
 *    they are final on the GPU (its last kernel, which copies the ids, may still be running: calls
 *    that read the IKJT must be enqueued on the context's stream, as always); this call waits for
 *    that publication only, not for work enqueued after the build.  It lets a caller enqueue the lookup and the expand (which need no host-side count: any
 *    max_lists sizes the launch, see call 2) behind the build and read U and M, which the backward's
 *    bounds want, while they run.  Blocks the calling thread; RECD_EINVAL before the first build. */
recd_status recd_last_ikjt_counts(recd_ctx *ctx, int64_t *host_U_M);
/* The number of runs (maximal blocks of adjacent rows of a feature that hold one list; call 23) of
 *    the same build: host_runs[0] = R.  Counted by every call 1 / 16 / 23, whether or not it stores a
 *    run index.  Same waiting rule as recd_last_ikjt_counts. */
recd_status recd_last_ikjt_run_count(recd_ctx *ctx, int64_t *host_runs);

/* 21, 22. Call 5 in two halves.  What the backward does before it touches a gradient (keys, the two
 *    stable sorts, the numbering of the segments, touched_rows and feat_roff) depends on the IKJT
 *    alone.  recd_backward_plan enqueues that half on the context's two side streams and returns; if
 *    inverse and u_values are the outputs of the context's most recent call 1 / 16, the side streams
 *    start where that build ended, so the plan runs next to calls 2 and 3 enqueued meanwhile on the
 *    context's stream; otherwise they start at the stream's current position.
 *    recd_backward_apply makes the stream wait for the plan and runs the two segment sums (and the
 *    optimizer) exactly as call 5 / call 15 would: same kernels, same results bit for bit.
 *    Between the two calls the context's workspace holds the plan: no other call that uses the
 *    workspace (builders, other backward calls, the sequence lookups) may come in between: such a call
 *    is safe (its kernels go behind the plan's) but drops the plan.  Calls 2, 3, 4 and
 *    recd_last_ikjt_counts may come in between; the IKJT arrays, touched_rows and feat_roff must stay as they are.
 *    recd_backward_apply returns RECD_EINVAL if no valid plan exists.  mode: RECD_POOL_SUM or
 *    RECD_POOL_MEAN.  Arguments as in call 5. */
recd_status recd_backward_plan(recd_ctx *ctx, int F, int64_t B, int D, const int32_t *inverse,
                               const int64_t *feat_uoff, const int64_t *u_values,
                               const int64_t *u_offsets, const int64_t *rows, int64_t U_cap,
                               int64_t M_cap, int64_t *touched_rows, int64_t *feat_roff);
/* 26. Call 21 for a batch with a run index (call 23 / 24): the first grouping (rows by unique list)
 *    sorts the runs, of which a session-clustered batch has about as many as unique lists, instead
 *    of all F*B rows, and writes the sorted runs out as the row list the full sort would have given:
 *    the plan is the same plan, recd_backward_apply and its results are unchanged bit for bit.
 *    run_index: device, must describe `inverse`.  runs_cap: host upper bound of the number of runs
 *    (recd_last_ikjt_run_count gives the exact value; F*B always bounds it; 0 = F*B); if it is too
 *    small, recd_backward_apply with host_R reports RECD_ECAPACITY.  All else as in call 21. */
recd_status recd_backward_plan_runs(recd_ctx *ctx, int F, int64_t B, int D, const int32_t *inverse,
                                    const int64_t *feat_uoff, const int64_t *u_values,
                                    const int64_t *u_offsets, const int64_t *rows, int64_t U_cap,
                                    int64_t M_cap, const int64_t *run_index, int64_t runs_cap,
                                    int64_t *touched_rows, int64_t *feat_roff);
recd_status recd_backward_apply(recd_ctx *ctx, recd_pooling mode, const float *grad_out,
                                float *grad_rows, void *const *tables, float *const *adagrad_state,
                                float lr, float eps, int64_t *host_R);

/* 20. Call 5 for the max-pooled lookup of call 11 (Sec. 2.2 names max among the pooling functions):
 *    element d of g_u[u,:] goes to the table row at the position of unique list u that holds the
 *    largest table element d; among equal values the first position of the list takes it (this
 *    build's reading):
 *      G_f[r, d] = sum over the unique lists u (ascending) whose winning position for d holds id r
 *                  of g_u[u, d]
 *    lookup_tables: HOST array of F device pointers to the fp32 tables [rows_f, D] the forward pass
 *    looked up (fp32 only); they are read before any update, so they may be the same as `tables`.
 *    The call materialises one masked gradient row per position of u_values in the workspace
 *    (M_cap * D * 4 bytes more than recd_workspace_bytes reports; the workspace grows on demand, which
 *    synchronises and allocates).  All other arguments, and the guarantees, as in call 5. */
recd_status recd_backward_dedup_max(recd_ctx *ctx, int F, int64_t B, int D, const float *grad_out,
                                    const int32_t *inverse, const int64_t *feat_uoff,
                                    const int64_t *u_values, const int64_t *u_offsets,
                                    const int64_t *rows, int64_t U_cap, int64_t M_cap,
                                    const void *const *lookup_tables, int64_t *touched_rows,
                                    int64_t *feat_roff, float *grad_rows, void *const *tables,
                                    float *const *adagrad_state, float lr, float eps,
                                    int64_t *host_R);

/* 23. Call 1 that also returns the batch's run index (Sec. 4.2: the rows of a batch are clustered
 *    by session, so the duplicates of a list sit right behind its first occurrence; a run is a
 *    maximal block of adjacent rows of one feature that hold the same list).  Calls 25 and the
 *    backward work run by run.
 *    run_index: device int64, capacity 3 * (F*B + 2), triples:
 *      triple 0           {number of runs R, U, M}
 *      triple 1 + r       run r, in (feature, row) order:
 *                         {row | (u | first << 31) << 32,  position of list u's ids in u_values,
 *                          number of ids}   with row = f*B + b of the run's first row (low 32 bits), u
 *                         the global unique-list index (feat_uoff[f] + inverse[row]) and first = 1 iff
 *                         the run starts at the first row of the batch that holds list u
 *      triple 1 + R       closing entry {F*B, M, 0}: run r covers the rows [row_r, row_{r+1})
 *    Everything else as in call 1 (same kernels; the entries are written by the builder's last
 *    kernel from what it holds anyway). */
recd_status recd_build_ikjt_runs(recd_ctx *ctx, int F, int64_t B, int64_t N,
                                 const int64_t *values, const int64_t *offsets,
                                 int64_t *u_values, int64_t *u_offsets, int32_t *inverse,
                                 int64_t *feat_uoff, int64_t *run_index, int64_t *host_U_M);

/* 24. The same run index from an IKJT's arrays alone, for IKJTs of the other builders (calls 9, 12,
 *    16) or of another producer.  inverse [F*B], feat_uoff [F+1], u_offsets [U+1]: device.
 *    Uses the context's workspace. */
recd_status recd_ikjt_run_index(recd_ctx *ctx, int F, int64_t B, const int32_t *inverse,
                                const int64_t *feat_uoff, const int64_t *u_offsets,
                                int64_t *run_index);

/* 25. Calls 2 and 3 in one pass (Sec. 5 "EMB Lookups": the lookup runs on the unique lists only;
 *    "Jagged Index Select": the index select back to the batch is the only work deduplication adds
 *    - here most of it rides on the lookup).  The wave that sums unique list u, for the run that
 *    starts at u's first row, stores the finished row to pooled[u,:] and to out[f,b,:] of every row
 *    of the run; a second short kernel copies pooled[u,:] to the runs of u that come later in the
 *    batch.  One entry of the run index tells a wave all it needs (the ids' position and count, the
 *    rows to write), so a list costs two dependent memory round trips before its first table row
 *    instead of three.  Results: pooled and out hold exactly the bits calls 2 and 3 produce.
 *    run_index: device, from call 23 or 24.  max_runs: the host's estimate of the number of runs
 *    (sizes the launch only, as max_lists in call 2; 0 = F*B).  u_values: device [M].
 *    pooled: device [U, D] of out_dt (room for U rows; F*B when U is not known).
 *    out: device [F, B, D] of out_dt, or NULL: then only pooled is written (call 2 driven by the
 *    run index; call 3 can follow).  Sum pooling; dtypes and D as in call 2.
 *    A batch of at most 16384 rows takes one kernel: every run sums its list, also the later runs of
 *    a list (same ids in the same order: the same bits), and no copy follows.
 *    The call does not use the context's workspace (a pending backward plan stays valid). */
recd_status recd_pooled_lookup_expand(recd_ctx *ctx, int F, int64_t B, int D, recd_dtype table_dt,
                                      recd_dtype out_dt, const void *const *tables,
                                      const int64_t *rows, const int64_t *u_values,
                                      const int64_t *run_index, int64_t max_runs, void *pooled,
                                      void *out);

/* Call 1 for callers that cannot allocate: code under HIP graph capture, serving loops and harnesses
 *    in which hipMalloc is forbidden.  Same arguments, same outputs bit for bit as recd_build_ikjt,
 *    but the builder's scratch (hash tables, per-list numbering arrays, block sums) lives in a
 *    file-scope device array of the library, about 3.1 MB, which every GPU the library runs on holds
 *    until the process ends; the call allocates and frees nothing, records no memset, does not
 *    synchronise and does not touch the context's workspace (a pending backward plan stays valid).
 *    Limit: F*B <= RECD_NOALLOC_MAX_LISTS, else RECD_ECAPACITY (nothing is enqueued).  No host
 *    counts: U = feat_uoff[F] and M = u_offsets[U] are on the device; recd_last_ikjt_counts and the
 *    "most recent build" of recd_backward_plan do not see this call.
 *    All calls on one GPU share the one array, whatever their context: calls that overlap on a GPU
 *    (two streams, two contexts) race; calls on one stream are ordered and safe.  The array keeps
 *    the previous call's contents; the call clears what it needs cleared. */
#define RECD_NOALLOC_MAX_LISTS 65536
recd_status recd_build_ikjt_noalloc(recd_ctx *ctx, int F, int64_t B, int64_t N,
                                    const int64_t *values, const int64_t *offsets,
                                    int64_t *u_values, int64_t *u_offsets, int32_t *inverse,
                                    int64_t *feat_uoff);

#ifdef __cplusplus
}
#endif
#endif /* RECD_H */
