// Internal declarations shared by the translation units of librecd (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <string>
#include <vector>

#include "recd.h"

// Optional HIP-event brackets around single kernel launches (benchmark instrumentation, off by
// default): `slot` names the kernel, every bracket is one pair of events on the stream the kernel is
// launched on; recd_internal_kernel_ms averages the pairs recorded since the last reset.
enum {
    RECD_T_LOOKUP_EXPAND = 0,  // fused unique lookup + first-run expand
    RECD_T_UNCOVERED = 1,      // second pass of the fused expand
    RECD_T_LOOKUP = 2,         // unique lookup (two-kernel path)
    RECD_T_EXPAND = 3,         // expand (two-kernel path)
    RECD_T_KJT = 4,            // KJT comparison lookup
    RECD_T_HASH = 5,           // builder: hash + insert
    RECD_T_GRAD_LISTS = 6,     // backward step A: sum of grad_out rows per unique list
    RECD_T_GRAD_ROWS = 7,      // backward step B: row-gradient segment sum with the fused update
    RECD_T_EMIT = 8,           // builder: inverse + copy of the unique lists
    RECD_T_COUNT = 9
};
struct KernelTimer {
    std::vector<hipEvent_t> a, b;
    int n = 0;
};

struct recd_ctx {
    int device = 0;
    hipStream_t stream = nullptr;
    hipStream_t side_stream = nullptr;   // independent work of one call (default priority, non-blocking)
    hipEvent_t ev_fork = nullptr, ev_join = nullptr;
    // Planned backward: the gradient-independent half (sorts, segment numbering) of a backward pass
    // runs on two side streams from the end of the last build on, next to the forward calls.
    hipStream_t side_stream2 = nullptr;
    hipEvent_t ev_built = nullptr;                    // end of the most recent plain / weighted build
    hipEvent_t ev_plan_a = nullptr, ev_plan_b = nullptr;   // end of each of the plan's two chains
    hipEvent_t ev_plan_rows = nullptr;  // step B's segments numbered (before the cut of the long ones)
    const void *built_inverse = nullptr, *built_u_values = nullptr;  // outputs of that build
    // A call that uses the workspace has been enqueued on the context's stream since that build (set
    // by recd_reserve, cleared by the builder): a plan must then start at the stream's current
    // position, not at ev_built, or its side streams would write the workspace under that call.
    bool ws_used_since_build = true;
    // Step B of the backward: table rows with more entries than this are cut into chunks that whole
    // blocks sum (RECD_OPT_LONG_SEGMENT_CUT).
    int long_seg_cut = 32;
    struct BackwardPlan {
        bool valid = false, empty = false, wide = false;
        // the side streams may still be working in the workspace: set by recd_backward_plan, cleared
        // once the context's stream has been made to wait for both of the plan's events
        bool pending = false;
        int F = 0, D = 0, row_bits = 0;
        int64_t B = 0, U_cap = 0, M_cap = 0;
        const void *ks_a = nullptr;
        const uint32_t *ps_a = nullptr, *ps_b = nullptr;
        const int64_t *u_offsets = nullptr;
        int64_t *touched_rows = nullptr, *feat_roff = nullptr;
        const char *ws = nullptr;   // the workspace the plan lives in must still be the context's
    } plan;
    // Hash tables of the plain / weighted builder: memory of their own that is all "empty" whenever
    // no build is running on the stream, because the builder's last kernel clears what the build
    // used (so no clearing kernel stands at the head of the next build).  table_clean is false
    // while that cannot be relied on (first use, or a build that failed half way).
    uint64_t *build_table = nullptr;
    size_t build_table_slots = 0;
    bool table_clean = false;
    char *ws = nullptr;          // device workspace
    size_t ws_bytes = 0;
    int64_t *host_pinned = nullptr;  // 8 x int64 pinned staging for scalar results
    // Mailbox for scalar results the host waits for: pinned, coherent, mapped host memory that a
    // one-thread kernel writes (values, then a sequence number); nullptr if it could not be set up.
    volatile int64_t *mailbox = nullptr;
    int64_t *mailbox_dev = nullptr;
    int64_t mailbox_seq = 0;
    // Counts {U, M} of the most recent plain or weighted IKJT build: a device array that outlives the
    // workspace's reuse, and the second half of the mailbox (entries 8..15, sequence number in 15),
    // which the builder fills without being asked so that recd_last_ikjt_counts can wait for the
    // build alone.
    int64_t *build_counts_dev = nullptr;
    int64_t build_seq = 0;        // sequence number of the latest publication (never reused)
    bool build_published = false; // the last build published its counts (else: read the device array)
    // that publication is three words that each carry the sequence number (RECD_MAILBOX_TAG_BIT)
    // instead of values followed by the number
    bool build_tagged = false;
    bool build_valid = false;     // a plain / weighted build has written build_counts_dev
    // this device's copy of the static scratch array of recd_build_ikjt_noalloc (found at creation)
    char *static_scratch = nullptr;
    // Small batches are built by one launch (a block per feature): 2 words per feature + 2 that the
    // blocks exchange their counts through, all zero between launches.  small_path: 0 = never, 1 =
    // whenever the batch qualifies, 2 = as 1 with every wait between the blocks made to expire.
    uint64_t *small_agg = nullptr;
    int small_path = 1;
    int timing = 0;  // RECD_OPT_INTERNAL_TIMING
    KernelTimer timers[RECD_T_COUNT];
    int validate = 0;
    int weak_hash = 0;
    int tune_lb = 0, tune_gens = 0, tune_flat = 0;  // launch-shape overrides of the gather-sum kernel (0 = automatic)
    int num_cu = 256;
    // feature groups of the last grouped call, kept on the device: [0, G] boundaries, then the
    // group of every feature from RECD_MAX_FEATURES + 1 on
    int32_t *group_map_dev = nullptr;
    std::vector<int32_t> group_map_host;
    std::string err;
};

// Not part of the public interface: launch-shape override of the gather-sum kernel, used by the
// tuning runs and by the test that shows results do not depend on the launch shape.
//   value = lists per block (1, 2, 4, 8 or 16) + 10000 * block generations per CU (< 100)
//           + 1000000 * (1 = no XCD-aware block mapping); 0 = automatic
#define RECD_OPT_INTERNAL_TUNE_SEGSUM 1003
// value != 0: bracket the kernels named by RECD_T_* with HIP events (see recd_internal_kernel_ms)
#define RECD_OPT_INTERNAL_TIMING 1004
// 0: small batches take the general builder too; 1 (default): the one-launch builder; 2: the
// one-launch builder with the waits between its blocks forced to expire (tests of the error path)
#define RECD_OPT_INTERNAL_SMALL_PATH 1005
#define RECD_SMALL_MAX_FEATURES 256
// Tagged mailbox words of the one-launch builder: bits 40..63 = RECD_MAILBOX_TAG_BIT | low 23 bits of
// the build's sequence number, bits 0..39 = the value (all ones: the build failed).  A word of the
// other builders (a plain count below 2^40) never carries a tag.
#define RECD_MAILBOX_TAG_BIT (1u << 23)
void recd_time_begin(recd_ctx *ctx, int slot, hipStream_t st);
void recd_time_end(recd_ctx *ctx, int slot, hipStream_t st);

recd_status recd_fail(recd_ctx *ctx, recd_status s, const char *fmt, ...);
// Ids must lie in [0, 2^31): a table the caller describes as larger is refused (rows may be null).
recd_status recd_check_rows(recd_ctx *ctx, int F, const int64_t *rows);
// After a builder wrote {U, M} into ctx->build_counts_dev: publish them to the host asynchronously.
recd_status recd_publish_build_counts(recd_ctx *ctx);
recd_status recd_reserve(recd_ctx *ctx, size_t bytes);
// Looks up the current device's copy of the static scratch array (with `device` current).
recd_status recd_static_scratch(recd_ctx *ctx, int device);

#define RECD_HIP(ctx, call)                                                                   \
    do {                                                                                      \
        hipError_t e_ = (call);                                                               \
        if (e_ != hipSuccess)                                                                 \
            return recd_fail((ctx), RECD_EHIP, "%s failed: %s", #call, hipGetErrorString(e_)); \
    } while (0)

#define RECD_TRY(expr)            \
    do {                          \
        recd_status s_ = (expr);  \
        if (s_ != RECD_OK)        \
            return s_;            \
    } while (0)

// Bump allocator over the context workspace (256-byte aligned pieces).
struct WsCarver {
    char *base;
    size_t off = 0;
    explicit WsCarver(char *b) : base(b) {}
    template <typename T> T *take(size_t count)
    {
        size_t bytes = (count * sizeof(T) + 255) & ~size_t(255);
        T *p = base ? reinterpret_cast<T *>(base + off) : nullptr;
        off += bytes;
        return p;
    }
};

static inline size_t elem_size(recd_dtype dt) { return dt == RECD_F32 ? 4 : 2; }

// Tables of up to this many features travel to a kernel by value.
#define RECD_F_PER_LAUNCH 128
struct TablePtrs {
    const void *p[RECD_F_PER_LAUNCH];
};

// Optional epilogue of the row-gradient segment sums: row-wise Adagrad applied to the table row a
// segment belongs to, straight from the registers that hold the segment's sum.
struct OptAdagrad {
    float *w[RECD_F_PER_LAUNCH];   // tables (n_feat == 0: no optimizer)
    float *m[RECD_F_PER_LAUNCH];   // accumulators
    const int64_t *touched_rows;   // [R] table row of every segment
    const int32_t *seg_feat;       // [R] feature of every segment
    int n_feat;
    float lr, eps;
};

// ---- cross-file entry points (host side launchers) -------------------------------------------
// Exclusive scan of n int64 pairs is private to each file; the segmented gather-sum is shared.
// GRAD_STREAM: as GRAD_LISTS, for source rows that are read once (step A reads every grad_out row
// exactly once): their loads bypass the caches' retention.
// UNIQUE_EXPAND: the unique lookup that also writes the output rows of every list's first run.
enum { RECD_SITE_UNIQUE = 0, RECD_SITE_KJT = 1, RECD_SITE_GRAD_LISTS = 2, RECD_SITE_GRAD_STREAM = 3,
       RECD_SITE_UNIQUE_EXPAND = 4 };
struct SegSumArgs {
    int F;                    // features in this launch (<= RECD_F_PER_LAUNCH)
    int D;
    recd_dtype table_dt, out_dt;
    TablePtrs tables;
    const void *values;       // int64 or int32 ids
    int values_are_i32;
    const int64_t *offsets;   // list l spans offsets[l]..offsets[l+1]
    const int64_t *list_off;  // device [F+1] or nullptr -> list_off[f] = f * lists_per_feature
    int64_t lists_per_feature;
    int64_t list_base;        // added to every list index (feature chunking of the KJT path)
    int64_t lists_bound;      // host upper bound of the number of lists in this launch (sizes the grid)
    int flat;                 // 1: no XCD-aware feature->block mapping
    const int64_t *ends;            // optional (single table, flat): list l ends at ends[l] ...
    const int64_t *count_dev;       // ... and the number of lists lives on the device
    const int64_t *lens;            // optional: list l spans offsets[l] .. offsets[l] + lens[l]
    const float *weights;           // mode 3 (weighted sum): one fp32 weight per id, beside values
    const int64_t *div_off;         // optional (backward sums only): the finished row of list l is
                                    // divided by div_off[l+1] - div_off[l] when that is positive
    // RECD_SITE_UNIQUE_EXPAND only: the IKJT's run index, the expanded output, rows per feature, the
    // launch's first feature and the call's feature count (lists_bound = host estimate of the runs)
    const int64_t *run_index;
    void *expanded;
    int64_t B;
    int feat_base;
    int F_all;
    int all_runs;             // 1: runs that are not their list's first sum the list too (no copy pass follows)
    int site;                 // RECD_SITE_*: which call site (each has its own kernel instantiation)
    int mode;                 // recd_pooling (forward sites only; 0 = sum)
    void *out;                // [lists, D]
    hipStream_t stream;       // nullptr: the context's stream
};
recd_status recd_launch_segsum(recd_ctx *ctx, const SegSumArgs &a);
recd_status recd_validate_inverse(recd_ctx *ctx, int F, int64_t B, const int64_t *feat_uoff,
                                  const int32_t *inverse);
recd_status recd_validate_kjt_offsets(recd_ctx *ctx, int F, int64_t B, int64_t N, const int64_t *offsets);
recd_status recd_validate_kjt_lists(recd_ctx *ctx, int F, int64_t B, int64_t N, const int64_t *rows,
                                    const int64_t *values, const int64_t *offsets);
recd_status recd_validate_unique_lists(recd_ctx *ctx, int F, const int64_t *rows,
                                       const int64_t *u_values, const int64_t *u_offsets,
                                       const int64_t *feat_uoff, int64_t max_lists, int64_t M_cap);
// Device copies of group_off[0..G] and of the group of every feature; copied (with a stream
// synchronisation) only when the grouping differs from the previous call's.
recd_status recd_group_map(recd_ctx *ctx, int F, int G, const int32_t *group_off,
                           const int32_t **dev_group_off, const int32_t **dev_feat_group);
// Brings n <= 6 int64 values at `dev` to the host once everything enqueued on the context's stream
// before the call has finished.
recd_status recd_fetch_scalars(recd_ctx *ctx, const int64_t *dev, int n, int64_t *host_out);
