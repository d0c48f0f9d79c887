// Context, workspace and status plumbing of librecd.
#include <stdarg.h>

#include "recd_internal.h"

#include <algorithm>
#include <atomic>
#include <chrono>

recd_status recd_fail(recd_ctx *ctx, recd_status s, const char *fmt, ...)
{
    if (ctx) {
        char buf[512];
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(buf, sizeof buf, fmt, ap);
        va_end(ap);
        ctx->err = buf;
    }
    return s;
}

recd_status recd_check_rows(recd_ctx *ctx, int F, const int64_t *rows)
{
    if (rows)
        for (int f = 0; f < F; f++)
            if (rows[f] < 0 || rows[f] > ((int64_t)1 << 31))
                return recd_fail(ctx, RECD_EINVAL, "rows[%d]=%lld: tables hold at most 2^31 rows", f,
                                 (long long)rows[f]);
    return RECD_OK;
}

recd_status recd_reserve(recd_ctx *ctx, size_t bytes)
{
    // Every call that is about to use the workspace comes through here first.  A plan that was never
    // applied may still be running on the side streams, in the same memory: the caller's kernels go
    // behind it.
    ctx->ws_used_since_build = true;
    if (ctx->plan.pending) {
        RECD_HIP(ctx, hipStreamWaitEvent(ctx->stream, ctx->ev_plan_a, 0));
        RECD_HIP(ctx, hipStreamWaitEvent(ctx->stream, ctx->ev_plan_b, 0));
        ctx->plan.pending = false;
    }
    if (bytes <= ctx->ws_bytes)
        return RECD_OK;
    // Growing: earlier kernels may still use the old block; a backward plan lives in it.
    RECD_HIP(ctx, hipStreamSynchronize(ctx->stream));
    if (ctx->side_stream)
        RECD_HIP(ctx, hipStreamSynchronize(ctx->side_stream));
    if (ctx->side_stream2)
        RECD_HIP(ctx, hipStreamSynchronize(ctx->side_stream2));
    ctx->plan.valid = false;
    if (ctx->ws) {
        RECD_HIP(ctx, hipFree(ctx->ws));
        ctx->ws = nullptr;
        ctx->ws_bytes = 0;
    }
    size_t want = bytes + bytes / 4 + (1u << 20);
    void *p = nullptr;
    if (hipMalloc(&p, want) != hipSuccess) {
        (void)hipGetLastError();
        return recd_fail(ctx, RECD_ENOMEM, "workspace allocation of %zu bytes failed", want);
    }
    ctx->ws = static_cast<char *>(p);
    ctx->ws_bytes = want;
    return RECD_OK;
}

constexpr int kTimerPairs = 1024;

void recd_time_begin(recd_ctx *ctx, int slot, hipStream_t st)
{
    if (!ctx->timing)
        return;
    KernelTimer &t = ctx->timers[slot];
    if (t.n >= kTimerPairs)
        return;
    if ((int)t.a.size() <= t.n) {
        hipEvent_t ea = nullptr, eb = nullptr;
        if (hipEventCreate(&ea) != hipSuccess || hipEventCreate(&eb) != hipSuccess) {
            (void)hipGetLastError();
            return;
        }
        t.a.push_back(ea);
        t.b.push_back(eb);
    }
    (void)hipEventRecord(t.a[t.n], st);
}

void recd_time_end(recd_ctx *ctx, int slot, hipStream_t st)
{
    if (!ctx->timing)
        return;
    KernelTimer &t = ctx->timers[slot];
    if (t.n >= kTimerPairs || (int)t.a.size() <= t.n)
        return;
    (void)hipEventRecord(t.b[t.n], st);
    t.n++;
}

// Not declared in the public header.  Average (and median) milliseconds of the event pairs recorded
// for `slot` since the last reset; synchronises the device.  count = pairs averaged.
extern "C" recd_status recd_internal_kernel_ms(recd_ctx *ctx, int slot, int reset, double *avg_ms, double *median_ms,
                                               int *count)
{
    if (!ctx || slot < 0 || slot >= RECD_T_COUNT)
        return RECD_EINVAL;
    KernelTimer &t = ctx->timers[slot];
    RECD_HIP(ctx, hipSetDevice(ctx->device));
    RECD_HIP(ctx, hipDeviceSynchronize());
    std::vector<float> ms;
    for (int i = 0; i < t.n; i++) {
        float x = 0.f;
        if (hipEventElapsedTime(&x, t.a[i], t.b[i]) == hipSuccess)
            ms.push_back(x);
        else
            (void)hipGetLastError();
    }
    double sum = 0.0;
    for (float x : ms)
        sum += x;
    std::sort(ms.begin(), ms.end());
    if (avg_ms)
        *avg_ms = ms.empty() ? 0.0 : sum / (double)ms.size();
    if (median_ms)
        *median_ms = ms.empty() ? 0.0 : (double)ms[ms.size() / 2];
    if (count)
        *count = (int)ms.size();
    if (reset)
        t.n = 0;
    return RECD_OK;
}

recd_status recd_group_map(recd_ctx *ctx, int F, int G, const int32_t *group_off,
                           const int32_t **dev_group_off, const int32_t **dev_feat_group)
{
    constexpr int kHalf = RECD_MAX_FEATURES + 1;
    std::vector<int32_t> map(2 * kHalf, 0);
    for (int g = 0; g <= G; g++)
        map[g] = group_off[g];
    for (int g = 0; g < G; g++)
        for (int f = group_off[g]; f < group_off[g + 1] && f < F; f++)
            map[kHalf + f] = g;
    if (!ctx->group_map_dev)
        RECD_HIP(ctx, hipMalloc(reinterpret_cast<void **>(&ctx->group_map_dev), sizeof(int32_t) * 2 * kHalf));
    if (map != ctx->group_map_host) {
        // earlier calls on either stream may still read the old map
        RECD_HIP(ctx, hipStreamSynchronize(ctx->stream));
        RECD_HIP(ctx, hipMemcpy(ctx->group_map_dev, map.data(), sizeof(int32_t) * 2 * kHalf,
                                hipMemcpyHostToDevice));
        ctx->group_map_host.swap(map);
    }
    *dev_group_off = ctx->group_map_dev;
    *dev_feat_group = ctx->group_map_dev + kHalf;
    return RECD_OK;
}

// values first, the sequence number last, each visible to the host before the next
__global__ void k_publish(const int64_t *__restrict__ src, int n, int64_t *mailbox, int64_t seq)
{
    for (int i = 0; i < n; i++)
        mailbox[i] = src[i];
    __threadfence_system();
    mailbox[7] = seq;
    __threadfence_system();
}

recd_status recd_publish_build_counts(recd_ctx *ctx)
{
    ctx->build_published = false;
    if (!ctx->mailbox)
        return RECD_OK;  // no mapped mailbox: recd_last_ikjt_counts copies from the device array
    const int64_t seq = ++ctx->build_seq;
    ctx->build_published = true;
    ctx->build_tagged = false;
    hipLaunchKernelGGL(k_publish, dim3(1), dim3(1), 0, ctx->stream, ctx->build_counts_dev, 3,
                       ctx->mailbox_dev + 8, seq);
    RECD_HIP(ctx, hipGetLastError());
    return RECD_OK;
}

recd_status recd_fetch_scalars(recd_ctx *ctx, const int64_t *dev, int n, int64_t *host_out)
{
    if (n < 0 || n > 6)
        return recd_fail(ctx, RECD_EINVAL, "recd_fetch_scalars: n=%d", n);
    if (ctx->mailbox) {
        // The host polls the mailbox instead of sleeping in a stream synchronisation: the wake-up
        // of a blocked thread costs more than the kernels of a small call.
        const int64_t seq = ++ctx->mailbox_seq;
        hipLaunchKernelGGL(k_publish, dim3(1), dim3(1), 0, ctx->stream, dev, n, ctx->mailbox_dev, seq);
        RECD_HIP(ctx, hipGetLastError());
        const auto t0 = std::chrono::steady_clock::now();
        bool seen = false;
        for (uint64_t spin = 0;; spin++) {
            if (ctx->mailbox[7] == seq) {
                seen = true;
                break;
            }
            if ((spin & 0xfff) == 0xfff &&
                std::chrono::steady_clock::now() - t0 > std::chrono::milliseconds(200))
                break;  // a long queue ahead of us, or an error: let the runtime wait
        }
        if (!seen) {
            RECD_HIP(ctx, hipStreamSynchronize(ctx->stream));
            if (ctx->mailbox[7] != seq)
                return recd_fail(ctx, RECD_EHIP, "result mailbox was not written");
        }
        std::atomic_thread_fence(std::memory_order_acquire);
        for (int i = 0; i < n; i++)
            host_out[i] = ctx->mailbox[i];
        return RECD_OK;
    }
    RECD_HIP(ctx, hipMemcpyAsync(ctx->host_pinned, dev, n * sizeof(int64_t), hipMemcpyDeviceToHost,
                                 ctx->stream));
    RECD_HIP(ctx, hipStreamSynchronize(ctx->stream));
    for (int i = 0; i < n; i++)
        host_out[i] = ctx->host_pinned[i];
    return RECD_OK;
}

extern "C" {

const char *recd_status_string(recd_status s)
{
    switch (s) {
    case RECD_OK: return "RECD_OK";
    case RECD_EINVAL: return "RECD_EINVAL";
    case RECD_ENOMEM: return "RECD_ENOMEM";
    case RECD_EHIP: return "RECD_EHIP";
    case RECD_EBOUNDS: return "RECD_EBOUNDS";
    case RECD_ECAPACITY: return "RECD_ECAPACITY";
    }
    return "RECD_UNKNOWN";
}

recd_status recd_create(recd_ctx **out, int device, void *hip_stream, size_t workspace_hint_bytes)
{
    if (!out || device < 0)
        return RECD_EINVAL;
    *out = nullptr;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || device >= ndev) {
        (void)hipGetLastError();
        return RECD_EHIP;
    }
    recd_ctx *ctx = new (std::nothrow) recd_ctx();
    if (!ctx)
        return RECD_ENOMEM;
    ctx->device = device;
    ctx->stream = static_cast<hipStream_t>(hip_stream);
    bool ok = hipSetDevice(device) == hipSuccess;
    hipDeviceProp_t prop;
    if (ok && hipGetDeviceProperties(&prop, device) == hipSuccess && prop.multiProcessorCount > 0)
        ctx->num_cu = prop.multiProcessorCount;
    ok = ok && hipStreamCreateWithFlags(&ctx->side_stream, hipStreamNonBlocking) == hipSuccess;
    ok = ok && hipStreamCreateWithFlags(&ctx->side_stream2, hipStreamNonBlocking) == hipSuccess;
    ok = ok && hipEventCreateWithFlags(&ctx->ev_built, hipEventDisableTiming) == hipSuccess;
    ok = ok && hipEventCreateWithFlags(&ctx->ev_plan_a, hipEventDisableTiming) == hipSuccess;
    ok = ok && hipEventCreateWithFlags(&ctx->ev_plan_b, hipEventDisableTiming) == hipSuccess;
    ok = ok && hipEventCreateWithFlags(&ctx->ev_plan_rows, hipEventDisableTiming) == hipSuccess;
    ok = ok && hipEventCreateWithFlags(&ctx->ev_fork, hipEventDisableTiming) == hipSuccess;
    ok = ok && hipEventCreateWithFlags(&ctx->ev_join, hipEventDisableTiming) == hipSuccess;
    void *p = nullptr;
    ok = ok && hipHostMalloc(&p, 8 * sizeof(int64_t), hipHostMallocDefault) == hipSuccess;
    ctx->host_pinned = static_cast<int64_t *>(p);
    void *mb = nullptr, *mb_dev = nullptr;
    if (ok && hipHostMalloc(&mb, 16 * sizeof(int64_t), hipHostMallocMapped | hipHostMallocCoherent) == hipSuccess) {
        if (hipHostGetDevicePointer(&mb_dev, mb, 0) == hipSuccess) {
            ctx->mailbox = static_cast<volatile int64_t *>(mb);
            ctx->mailbox_dev = static_cast<int64_t *>(mb_dev);
            for (int i = 0; i < 16; i++)
                ctx->mailbox[i] = 0;
        } else {
            (void)hipGetLastError();
            (void)hipHostFree(mb);
        }
    } else if (ok) {
        (void)hipGetLastError();
    }
    void *bc = nullptr;
    ok = ok && hipMalloc(&bc, 4 * sizeof(int64_t)) == hipSuccess;
    ctx->build_counts_dev = static_cast<int64_t *>(bc);
    void *sa = nullptr;
    const size_t sa_bytes = (2 * RECD_SMALL_MAX_FEATURES + 2) * sizeof(uint64_t);
    ok = ok && hipMalloc(&sa, sa_bytes) == hipSuccess;
    ok = ok && hipMemset(sa, 0, sa_bytes) == hipSuccess;
    ok = ok && hipStreamSynchronize(nullptr) == hipSuccess;  // cleared before any stream of the context reads it
    ctx->small_agg = static_cast<uint64_t *>(sa);
    ok = ok && recd_static_scratch(ctx, device) == RECD_OK;
    if (ok && workspace_hint_bytes)
        ok = recd_reserve(ctx, workspace_hint_bytes) == RECD_OK;
    if (!ok) {
        (void)hipGetLastError();
        recd_destroy(ctx);
        return RECD_EHIP;
    }
    *out = ctx;
    return RECD_OK;
}

recd_status recd_destroy(recd_ctx *ctx)
{
    if (!ctx)
        return RECD_OK;
    (void)hipSetDevice(ctx->device);
    (void)hipStreamSynchronize(ctx->stream);
    if (ctx->side_stream) {
        (void)hipStreamSynchronize(ctx->side_stream);
        (void)hipStreamDestroy(ctx->side_stream);
    }
    if (ctx->side_stream2) {
        (void)hipStreamSynchronize(ctx->side_stream2);
        (void)hipStreamDestroy(ctx->side_stream2);
    }
    for (KernelTimer &t : ctx->timers)
        for (size_t i = 0; i < t.a.size(); i++) {
            (void)hipEventDestroy(t.a[i]);
            (void)hipEventDestroy(t.b[i]);
        }
    if (ctx->ev_built)
        (void)hipEventDestroy(ctx->ev_built);
    if (ctx->ev_plan_a)
        (void)hipEventDestroy(ctx->ev_plan_a);
    if (ctx->ev_plan_b)
        (void)hipEventDestroy(ctx->ev_plan_b);
    if (ctx->ev_plan_rows)
        (void)hipEventDestroy(ctx->ev_plan_rows);
    if (ctx->ev_fork)
        (void)hipEventDestroy(ctx->ev_fork);
    if (ctx->ev_join)
        (void)hipEventDestroy(ctx->ev_join);
    if (ctx->ws)
        (void)hipFree(ctx->ws);
    if (ctx->group_map_dev)
        (void)hipFree(ctx->group_map_dev);
    if (ctx->build_counts_dev)
        (void)hipFree(ctx->build_counts_dev);
    if (ctx->small_agg)
        (void)hipFree(ctx->small_agg);
    if (ctx->build_table)
        (void)hipFree(ctx->build_table);
    if (ctx->host_pinned)
        (void)hipHostFree(ctx->host_pinned);
    if (ctx->mailbox)
        (void)hipHostFree(const_cast<int64_t *>(ctx->mailbox));
    delete ctx;
    return RECD_OK;
}

recd_status recd_set_option(recd_ctx *ctx, recd_option opt, int64_t value)
{
    if (!ctx)
        return RECD_EINVAL;
    switch (opt) {
    case RECD_OPT_VALIDATE: ctx->validate = value != 0; return RECD_OK;
    case RECD_OPT_WEAK_HASH: ctx->weak_hash = value != 0; return RECD_OK;
    case RECD_OPT_LONG_SEGMENT_CUT:
        if (value != 16 && value != 32 && value != 64 && value != 128)
            return recd_fail(ctx, RECD_EINVAL, "RECD_OPT_LONG_SEGMENT_CUT must be 16, 32, 64 or 128");
        ctx->long_seg_cut = (int)value;
        ctx->plan.valid = false;  // a plan made with another cut no longer fits the buffers
        return RECD_OK;
    default: break;
    }
    switch ((int)opt) {
    case RECD_OPT_INTERNAL_TIMING: ctx->timing = value != 0; return RECD_OK;
    case RECD_OPT_INTERNAL_SMALL_PATH:
        if (value < 0 || value > 2)
            return recd_fail(ctx, RECD_EINVAL, "small-path option takes 0, 1 or 2");
        ctx->small_path = (int)value;
        return RECD_OK;
    case RECD_OPT_INTERNAL_TUNE_SEGSUM:
        ctx->tune_lb = (int)(value % 100);
        ctx->tune_gens = (int)(value / 10000 % 100);
        ctx->tune_flat = (int)(value / 1000000 % 10);
        if (value < 0 || value / 100 % 100 != 0 || value >= 2000000 ||
            (ctx->tune_lb != 0 && ctx->tune_lb != 1 && ctx->tune_lb != 2 && ctx->tune_lb != 4 && ctx->tune_lb != 8 &&
             ctx->tune_lb != 16)) {
            ctx->tune_lb = ctx->tune_gens = ctx->tune_flat = 0;
            return recd_fail(ctx, RECD_EINVAL, "bad launch-shape override");
        }
        return RECD_OK;
    }
    return recd_fail(ctx, RECD_EINVAL, "unknown option %d", (int)opt);
}

// {U, M, runs} of the most recent plain / weighted build: from the build's own publication if there
// is one (waits for that build only), else from the device array (waits for the stream).
static recd_status last_build_counts_raw(recd_ctx *ctx, int64_t out[3]);
static recd_status last_build_counts(recd_ctx *ctx, int64_t out[3])
{
    RECD_TRY(last_build_counts_raw(ctx, out));
    if (out[0] < 0)  // the one-launch builder of small batches reports a failed build this way
        return recd_fail(ctx, RECD_EHIP, "the builder's blocks did not receive each other's counts in time");
    return RECD_OK;
}

static recd_status last_build_counts_raw(recd_ctx *ctx, int64_t out[3])
{
    if (!ctx->build_valid)
        return recd_fail(ctx, RECD_EINVAL, "no recd_build_ikjt / recd_build_ikjt_weighted call on this context yet");
    RECD_HIP(ctx, hipSetDevice(ctx->device));
    if (ctx->mailbox && ctx->build_published) {
        // wait for the build's own publication, not for what was enqueued after it
        const auto t0 = std::chrono::steady_clock::now();
        for (uint64_t spin = 0;; spin++) {
            if (ctx->build_tagged) {
                const uint64_t tag = (uint64_t)RECD_MAILBOX_TAG_BIT | ((uint64_t)ctx->build_seq & (RECD_MAILBOX_TAG_BIT - 1));
                const uint64_t w0 = (uint64_t)ctx->mailbox[8], w1 = (uint64_t)ctx->mailbox[9], w2 = (uint64_t)ctx->mailbox[10];
                if ((w0 >> 40) == tag && (w1 >> 40) == tag && (w2 >> 40) == tag) {
                    const uint64_t m = 0xffffffffffull;
                    out[0] = (w0 & m) == m ? -1 : (int64_t)(w0 & m);
                    out[1] = (w1 & m) == m ? -1 : (int64_t)(w1 & m);
                    out[2] = (w2 & m) == m ? -1 : (int64_t)(w2 & m);
                    return RECD_OK;
                }
            } else if (ctx->mailbox[15] == ctx->build_seq) {
                std::atomic_thread_fence(std::memory_order_acquire);
                out[0] = ctx->mailbox[8];
                out[1] = ctx->mailbox[9];
                out[2] = ctx->mailbox[10];
                return RECD_OK;
            }
            if ((spin & 0xfff) == 0xfff &&
                std::chrono::steady_clock::now() - t0 > std::chrono::milliseconds(200))
                break;  // a long queue ahead of the build, a replayed graph, or an error
        }
    }
    RECD_HIP(ctx, hipStreamSynchronize(ctx->stream));
    RECD_HIP(ctx, hipMemcpy(out, ctx->build_counts_dev, 3 * sizeof(int64_t), hipMemcpyDeviceToHost));
    return RECD_OK;
}

recd_status recd_last_ikjt_counts(recd_ctx *ctx, int64_t *host_U_M)
{
    if (!ctx || !host_U_M)
        return RECD_EINVAL;
    int64_t c[3];
    RECD_TRY(last_build_counts(ctx, c));
    host_U_M[0] = c[0];
    host_U_M[1] = c[1];
    return RECD_OK;
}

recd_status recd_last_ikjt_run_count(recd_ctx *ctx, int64_t *host_runs)
{
    if (!ctx || !host_runs)
        return RECD_EINVAL;
    int64_t c[3];
    RECD_TRY(last_build_counts(ctx, c));
    host_runs[0] = c[2];
    return RECD_OK;
}

const char *recd_last_error(const recd_ctx *ctx) { return ctx ? ctx->err.c_str() : "null context"; }

} // extern "C"
