// Unpooled (sequence) embedding lookup and the jagged index select.
//
// A sequence feature keeps one activation row per id instead of a pooled sum (Sec. 2.2).  With an
// IKJT the rows are gathered for the ids of the unique lists only (Sec. 5 "EMB Inputs and
// Activations") and a jagged index select then rebuilds the KJT-shaped activations by copying, for
// every sample, the slice of its unique list (Sec. 5 "Jagged Index Select"): no padding of the
// jagged dimension to dense.
//
// Both kernels are pure 16-byte-piece copies, bound by HBM traffic, and follow the shape of the
// pooled expand: a row is covered by `vecs` consecutive threads, a thread first issues the loads of
// all its kRPT rows and only then stores them, so that kRPT * (256 / vecs) rows are in flight per
// block.
//   gather:  positions (ids) are dealt to blocks in tiles; the feature of a position - which table
//            to read - is found from the F+1 position bounds kept in LDS (one search per tile, a
//            short walk only for tiles that straddle a feature boundary).
//   jagged:  a block owns a few consecutive KJT rows, folds neighbours that share a unique slot
//            into runs (read once, stored once per member) and numbers the rows to read flat
//            across its runs, so long and short lists load the threads alike.
#include "recd_internal.h"

#include <hip/hip_fp16.h>

namespace {

constexpr int kBlock = 256;
constexpr int kRPT = 8;        // rows a thread has in flight
constexpr int kXcds = 8;       // accelerator dies, each with a private L2
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// pb[f] = position of the first id of feature f, pb[F] = one past the last id
__global__ void k_seq_bounds(const int64_t *__restrict__ offsets, const int64_t *__restrict__ list_off,
                             int64_t lists_per_feature, int F, int64_t *__restrict__ pb)
{
    const int f = blockIdx.x * blockDim.x + threadIdx.x;
    if (f <= F)
        pb[f] = offsets[list_off ? list_off[f] : (int64_t)f * lists_per_feature];
}

__device__ __forceinline__ u32x4 widen_lo(const u32x4 &v, int conv)
{
    // elements 0..3 of eight 16-bit values as fp32 bit patterns
    u32x4 r;
    if (conv == 2) {
        r.x = v.x << 16; r.y = v.x & 0xffff0000u; r.z = v.y << 16; r.w = v.y & 0xffff0000u;
    } else {
        r.x = __float_as_uint(__half2float(__ushort_as_half((unsigned short)(v.x & 0xffffu))));
        r.y = __float_as_uint(__half2float(__ushort_as_half((unsigned short)(v.x >> 16))));
        r.z = __float_as_uint(__half2float(__ushort_as_half((unsigned short)(v.y & 0xffffu))));
        r.w = __float_as_uint(__half2float(__ushort_as_half((unsigned short)(v.y >> 16))));
    }
    return r;
}

// CONV 0: out rows have the table's element type (16-byte pieces copied as they are);
//      1: fp16 table, fp32 out; 2: bf16 table, fp32 out (both exact).
// STREAM: the output is written with non-temporal stores (nothing on this path reads it again).
template <int CONV, bool STREAM>
__global__ __launch_bounds__(kBlock) void k_seq_gather(TablePtrs tables, int Fc,
                                                       const int64_t *__restrict__ pb,
                                                       const int64_t *__restrict__ values,
                                                       u32x4 *__restrict__ out, int vecs,
                                                       int64_t out_rows_cap)
{
    __shared__ int64_t pb_s[RECD_F_PER_LAUNCH + 1];
    __shared__ const void *tab_s[RECD_F_PER_LAUNCH];
    for (int i = threadIdx.x; i <= Fc; i += kBlock)
        pb_s[i] = pb[i];
    for (int i = threadIdx.x; i < Fc; i += kBlock)
        tab_s[i] = tables.p[i];
    __syncthreads();
    const int rows_per_sweep = kBlock / vecs;  // vecs <= 256
    const int piece = threadIdx.x % vecs;
    const int sub = threadIdx.x / vecs;
    if (sub >= rows_per_sweep)
        return;
    const int64_t tile_rows = (int64_t)rows_per_sweep * kRPT;
    const int64_t lo = pb_s[0];
    int64_t hi = pb_s[Fc];
    if (hi > out_rows_cap)
        hi = out_rows_cap;
    // KJT path (STREAM): within one sweep of the grid every XCD (consecutive blocks go to consecutive
    // XCDs) takes a contiguous eighth of the tiles: neighbouring positions, which in a
    // session-clustered batch mostly name the same table rows, then gather through the same L2
    // (a quarter of the HBM reads at the benchmark shape).  The unique lists hold few repeats and
    // measure faster with the plain order.
    const uint32_t per_xcd = gridDim.x / kXcds;  // the grid is a multiple of kXcds
    const uint32_t item = STREAM ? (blockIdx.x % kXcds) * per_xcd + blockIdx.x / kXcds : blockIdx.x;
    for (int64_t t0 = lo + (int64_t)item * tile_rows; t0 < hi; t0 += (int64_t)gridDim.x * tile_rows) {
        // feature of the tile's first position: the last f with pb_s[f] <= t0 (t0 < pb_s[Fc], so
        // that feature is not empty)
        int f0 = 0;
#pragma unroll
        for (int s = RECD_F_PER_LAUNCH / 2; s >= 1; s >>= 1)
            if (f0 + s < Fc && pb_s[f0 + s] <= t0)
                f0 += s;
        const int64_t next = pb_s[f0 + 1];
        int64_t pos[kRPT], ids[kRPT];
#pragma unroll
        for (int k = 0; k < kRPT; k++) {
            const int64_t p = t0 + k * rows_per_sweep + sub;
            pos[k] = p < hi ? p : hi - 1;  // clamped: loads are unconditional, stores predicated
            ids[k] = values[pos[k]];
        }
        u32x4 v[kRPT];
#pragma unroll
        for (int k = 0; k < kRPT; k++) {
            int f = f0;
            if (pos[k] >= next) {
                f = f0 + 1;
                while (pos[k] >= pb_s[f + 1])  // ends: pos[k] < pb_s[Fc]
                    f++;
            }
            v[k] = static_cast<const u32x4 *>(tab_s[f])[ids[k] * vecs + piece];
        }
#pragma unroll
        for (int k = 0; k < kRPT; k++) {
            const int64_t p = t0 + k * rows_per_sweep + sub;
            if (p < hi) {
                if (CONV == 0) {
                    u32x4 *dst = &out[p * vecs + piece];
                    if (STREAM)
                        __builtin_nontemporal_store(v[k], dst);
                    else
                        *dst = v[k];
                } else {
                    u32x4 *dst = &out[(p * vecs + piece) * 2];
                    u32x4 hi4;
                    hi4.x = v[k].z; hi4.y = v[k].w; hi4.z = 0; hi4.w = 0;
                    const u32x4 a = widen_lo(v[k], CONV), b = widen_lo(hi4, CONV);
                    if (STREAM) {
                        __builtin_nontemporal_store(a, dst);
                        __builtin_nontemporal_store(b, dst + 1);
                    } else {
                        dst[0] = a;
                        dst[1] = b;
                    }
                }
            }
        }
    }
}

// out[offsets[l] + t, :] = emb[u_offsets[feat_uoff[f] + inverse[l]] + t, :] for the rows
// l = f*B + b of the KJT, t in [0, offsets[l+1] - offsets[l]).
// A block owns LISTS <= 64 consecutive KJT rows.  Its first wave folds neighbouring rows that point
// at the same unique slot into runs (the samples of a session are adjacent, so most duplicates
// are): a run is read once and stored once per member.  The rows to read are numbered flat across
// the block's runs, so long and short lists load the threads alike; a thread finds the run of its
// row by a fixed-depth search of the runs' flat starts in LDS.
template <int LISTS, int RPT>
__global__ __launch_bounds__(kBlock) void k_jagged_expand(const u32x4 *__restrict__ emb,
                                                          const int64_t *__restrict__ u_offsets,
                                                          const int64_t *__restrict__ feat_uoff,
                                                          const int32_t *__restrict__ inverse,
                                                          const int64_t *__restrict__ offsets,
                                                          u32x4 *__restrict__ out, uint32_t B,
                                                          uint32_t L, int vecs, int64_t emb_rows_cap,
                                                          int64_t out_rows)
{
    static_assert(LISTS <= 64 && (LISTS & (LISTS - 1)) == 0, "one wave prepares the runs");
    __shared__ int64_t run_src[LISTS];   // first emb row of the run's list
    __shared__ uint32_t run_dst[LISTS];  // first output row of the run, relative to the block's
    __shared__ uint32_t run_len[LISTS];  // ids per member list
    __shared__ uint32_t run_cnt[LISTS];  // member lists
    __shared__ uint32_t run_rel[LISTS + 1];  // flat number of the run's first row to read
    __shared__ uint32_t n_runs_s;
    // Consecutive blocks go to consecutive XCDs.  Each XCD takes one contiguous eighth of the rows
    // instead, so that blocks which split a run of duplicates read its unique list through the
    // same L2.
    const uint32_t per_xcd = gridDim.x / kXcds;  // the grid is a multiple of kXcds
    const uint32_t item = (blockIdx.x % kXcds) * per_xcd + blockIdx.x / kXcds;
    if ((uint64_t)item * LISTS >= L)
        return;
    const uint32_t l0 = item * LISTS;
    const uint32_t nl = L - l0 < (uint32_t)LISTS ? L - l0 : (uint32_t)LISTS;
    const int64_t d0 = offsets[l0];
    if (threadIdx.x < 64) {
        const uint32_t i = threadIdx.x;
        const bool live = i < nl;
        int64_t u = -1, src = 0;
        uint32_t dst = 0, len = 0;
        if (live) {
            const uint32_t l = l0 + i;
            u = feat_uoff[l / B] + inverse[l];  // slot index, distinct across features
            src = u_offsets[u];
            const int64_t o0 = offsets[l];
            dst = (uint32_t)(o0 - d0);
            len = (uint32_t)(offsets[l + 1] - o0);
        }
        const int64_t prev = __shfl_up(u, 1);
        const bool head = live && (i == 0 || u != prev);
        const uint64_t heads = __ballot(head);
        uint32_t incl = head ? len : 0;  // inclusive scan over the run heads' lengths
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const uint32_t t = __shfl_up(incl, d);
            if (i >= (uint32_t)d)
                incl += t;
        }
        if (head) {
            const uint32_t r = __popcll(heads & ((1ull << i) - 1));
            const uint64_t above = i == 63 ? 0 : heads >> (i + 1);
            const uint32_t next = above ? i + 1 + (uint32_t)__builtin_ctzll(above) : nl;
            run_src[r] = src;
            run_dst[r] = dst;
            run_len[r] = len;
            run_cnt[r] = next - i;
            run_rel[r] = incl - len;
        }
        if (i == 63) {
            run_rel[__popcll(heads)] = incl;
            n_runs_s = __popcll(heads);
        }
    }
    __syncthreads();
    const uint32_t n_runs = n_runs_s;
    const uint32_t total = run_rel[n_runs];
    const uint32_t rows_per_sweep = kBlock / vecs;
    const uint32_t piece = threadIdx.x % vecs;
    const uint32_t sub = threadIdx.x / vecs;
    if (sub >= rows_per_sweep)
        return;
    for (uint32_t base = 0; base < total; base += rows_per_sweep * RPT) {
        u32x4 v[RPT] = {};
        uint32_t run[RPT] = {};
#pragma unroll
        for (int k = 0; k < RPT; k++) {
            if (base + k * rows_per_sweep >= total)
                break;  // the whole sweep lies beyond the block's rows (same decision in every thread)
            const uint32_t r = base + k * rows_per_sweep + sub;
            const uint32_t rc = r < total ? r : total - 1;
            // the last run i with run_rel[i] <= rc; rc < run_rel[n_runs], so run i is not empty
            uint32_t i = 0;
#pragma unroll
            for (uint32_t s = LISTS / 2; s >= 1; s >>= 1)
                if (i + s < n_runs && run_rel[i + s] <= rc)
                    i += s;
            run[k] = i;
            int64_t srow = run_src[i] + (rc - run_rel[i]);
            // a slot whose list is shorter than the row (malformed input) must not read past emb
            srow = srow < emb_rows_cap ? srow : emb_rows_cap - 1;
            srow = srow < 0 ? 0 : srow;
            v[k] = emb[srow * vecs + piece];
        }
#pragma unroll
        for (int k = 0; k < RPT; k++) {
            const uint32_t r = base + k * rows_per_sweep + sub;
            if (r < total) {
                const uint32_t i = run[k];
                const uint32_t len = run_len[i], cnt = run_cnt[i];
                int64_t row = d0 + run_dst[i] + (r - run_rel[i]);
                for (uint32_t j = 0; j < cnt; j++, row += len)
                    if (row < out_rows)  // false only for malformed input (members of unequal length)
                        __builtin_nontemporal_store(v[k], &out[row * vecs + piece]);
            }
        }
    }
}

// err[0] |= 8: a row's slot holds a list of another length
__global__ void k_validate_jagged(const int64_t *u_offsets, const int64_t *feat_uoff,
                                  const int32_t *inverse, const int64_t *offsets, int64_t B, int64_t L,
                                  int *err)
{
    const int64_t l = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (l < L) {
        const int64_t u = feat_uoff[l / B] + inverse[l];
        if (u_offsets[u + 1] - u_offsets[u] != offsets[l + 1] - offsets[l])
            atomicOr(err, 8);
    }
}

recd_status check_row_shape(recd_ctx *ctx, int F, int D, recd_dtype table_dt, recd_dtype out_dt)
{
    if (!ctx)
        return RECD_EINVAL;
    if (F < 0 || F > RECD_MAX_FEATURES)
        return recd_fail(ctx, RECD_EINVAL, "F=%d outside [0,%d]", F, RECD_MAX_FEATURES);
    if ((int)table_dt < 0 || (int)table_dt > 2 || (int)out_dt < 0 || (int)out_dt > 2)
        return recd_fail(ctx, RECD_EINVAL, "unknown dtype");
    if (out_dt != table_dt && out_dt != RECD_F32)
        return recd_fail(ctx, RECD_EINVAL, "out_dt must be the table dtype or RECD_F32");
    const size_t rb = (size_t)D * elem_size(table_dt);
    if (D <= 0 || rb % 16 != 0 || rb > RECD_MAX_ROW_BYTES)
        return recd_fail(ctx, RECD_EINVAL, "D=%d: row bytes %zu must be a multiple of 16 and <= %d", D,
                         rb, RECD_MAX_ROW_BYTES);
    return RECD_OK;
}

// Gathers the rows of every position of the lists [list_off[f], list_off[f+1]) (or the B rows of
// feature f when list_off is null) into out[position, :].
recd_status sequence_gather(recd_ctx *ctx, int F, int D, recd_dtype table_dt, recd_dtype out_dt,
                            const void *const *tables, const int64_t *values, const int64_t *offsets,
                            const int64_t *list_off, int64_t lists_per_feature, int64_t rows_cap,
                            void *out, bool stream_out)
{
    RECD_TRY(recd_reserve(ctx, 256 + (size_t)(F + 1) * sizeof(int64_t)));
    ctx->plan.valid = false;  // the position bounds below overwrite the workspace a backward plan would live in
    int64_t *pb = reinterpret_cast<int64_t *>(ctx->ws);
    hipLaunchKernelGGL(k_seq_bounds, dim3((unsigned)(F / 256 + 1)), dim3(256), 0, ctx->stream, offsets,
                       list_off, lists_per_feature, F, pb);
    const int vecs = (int)((size_t)D * elem_size(table_dt) / 16);
    const int64_t tile_rows = (int64_t)(kBlock / vecs) * kRPT;
    int64_t blocks = (rows_cap + tile_rows - 1) / tile_rows;
    // rows_cap is exact for the KJT (one block per tile measures fastest); for unique lists it may
    // be a loose bound, so the grid is capped and the kernel strides over the tiles
    const int64_t cap = stream_out ? ((int64_t)1 << 30) : (int64_t)ctx->num_cu * 8 * 16;
    if (blocks > cap)
        blocks = cap;
    blocks = (blocks + kXcds - 1) / kXcds * kXcds;
    const int conv = out_dt == table_dt ? 0 : (table_dt == RECD_F16 ? 1 : 2);
    for (int f0 = 0; f0 < F; f0 += RECD_F_PER_LAUNCH) {
        const int fc = F - f0 < RECD_F_PER_LAUNCH ? F - f0 : RECD_F_PER_LAUNCH;
        TablePtrs t{};
        for (int f = 0; f < fc; f++)
            t.p[f] = tables[f0 + f];
#define RECD_SEQ_LAUNCH(CONV, STREAM)                                                              \
    hipLaunchKernelGGL((k_seq_gather<CONV, STREAM>), dim3((unsigned)blocks), dim3(kBlock), 0,       \
                       ctx->stream, t, fc, pb + f0, static_cast<const int64_t *>(values),           \
                       static_cast<u32x4 *>(out), vecs, rows_cap)
        if (conv == 0 && stream_out)
            RECD_SEQ_LAUNCH(0, true);
        else if (conv == 0)
            RECD_SEQ_LAUNCH(0, false);
        else if (conv == 1 && stream_out)
            RECD_SEQ_LAUNCH(1, true);
        else if (conv == 1)
            RECD_SEQ_LAUNCH(1, false);
        else if (stream_out)
            RECD_SEQ_LAUNCH(2, true);
        else
            RECD_SEQ_LAUNCH(2, false);
#undef RECD_SEQ_LAUNCH
    }
    RECD_HIP(ctx, hipGetLastError());
    return RECD_OK;
}

} // namespace

extern "C" {

recd_status recd_sequence_lookup_unique(recd_ctx *ctx, int F, int D, recd_dtype table_dt,
                                        recd_dtype out_dt, const void *const *tables,
                                        const int64_t *rows, const int64_t *u_values,
                                        const int64_t *u_offsets, const int64_t *feat_uoff,
                                        int64_t max_lists, int64_t M_cap, void *emb)
{
    RECD_TRY(check_row_shape(ctx, F, D, table_dt, out_dt));
    RECD_TRY(recd_check_rows(ctx, F, rows));
    if (max_lists < 0 || M_cap < 0)
        return recd_fail(ctx, RECD_EINVAL, "max_lists or M_cap < 0");
    if (F == 0 || M_cap == 0)
        return RECD_OK;
    if (!tables || !u_values || !u_offsets || !feat_uoff || !emb)
        return recd_fail(ctx, RECD_EINVAL, "null pointer argument");
    for (int f = 0; f < F; f++)
        if (!tables[f])
            return recd_fail(ctx, RECD_EINVAL, "tables[%d] is null", f);
    RECD_HIP(ctx, hipSetDevice(ctx->device));
    if (ctx->validate)
        RECD_TRY(recd_validate_unique_lists(ctx, F, rows, u_values, u_offsets, feat_uoff, max_lists, M_cap));
    return sequence_gather(ctx, F, D, table_dt, out_dt, tables, u_values, u_offsets, feat_uoff, 0, M_cap,
                           emb, false);
}

recd_status recd_kjt_sequence_lookup(recd_ctx *ctx, int F, int64_t B, int64_t N, int D,
                                     recd_dtype table_dt, recd_dtype out_dt,
                                     const void *const *tables, const int64_t *rows,
                                     const int64_t *values, const int64_t *offsets, void *out)
{
    RECD_TRY(check_row_shape(ctx, F, D, table_dt, out_dt));
    RECD_TRY(recd_check_rows(ctx, F, rows));
    if (B < 0 || N < 0)
        return recd_fail(ctx, RECD_EINVAL, "B or N < 0");
    if (F == 0 || B == 0 || N == 0)
        return RECD_OK;
    if (!tables || !values || !offsets || !out)
        return recd_fail(ctx, RECD_EINVAL, "null pointer argument");
    for (int f = 0; f < F; f++)
        if (!tables[f])
            return recd_fail(ctx, RECD_EINVAL, "tables[%d] is null", f);
    RECD_HIP(ctx, hipSetDevice(ctx->device));
    if (ctx->validate)
        RECD_TRY(recd_validate_kjt_lists(ctx, F, B, N, rows, values, offsets));
    return sequence_gather(ctx, F, D, table_dt, out_dt, tables, values, offsets, nullptr, B, N, out, true);
}

recd_status recd_jagged_expand_inverse(recd_ctx *ctx, int F, int64_t B, int64_t N, int D,
                                       recd_dtype dt, const void *emb, int64_t M_cap,
                                       const int64_t *u_offsets, const int64_t *feat_uoff,
                                       const int32_t *inverse, const int64_t *offsets, void *out)
{
    RECD_TRY(check_row_shape(ctx, F, D, dt, dt));
    if (B < 0 || N < 0 || M_cap < 0)
        return recd_fail(ctx, RECD_EINVAL, "B, N or M_cap < 0");
    if (F == 0 || B == 0 || N == 0)
        return RECD_OK;
    if (!emb || !u_offsets || !feat_uoff || !inverse || !offsets || !out)
        return recd_fail(ctx, RECD_EINVAL, "null pointer argument");
    if (M_cap == 0)
        return recd_fail(ctx, RECD_EINVAL, "M_cap = 0 with N > 0");
    const int64_t L = (int64_t)F * B;
    if (L >= (int64_t)1 << 31 || N >= (int64_t)1 << 31)
        return recd_fail(ctx, RECD_EINVAL, "F*B and N must stay below 2^31");
    RECD_HIP(ctx, hipSetDevice(ctx->device));
    if (ctx->validate) {
        RECD_TRY(recd_validate_kjt_offsets(ctx, F, B, N, offsets));
        RECD_TRY(recd_validate_inverse(ctx, F, B, feat_uoff, inverse));
        int *err = reinterpret_cast<int *>(ctx->ws);
        RECD_HIP(ctx, hipMemsetAsync(err, 0, sizeof(int), ctx->stream));
        hipLaunchKernelGGL(k_validate_jagged, dim3((unsigned)((L + 255) / 256)), dim3(256), 0, ctx->stream,
                           u_offsets, feat_uoff, inverse, offsets, B, L, err);
        ctx->host_pinned[0] = 0;
        RECD_HIP(ctx, hipMemcpyAsync(ctx->host_pinned, err, sizeof(int), hipMemcpyDeviceToHost, ctx->stream));
        RECD_HIP(ctx, hipStreamSynchronize(ctx->stream));
        if ((int)ctx->host_pinned[0] & 8)
            return recd_fail(ctx, RECD_EBOUNDS, "a row's unique slot holds a list of another length");
    }
    const int vecs = (int)((size_t)D * elem_size(dt) / 16);
    // Lists per block: about 128 rows to read and write per block.  Small blocks keep the region
    // that the resident blocks write at any one time compact, which measures faster than large
    // blocks although runs of duplicates are cut at block borders.
    const double avg = (double)N / (double)L;
    int lists = 2;
    while (lists < 64 && 2.0 * lists * avg <= 192.0)
        lists *= 2;
#define JAG(LISTS)                                                                                \
    hipLaunchKernelGGL((k_jagged_expand<LISTS, kRPT>),                                             \
                       dim3((unsigned)(((L + LISTS - 1) / LISTS + kXcds - 1) / kXcds * kXcds)),     \
                       dim3(kBlock), 0, ctx->stream, static_cast<const u32x4 *>(emb), u_offsets,   \
                       feat_uoff, inverse, offsets, static_cast<u32x4 *>(out), (uint32_t)B,        \
                       (uint32_t)L, vecs, M_cap, N)
    switch (lists) {
    case 2: JAG(2); break;
    case 4: JAG(4); break;
    case 8: JAG(8); break;
    case 16: JAG(16); break;
    case 32: JAG(32); break;
    default: JAG(64); break;
    }
#undef JAG
    RECD_HIP(ctx, hipGetLastError());
    return RECD_OK;
}

} // extern "C"
