// Segmented row gather-sum (the pooled embedding lookup), the inverse expand, and input validation.
//
// One kernel body serves the deduplicated lookup on an IKJT's unique lists, the non-deduplicated
// KJT lookup and both segment reductions of the backward pass: "for every list l, sum the table
// rows named by values[offsets[l] .. offsets[l+1]) and store the sum as row l of the output".
//
// Mapping to the machine (gfx950: 64-lane waves, 8 XCDs each with a private L2):
//   * a row of D elements is covered by LPR lanes x 16 bytes (x VPL vectors per lane when the row is
//     longer than 1 KiB); the 64/LPR lane groups of a wave take the ids of one list round-robin
//     (id k of the list goes to group k mod G) and are combined by a fixed butterfly at the end, so
//     the summation order is a function of the list alone, never of where the list sits in a batch;
//   * every load instruction of a wave therefore fetches G whole rows as 16-byte-per-lane
//     contiguous pieces, and UNR of them are issued before the first add to keep many rows in flight;
//   * work is handed out in items of CH consecutive lists from eight queues, queue q holding the
//     lists of the features f with f mod 8 = q.  A wave first drains the queue of the XCD it runs
//     on, so that the hot rows of a table stay in one XCD's L2, then helps the other queues.
//     The grid is persistent (a fixed number of blocks); the queues are atomic counters that the
//     last wave to leave resets, so no host-side knowledge of the number of unique lists is needed.
#include "recd_internal.h"

#include <hip/hip_fp16.h>

namespace {

constexpr int kNQ = 8;                          // work queues = XCDs
constexpr int kQF = RECD_F_PER_LAUNCH / kNQ;     // features per queue in one launch
constexpr int kCH = 4;                          // lists per work item
constexpr int kBlock = 256;
constexpr int kWavesPerBlock = kBlock / 64;

__device__ __forceinline__ int xcc_id()
{
    // XCC_ID hardware register, bits [3:0]: the XCD this wave runs on.  Only locality depends on it.
    int v;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID, 0, 4)" : "=s"(v));
    return v & (kNQ - 1);
}

__device__ __forceinline__ int64_t uniform64(int64_t v)
{
    // the value is the same in every lane: move it to scalar registers
    uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)(uint64_t)v);
    uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)((uint64_t)v >> 32));
    return (int64_t)(((uint64_t)hi << 32) | lo);
}

template <int TT> struct Elem;
template <> struct Elem<RECD_F32> { static constexpr int per_vec = 4; };
template <> struct Elem<RECD_F16> { static constexpr int per_vec = 8; };
template <> struct Elem<RECD_BF16> { static constexpr int per_vec = 8; };

__device__ __forceinline__ float bf16_to_f32(uint32_t h) { return __uint_as_float(h << 16); }
__device__ __forceinline__ uint32_t f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u)
        return 0x7fc0u;
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

// add the elements of one 16-byte vector into acc[0..per_vec)
template <int TT> __device__ __forceinline__ void accumulate(float *acc, const uint4 &v)
{
    if constexpr (TT == RECD_F32) {
        acc[0] += __uint_as_float(v.x);
        acc[1] += __uint_as_float(v.y);
        acc[2] += __uint_as_float(v.z);
        acc[3] += __uint_as_float(v.w);
    } else if constexpr (TT == RECD_F16) {
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; i++) {
            acc[2 * i] += __half2float(__ushort_as_half((unsigned short)(w[i] & 0xffffu)));
            acc[2 * i + 1] += __half2float(__ushort_as_half((unsigned short)(w[i] >> 16)));
        }
    } else {
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; i++) {
            acc[2 * i] += bf16_to_f32(w[i] & 0xffffu);
            acc[2 * i + 1] += bf16_to_f32(w[i] >> 16);
        }
    }
}

// store n fp32 accumulators (n = 4 or 8) as elements of type OT at dst (16-byte aligned pieces)
template <int OT, int N> __device__ __forceinline__ void store_row_piece(void *dst, const float *acc)
{
    if constexpr (OT == RECD_F32) {
#pragma unroll
        for (int i = 0; i < N; i += 4) {
            float4 o = make_float4(acc[i], acc[i + 1], acc[i + 2], acc[i + 3]);
            reinterpret_cast<float4 *>(dst)[i / 4] = o;
        }
    } else {
        static_assert(OT == RECD_F32 || N == 8, "16-bit outputs come from 16-bit tables");
        uint32_t w[4];
#pragma unroll
        for (int i = 0; i < 4; i++) {
            uint32_t lo, hi;
            if constexpr (OT == RECD_F16) {
                lo = __half_as_ushort(__float2half_rn(acc[2 * i]));
                hi = __half_as_ushort(__float2half_rn(acc[2 * i + 1]));
            } else {
                lo = f32_to_bf16(acc[2 * i]);
                hi = f32_to_bf16(acc[2 * i + 1]);
            }
            w[i] = lo | (hi << 16);
        }
        *reinterpret_cast<uint4 *>(dst) = make_uint4(w[0], w[1], w[2], w[3]);
    }
}

struct SegSumParams {
    TablePtrs tables;
    const void *values;
    const int64_t *offsets;
    const int64_t *list_off;
    int64_t lists_per_feature;
    int64_t list_base;
    void *out;
    uint32_t *ctr;  // [0..7] queue heads, [8] waves done
    int F;
    int D;
    int vecs_per_row;  // D / elements per 16-byte vector
};

template <int LPR, int VPL, int TT, int OT, typename IdxT>
__global__ __launch_bounds__(kBlock) void k_segsum(const SegSumParams p)
{
    constexpr int EPV = Elem<TT>::per_vec;
    constexpr int G = 64 / LPR;
    constexpr int UNR = (VPL == 1) ? 8 : (VPL == 2 ? 4 : 2);
    constexpr int NACC = EPV * VPL;

    __shared__ int64_t s_loff[RECD_F_PER_LAUNCH + 1];
    __shared__ int64_t s_qpref[kNQ][kQF + 1];

    const int tid = threadIdx.x;
    for (int f = tid; f <= p.F; f += kBlock)
        s_loff[f] = p.list_off ? p.list_off[f] : (int64_t)f * p.lists_per_feature;
    __syncthreads();
    if (tid < kNQ) {
        int64_t run = 0;
        s_qpref[tid][0] = 0;
        for (int k = 0; k < kQF; k++) {
            int f = tid + k * kNQ;
            if (f < p.F)
                run += s_loff[f + 1] - s_loff[f];
            s_qpref[tid][k + 1] = run;
        }
    }
    __syncthreads();

    const int lane = tid & 63;
    const int g = lane / LPR;       // lane group = which of the G rows of a load
    const int r = lane % LPR;       // 16-byte piece of the row
    const bool piece_ok = r < p.vecs_per_row || VPL > 1;
    const IdxT *values = static_cast<const IdxT *>(p.values);
    const int64_t row_bytes = (int64_t)p.D * (TT == RECD_F32 ? 4 : 2);
    const int64_t out_row_bytes = (int64_t)p.D * (OT == RECD_F32 ? 4 : 2);

    int q = xcc_id();
    for (int tried = 0; tried < kNQ;) {
        uint32_t item = 0;
        if (lane == 0)
            item = atomicAdd(&p.ctr[q], 1u);
        item = __builtin_amdgcn_readfirstlane(item);
        const int64_t total = s_qpref[q][kQF];
        int64_t t0 = (int64_t)item * kCH;
        if (t0 >= total) {
            q = (q + 1) & (kNQ - 1);
            tried++;
            continue;
        }
        int64_t t1 = t0 + kCH < total ? t0 + kCH : total;
        int k = 0;
        for (int64_t t = t0; t < t1; t++) {
            while (t >= s_qpref[q][k + 1])
                k++;
            const int f = q + k * kNQ;
            const int64_t l = p.list_base + s_loff[f] + (t - s_qpref[q][k]);
            const char *table = static_cast<const char *>(p.tables.p[f]);
            const int64_t start = uniform64(p.offsets[l]), end = uniform64(p.offsets[l + 1]);

            float acc[NACC];
#pragma unroll
            for (int i = 0; i < NACC; i++)
                acc[i] = 0.f;

            for (int64_t base = start; base < end; base += 64) {
                const int n = (int)((end - base) < 64 ? (end - base) : 64);
                int64_t my_id = 0;
                if (lane < n)
                    my_id = (int64_t)values[base + lane];
                for (int k0 = 0; k0 < n; k0 += G * UNR) {
                    uint4 v[UNR][VPL];
#pragma unroll
                    for (int u = 0; u < UNR; u++) {
                        const int idx = k0 + u * G + g;
                        const int64_t id = __shfl(my_id, idx & 63);
                        const char *src = table + id * row_bytes + (int64_t)r * 16;
#pragma unroll
                        for (int w = 0; w < VPL; w++) {
                            if (idx < n && piece_ok)
                                v[u][w] = *reinterpret_cast<const uint4 *>(src + (int64_t)w * LPR * 16);
                            else
                                v[u][w] = make_uint4(0, 0, 0, 0);
                        }
                    }
#pragma unroll
                    for (int u = 0; u < UNR; u++)
#pragma unroll
                        for (int w = 0; w < VPL; w++)
                            accumulate<TT>(acc + w * EPV, v[u][w]);
                }
            }
            // fold the G lane groups: fixed butterfly, group 0 ends up with the total
#pragma unroll
            for (int s = LPR; s < 64; s <<= 1)
#pragma unroll
                for (int i = 0; i < NACC; i++)
                    acc[i] += __shfl_xor(acc[i], s);

            if (g == 0 && piece_ok) {
                char *dst = static_cast<char *>(p.out) + l * out_row_bytes;
#pragma unroll
                for (int w = 0; w < VPL; w++) {
                    constexpr int OB = (OT == RECD_F32) ? EPV * 4 : 16;  // bytes this lane writes per vector
                    store_row_piece<OT, EPV>(dst + ((int64_t)w * LPR + r) * OB, acc + w * EPV);
                }
            }
        }
    }

    // the last wave to leave re-arms the queues for the next launch
    if (lane == 0) {
        __threadfence();
        const uint32_t waves = gridDim.x * kWavesPerBlock;
        if (atomicAdd(&p.ctr[kNQ], 1u) == waves - 1) {
            for (int i = 0; i <= kNQ; i++)
                atomicExch(&p.ctr[i], 0u);
        }
    }
}

template <int LPR, int VPL, int TT, int OT, typename IdxT>
void launch_one(hipStream_t st, int blocks, const SegSumParams &p)
{
    hipLaunchKernelGGL((k_segsum<LPR, VPL, TT, OT, IdxT>), dim3(blocks), dim3(kBlock), 0, st, p);
}

template <int TT, int OT, typename IdxT>
bool launch_shape(hipStream_t st, int blocks, int vecs, const SegSumParams &p)
{
    if (vecs <= 8) launch_one<8, 1, TT, OT, IdxT>(st, blocks, p);
    else if (vecs <= 16) launch_one<16, 1, TT, OT, IdxT>(st, blocks, p);
    else if (vecs <= 32) launch_one<32, 1, TT, OT, IdxT>(st, blocks, p);
    else if (vecs <= 64) launch_one<64, 1, TT, OT, IdxT>(st, blocks, p);
    else if (vecs == 128) launch_one<64, 2, TT, OT, IdxT>(st, blocks, p);
    else if (vecs == 256) launch_one<64, 4, TT, OT, IdxT>(st, blocks, p);
    else return false;
    return true;
}

// ---- expand: out[f,b,:] = pooled[feat_uoff[f] + inverse[f,b], :]  (16-byte pieces) ------------
__global__ __launch_bounds__(kBlock) void k_expand(const uint4 *__restrict__ pooled,
                                                   const int64_t *__restrict__ feat_uoff,
                                                   const int32_t *__restrict__ inverse,
                                                   uint4 *__restrict__ out, int64_t B,
                                                   int64_t n_rows, int vecs_per_row,
                                                   int rows_per_block)
{
    // a block copies rows_per_block consecutive output rows; thread t moves piece (t % vecs) of row
    // (t / vecs) and strides by blockDim/vecs rows
    const int64_t row0 = (int64_t)blockIdx.x * rows_per_block;
    const int lanes_rows = kBlock / vecs_per_row;  // rows moved per sweep (vecs_per_row <= 256)
    const int piece = threadIdx.x % vecs_per_row;
    const int sub = threadIdx.x / vecs_per_row;
    if (sub >= lanes_rows)
        return;
    for (int i = sub; i < rows_per_block; i += lanes_rows) {
        const int64_t row = row0 + i;
        if (row >= n_rows)
            break;
        const int64_t f = row / B;
        const int64_t u = feat_uoff[f] + (int64_t)inverse[row];
        out[row * vecs_per_row + piece] = pooled[u * vecs_per_row + piece];
    }
}

// ---- validation --------------------------------------------------------------------------------
// err[0] |= 1: offsets malformed, |= 2: id out of range
__global__ void k_validate_offsets(const int64_t *offsets, int64_t n_lists, int64_t N, int *err)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i == 0 && (offsets[0] != 0 || (N >= 0 && offsets[n_lists] != N)))
        atomicOr(err, 1);
    if (i < n_lists && offsets[i + 1] < offsets[i])
        atomicOr(err, 1);
}

__global__ void k_validate_ids(const int64_t *values, const int64_t *offsets,
                               const int64_t *list_off, int64_t lists_per_feature, int f,
                               int64_t rows_f, int *err)
{
    // ids of feature f: values[offsets[first list] .. offsets[last list + 1])
    const int64_t l0 = list_off ? list_off[f] : (int64_t)f * lists_per_feature;
    const int64_t l1 = list_off ? list_off[f + 1] : (int64_t)(f + 1) * lists_per_feature;
    const int64_t j0 = offsets[l0], j1 = offsets[l1];
    for (int64_t j = j0 + (int64_t)blockIdx.x * blockDim.x + threadIdx.x; j < j1;
         j += (int64_t)gridDim.x * blockDim.x)
        if (values[j] < 0 || values[j] >= rows_f)
            atomicOr(err, 2);
}

__global__ void k_read_i64(const int64_t *src, int64_t *dst) { *dst = *src; }

} // namespace

recd_status recd_launch_segsum(recd_ctx *ctx, const SegSumArgs &a)
{
    SegSumParams p;
    p.tables = a.tables;
    p.values = a.values;
    p.offsets = a.offsets;
    p.list_off = a.list_off;
    p.lists_per_feature = a.lists_per_feature;
    p.list_base = a.list_base;
    p.out = a.out;
    p.ctr = ctx->queue_ctr;
    p.F = a.F;
    p.D = a.D;
    const int epv = a.table_dt == RECD_F32 ? 4 : 8;
    p.vecs_per_row = a.D / epv;
    const int blocks = ctx->num_cu * 8;
    bool ok = false;
    hipStream_t st = ctx->stream;
    const int v = p.vecs_per_row;
    if (a.values_are_i32) {
        if (a.table_dt == RECD_F32 && a.out_dt == RECD_F32)
            ok = launch_shape<RECD_F32, RECD_F32, int32_t>(st, blocks, v, p);
    } else if (a.table_dt == RECD_F32 && a.out_dt == RECD_F32)
        ok = launch_shape<RECD_F32, RECD_F32, int64_t>(st, blocks, v, p);
    else if (a.table_dt == RECD_F16 && a.out_dt == RECD_F16)
        ok = launch_shape<RECD_F16, RECD_F16, int64_t>(st, blocks, v, p);
    else if (a.table_dt == RECD_F16 && a.out_dt == RECD_F32)
        ok = launch_shape<RECD_F16, RECD_F32, int64_t>(st, blocks, v, p);
    else if (a.table_dt == RECD_BF16 && a.out_dt == RECD_BF16)
        ok = launch_shape<RECD_BF16, RECD_BF16, int64_t>(st, blocks, v, p);
    else if (a.table_dt == RECD_BF16 && a.out_dt == RECD_F32)
        ok = launch_shape<RECD_BF16, RECD_F32, int64_t>(st, blocks, v, p);
    if (!ok)
        return recd_fail(ctx, RECD_EINVAL, "unsupported row shape: D=%d table dtype %d out dtype %d",
                         a.D, (int)a.table_dt, (int)a.out_dt);
    RECD_HIP(ctx, hipGetLastError());
    return RECD_OK;
}

static recd_status check_lookup_shape(recd_ctx *ctx, int F, int D, recd_dtype table_dt,
                                      recd_dtype out_dt)
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
    const size_t vecs = rb / 16;
    if (vecs > 64 && vecs != 128 && vecs != 256)
        return recd_fail(ctx, RECD_EINVAL, "D=%d: rows above 1 KiB must be 2 KiB or 4 KiB", D);
    return RECD_OK;
}

// Runs the device checks and returns RECD_EBOUNDS when they fail.  Synchronises.
static recd_status validate_lists(recd_ctx *ctx, int F, const int64_t *rows, const int64_t *values,
                                  const int64_t *offsets, const int64_t *list_off,
                                  int64_t lists_per_feature, int64_t n_lists_host, int64_t N)
{
    RECD_TRY(recd_reserve(ctx, 512));
    int *err = reinterpret_cast<int *>(ctx->ws);
    RECD_HIP(ctx, hipMemsetAsync(err, 0, sizeof(int), ctx->stream));
    if (n_lists_host >= 0) {
        const int64_t blocks = (n_lists_host + 1 + 255) / 256;
        hipLaunchKernelGGL(k_validate_offsets, dim3((unsigned)blocks), dim3(256), 0, ctx->stream,
                           offsets, n_lists_host, N, err);
    }
    ctx->host_pinned[0] = 0;
    RECD_HIP(ctx, hipMemcpyAsync(ctx->host_pinned, err, sizeof(int), hipMemcpyDeviceToHost, ctx->stream));
    RECD_HIP(ctx, hipStreamSynchronize(ctx->stream));
    if ((int)ctx->host_pinned[0] & 1)
        return recd_fail(ctx, RECD_EBOUNDS, "offsets are not a valid KJT offsets slice");
    if (rows && values) {
        for (int f = 0; f < F; f++)
            hipLaunchKernelGGL(k_validate_ids, dim3(64), dim3(256), 0, ctx->stream, values, offsets,
                               list_off, lists_per_feature, f, rows[f], err);
        RECD_HIP(ctx, hipMemcpyAsync(ctx->host_pinned, err, sizeof(int), hipMemcpyDeviceToHost, ctx->stream));
        RECD_HIP(ctx, hipStreamSynchronize(ctx->stream));
        if ((int)ctx->host_pinned[0] & 2)
            return recd_fail(ctx, RECD_EBOUNDS, "an id lies outside its embedding table");
    }
    return RECD_OK;
}

recd_status recd_validate_kjt_offsets(recd_ctx *ctx, int F, int64_t B, int64_t N, const int64_t *offsets)
{
    return validate_lists(ctx, F, nullptr, nullptr, offsets, nullptr, B, (int64_t)F * B, N);
}

extern "C" {

recd_status recd_pooled_lookup_unique(recd_ctx *ctx, int F, int D, recd_dtype table_dt,
                                      recd_dtype out_dt, const void *const *tables,
                                      const int64_t *rows, const int64_t *u_values,
                                      const int64_t *u_offsets, const int64_t *feat_uoff,
                                      int64_t max_lists, void *pooled)
{
    RECD_TRY(check_lookup_shape(ctx, F, D, table_dt, out_dt));
    if (max_lists < 0)
        return recd_fail(ctx, RECD_EINVAL, "max_lists < 0");
    if (F == 0 || max_lists == 0)
        return RECD_OK;
    if (!tables || !u_values || !u_offsets || !feat_uoff || !pooled)
        return recd_fail(ctx, RECD_EINVAL, "null pointer argument");
    for (int f = 0; f < F; f++)
        if (!tables[f])
            return recd_fail(ctx, RECD_EINVAL, "tables[%d] is null", f);
    RECD_HIP(ctx, hipSetDevice(ctx->device));
    if (ctx->validate) {
        if (!rows)
            return recd_fail(ctx, RECD_EINVAL, "validation needs rows[]");
        // U lives on the device: fetch it to size the offsets check
        RECD_TRY(recd_reserve(ctx, 512));
        hipLaunchKernelGGL(k_read_i64, dim3(1), dim3(1), 0, ctx->stream, feat_uoff + F,
                           reinterpret_cast<int64_t *>(ctx->ws + 256));
        RECD_HIP(ctx, hipMemcpyAsync(ctx->host_pinned + 1, ctx->ws + 256, 8, hipMemcpyDeviceToHost, ctx->stream));
        RECD_HIP(ctx, hipStreamSynchronize(ctx->stream));
        const int64_t U = ctx->host_pinned[1];
        if (U < 0 || U > max_lists)
            return recd_fail(ctx, RECD_ECAPACITY, "U=%lld exceeds max_lists=%lld", (long long)U,
                             (long long)max_lists);
        RECD_TRY(validate_lists(ctx, F, rows, u_values, u_offsets, feat_uoff, 0, U, -1));
    }
    for (int f0 = 0; f0 < F; f0 += RECD_F_PER_LAUNCH) {
        SegSumArgs a{};
        a.F = F - f0 < RECD_F_PER_LAUNCH ? F - f0 : RECD_F_PER_LAUNCH;
        a.D = D;
        a.table_dt = table_dt;
        a.out_dt = out_dt;
        for (int f = 0; f < a.F; f++)
            a.tables.p[f] = tables[f0 + f];
        a.values = u_values;
        a.values_are_i32 = 0;
        a.offsets = u_offsets;
        a.list_off = feat_uoff + f0;
        a.out = pooled;
        RECD_TRY(recd_launch_segsum(ctx, a));
    }
    return RECD_OK;
}

recd_status recd_kjt_pooled_lookup(recd_ctx *ctx, int F, int64_t B, int D, recd_dtype table_dt,
                                   recd_dtype out_dt, const void *const *tables,
                                   const int64_t *rows, const int64_t *values,
                                   const int64_t *offsets, void *out)
{
    RECD_TRY(check_lookup_shape(ctx, F, D, table_dt, out_dt));
    if (B < 0)
        return recd_fail(ctx, RECD_EINVAL, "B < 0");
    if (F == 0 || B == 0)
        return RECD_OK;
    if (!tables || !values || !offsets || !out)
        return recd_fail(ctx, RECD_EINVAL, "null pointer argument");
    for (int f = 0; f < F; f++)
        if (!tables[f])
            return recd_fail(ctx, RECD_EINVAL, "tables[%d] is null", f);
    RECD_HIP(ctx, hipSetDevice(ctx->device));
    if (ctx->validate) {
        if (!rows)
            return recd_fail(ctx, RECD_EINVAL, "validation needs rows[]");
        RECD_TRY(validate_lists(ctx, F, rows, values, offsets, nullptr, B, (int64_t)F * B, -1));
    }
    for (int f0 = 0; f0 < F; f0 += RECD_F_PER_LAUNCH) {
        SegSumArgs a{};
        a.F = F - f0 < RECD_F_PER_LAUNCH ? F - f0 : RECD_F_PER_LAUNCH;
        a.D = D;
        a.table_dt = table_dt;
        a.out_dt = out_dt;
        for (int f = 0; f < a.F; f++)
            a.tables.p[f] = tables[f0 + f];
        a.values = values;
        a.values_are_i32 = 0;
        a.offsets = offsets;
        a.list_off = nullptr;
        a.lists_per_feature = B;
        a.list_base = (int64_t)f0 * B;
        a.out = out;
        RECD_TRY(recd_launch_segsum(ctx, a));
    }
    return RECD_OK;
}

recd_status recd_expand_inverse(recd_ctx *ctx, int F, int64_t B, int D, recd_dtype dt,
                                const void *pooled, const int64_t *feat_uoff,
                                const int32_t *inverse, void *out)
{
    RECD_TRY(check_lookup_shape(ctx, F, D, dt, dt));
    if (B < 0)
        return recd_fail(ctx, RECD_EINVAL, "B < 0");
    if (F == 0 || B == 0)
        return RECD_OK;
    if (!pooled || !feat_uoff || !inverse || !out)
        return recd_fail(ctx, RECD_EINVAL, "null pointer argument");
    RECD_HIP(ctx, hipSetDevice(ctx->device));
    const int vecs = (int)((size_t)D * elem_size(dt) / 16);
    const int64_t n_rows = (int64_t)F * B;
    const int rows_per_block = 32;
    const int64_t blocks = (n_rows + rows_per_block - 1) / rows_per_block;
    if (blocks > 0x7fffffff)
        return recd_fail(ctx, RECD_EINVAL, "F*B too large");
    hipLaunchKernelGGL(k_expand, dim3((unsigned)blocks), dim3(kBlock), 0, ctx->stream,
                       static_cast<const uint4 *>(pooled), feat_uoff, inverse,
                       static_cast<uint4 *>(out), B, n_rows, vecs, rows_per_block);
    RECD_HIP(ctx, hipGetLastError());
    return RECD_OK;
}

} // extern "C"
