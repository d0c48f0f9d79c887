// Segmented row gather-sum (the pooled embedding lookup), the inverse expand, and input validation.
//
// One kernel body serves the deduplicated lookup on an IKJT's unique lists, the non-deduplicated
// KJT lookup and both segment reductions of the backward pass: "for every list l, sum the table
// rows named by values[offsets[l] .. offsets[l+1]) and store the sum as row l of the output".
//
// Mapping to the machine (gfx950: 64-lane waves, 8 XCDs each with a private L2):
//   * a row of D elements is covered by LPR lanes x 16 bytes (x VPL vectors per lane when the row is
//     longer than 1 KiB).  The G = 64/LPR lane groups of a wave take the ids of a list round-robin
//     (id k goes to group k mod G), each group adds its rows in order, and a fixed butterfly folds
//     the groups.  Every load instruction of a wave thus fetches G whole rows as contiguous 16-byte
//     pieces, and UNR loads are issued before the first add so that many rows are in flight.
//   * a block of W waves owns LB consecutive lists (W = 1 for the two lookups, 4 for the backward's
//     sums).  Lists of at most 64 ids are summed by one wave each.  A longer list is summed by the
//     whole block: its 64-id chunks go to the waves round-robin, the W wave partials are added in
//     wave order.  Which path a list takes and the order of every addition depend on the list's
//     length and content only, never on where the list sits in a batch: the deduplicated and the
//     non-deduplicated lookup (same W) agree bit for bit.
//   * blocks are dealt to lists statically (no atomics; the hardware's block dispatch balances the
//     load).  With F a multiple of 8 the mapping is XCD-aware: block b serves the features
//     f with f mod 8 = b mod 8, and since consecutive blocks go to consecutive XCDs, the hot rows of
//     a table stay in one XCD's L2.  The number of lists may live on the device only (unique
//     lists): the grid is sized from a host-side bound and every block strides until its queue is
//     exhausted, so any grid size is correct.
#include "recd_internal.h"

#include <hip/hip_fp16.h>

namespace {

constexpr int kNQ = 8;         // XCDs
constexpr int kBlock = 256;
// Threads per block of the gather-sum kernel.  The forward lookups run one wave per block: the
// waves of a block finish their lists at different times, and a block's registers are only free
// again when its last wave is done, so with lists of 1 to 256 ids a four-wave block keeps idle
// waves resident (unique lookup 0.124 ms against 0.133, KJT lookup 0.99 against 1.16).  The
// backward's sums keep four waves: their long segments and 256-entry chunks want the whole block.
template <int SITE> struct SegBlock {
    static constexpr int threads = (SITE == 0 || SITE == 1 || SITE == 4) ? 64 : 256;
};
constexpr int kMaxLB = 16;     // lists per block item (upper bound)
constexpr int kChunk = 64;     // ids per chunk: a wave loads a chunk's ids with one instruction

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

// Pooling functions (Sec. 2.2: sum, average, max).  The average is the sum scaled at the end.
// POOL_WSUM: the sum with one fp32 weight per id, acc = fma(weight, row element, acc).
enum { POOL_SUM = 0, POOL_MEAN = 1, POOL_MAX = 2, POOL_WSUM = 3 };
template <int MODE> __device__ __forceinline__ float pool2(float a, float x, float wt = 1.f)
{
    return MODE == POOL_MAX ? fmaxf(a, x) : (MODE == POOL_WSUM ? __fmaf_rn(wt, x, a) : a + x);
}
template <int MODE> __device__ __forceinline__ float pool_identity()
{
    return MODE == POOL_MAX ? -INFINITY : 0.f;
}

// fold the elements of one 16-byte vector into acc[0..per_vec); wt: the id's weight (POOL_WSUM)
template <int TT, int MODE = POOL_SUM>
__device__ __forceinline__ void accumulate(float *acc, const uint4 &v, float wt = 1.f)
{
    if constexpr (TT == RECD_F32) {
        acc[0] = pool2<MODE>(acc[0], __uint_as_float(v.x), wt);
        acc[1] = pool2<MODE>(acc[1], __uint_as_float(v.y), wt);
        acc[2] = pool2<MODE>(acc[2], __uint_as_float(v.z), wt);
        acc[3] = pool2<MODE>(acc[3], __uint_as_float(v.w), wt);
    } else if constexpr (TT == RECD_F16) {
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; i++) {
            acc[2 * i] = pool2<MODE>(acc[2 * i], __half2float(__ushort_as_half((unsigned short)(w[i] & 0xffffu))), wt);
            acc[2 * i + 1] =
                pool2<MODE>(acc[2 * i + 1], __half2float(__ushort_as_half((unsigned short)(w[i] >> 16))), wt);
        }
    } else {
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; i++) {
            acc[2 * i] = pool2<MODE>(acc[2 * i], bf16_to_f32(w[i] & 0xffffu), wt);
            acc[2 * i + 1] = pool2<MODE>(acc[2 * i + 1], bf16_to_f32(w[i] >> 16), wt);
        }
    }
}

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// store N fp32 accumulators (N = 4 or 8) as elements of type OT at dst; NT = streaming store for
// outputs that are written once and not read again by the path
template <int OT, int N, bool NT> __device__ __forceinline__ void store_row_piece(void *dst, const float *acc)
{
    if constexpr (OT == RECD_F32) {
#pragma unroll
        for (int i = 0; i < N; i += 4) {
            const u32x4 o = {__float_as_uint(acc[i]), __float_as_uint(acc[i + 1]),
                             __float_as_uint(acc[i + 2]), __float_as_uint(acc[i + 3])};
            if constexpr (NT)
                __builtin_nontemporal_store(o, reinterpret_cast<u32x4 *>(dst) + i / 4);
            else
                reinterpret_cast<u32x4 *>(dst)[i / 4] = o;
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
        const u32x4 o = {w[0], w[1], w[2], w[3]};
        if constexpr (NT)
            __builtin_nontemporal_store(o, reinterpret_cast<u32x4 *>(dst));
        else
            *reinterpret_cast<u32x4 *>(dst) = o;
    }
}

// Call sites of the gather-sum kernel.  Each gets its own instantiation (and symbol): the unique
// lookup, the KJT comparison lookup, and the backward's sums over grad_out rows / chunk partials.
// SITE_UNIQUE_EXPAND: the unique lookup whose waves also store a finished row to the output rows of
// the run of adjacent samples that starts at the list's first row (Sec. 5: lookup on the unique
// lists, then the index select back to the batch - here for the samples a session put side by side).
enum { SITE_UNIQUE = 0, SITE_KJT = 1, SITE_GRAD_LISTS = 2, SITE_GRAD_STREAM = 3, SITE_UNIQUE_EXPAND = 4 };

struct SegSumParams {
    TablePtrs tables;
    const void *values;
    const int64_t *offsets;
    const int64_t *list_off;
    int64_t lists_per_feature;
    int64_t list_base;
    void *out;
    int F;
    int D;
    int vecs_per_row;  // D / elements per 16-byte vector
    int nq;            // 8: XCD-aware queues (feature f -> queue f mod 8); 1: one flat queue
    int lb;            // lists per block item, <= kMaxLB
    // optional (flat queue only): list l ends at ends[l] instead of offsets[l+1], and the number of
    // lists is *count_dev
    const int64_t *ends;
    const int64_t *count_dev;
    // optional: list l spans offsets[l] .. offsets[l] + lens[l] (windows of a partial IKJT)
    const int64_t *lens;
    // optional (SITE_GRAD_LISTS only): the finished row of list l is divided by
    // div_off[l+1] - div_off[l] when that is positive (backward of average pooling)
    const int64_t *div_off;
    // POOL_WSUM: one fp32 weight per id, aligned with values
    const float *weights;
    // SITE_UNIQUE_EXPAND: the IKJT's run index (header, one entry per run of adjacent rows that name
    // the same unique list, closing entry), the expanded output [F*B, D], rows per feature, the
    // launch's first feature, and how the runs are dealt to the eight block queues
    const int64_t *run_index;
    void *expanded;
    int64_t B;
    int64_t run_cap;         // no run number reaches this (F*B)
    int64_t runs_per_queue;  // queue q takes the runs [q * runs_per_queue, (q+1) * runs_per_queue) first
    int all_runs;            // later runs of a list sum it again instead of waiting for a copy pass
    int feat_base;
};

// Adds the rows of NL chunks (chunk j: ns[j] <= 64 ids starting at values[starts[j]], rows of the
// table whose per-lane base pointer is bases[j]) into acc[j], all NL chunks in flight together.
// Inside a chunk, lane group g adds the ids g, g+G, g+2G, ... in that order, whatever NL and US are.
// ns[] and starts[] are wave-uniform, so every "is this load slot used" test is a scalar branch and
// unused slots cost nothing; only a chunk's last slot can hold lane groups beyond the end (they
// fetch row 0, which exists, and are masked out of the add).  Ids are used modulo 2^32.
template <int LPR, int VPL, int TT, typename IdxT, int NL, int US, int MODE = POOL_SUM, bool NTL = false>
__device__ __forceinline__ void add_chunks(float (*acc)[Elem<TT>::per_vec * VPL],
                                           const char *const *bases, const IdxT *values,
                                           const int64_t *starts, const int *ns, uint32_t row_bytes,
                                           int lane, int g, const float *weights = nullptr,
                                           const uint32_t *pre_id = nullptr)
{
    constexpr int EPV = Elem<TT>::per_vec;
    constexpr int G = 64 / LPR;
    constexpr bool WT = MODE == POOL_WSUM;
    uint32_t my_id[NL];
    float my_wt[NL];
    int nmax = 0;
#pragma unroll
    for (int j = 0; j < NL; j++) {
        // pre_id: the caller fetched this lane's id earlier (while the previous chunk's rows were in flight)
        my_id[j] = pre_id ? pre_id[j] : (lane < ns[j] ? (uint32_t)values[starts[j] + lane] : 0u);
        my_wt[j] = (WT && lane < ns[j]) ? weights[starts[j] + lane] : 0.f;
        nmax = ns[j] > nmax ? ns[j] : nmax;
    }
    for (int k0 = 0; k0 < nmax; k0 += G * US) {
        uint4 v[NL][US][VPL];
#pragma unroll
        for (int j = 0; j < NL; j++)
#pragma unroll
            for (int u = 0; u < US; u++) {
                if (k0 + u * G < ns[j]) {  // scalar test
                    const uint32_t id = __shfl(my_id[j], k0 + u * G + g);
                    const char *src = bases[j] + (uint64_t)id * row_bytes;
#pragma unroll
                    for (int w = 0; w < VPL; w++) {
                        if constexpr (NTL) {  // rows read once: streaming loads
                            const u32x4 t = __builtin_nontemporal_load(
                                reinterpret_cast<const u32x4 *>(src + w * LPR * 16));
                            v[j][u][w] = make_uint4(t.x, t.y, t.z, t.w);
                        } else {
                            v[j][u][w] = *reinterpret_cast<const uint4 *>(src + w * LPR * 16);
                        }
                    }
                }
            }
#pragma unroll
        for (int j = 0; j < NL; j++)
#pragma unroll
            for (int u = 0; u < US; u++) {
                // the weight is fetched from its lane only now: held since the loads were issued it
                // would cost a register per load slot
                const float wt = (WT && k0 + u * G < ns[j]) ? __shfl(my_wt[j], k0 + u * G + g) : 1.f;
                if (k0 + u * G + G <= ns[j]) {  // scalar test: every lane group holds a real id
#pragma unroll
                    for (int w = 0; w < VPL; w++)
                        accumulate<TT, MODE>(acc[j] + w * EPV, v[j][u][w], wt);
                } else if (k0 + u * G < ns[j]) {
                    if (k0 + u * G + g < ns[j]) {
#pragma unroll
                        for (int w = 0; w < VPL; w++)
                            accumulate<TT, MODE>(acc[j] + w * EPV, v[j][u][w], wt);
                    }
                }
            }
    }
}

// Occupancy target: 7 waves per SIMD (72 VGPRs) measured best for one-vector-per-lane fp32 rows; more
// loads in flight per wave at lower occupancy, or fewer at 8 waves, were both slower.  The
// instantiations that need more registers than that (16-bit tables decode into twice the
// accumulators, rows of at most 128 bytes put 8 rows into every load, the weighted sum carries
// the weights: 6 waves for the KJT lookup, 5 for the unique lists) get a lower target instead of
// spilling: a spilled accumulator costs more than the lost wave.
template <int LPR, int VPL, int TT, int OT, int SITE, int MODE> constexpr int segsum_waves()
{
    if (VPL > 1)
        return 1;
#ifndef RECD_BASE_WAVES
#define RECD_BASE_WAVES 7
#endif
    int w = MODE == POOL_WSUM ? (SITE == SITE_KJT ? 6 : 5) : RECD_BASE_WAVES;
    if (LPR == 8)
        w -= 2;
    else if (TT != RECD_F32 && SITE == SITE_UNIQUE_EXPAND)
        w -= 2;
    else if (TT != RECD_F32 && (MODE != POOL_SUM || OT == RECD_BF16))
        w -= 1;
    return w < 3 ? 3 : w;
}

template <int LPR, int VPL, int TT, int OT, typename IdxT, int SITE, int MODE = POOL_SUM>
__global__ __launch_bounds__(SegBlock<SITE>::threads)
__attribute__((amdgpu_waves_per_eu(segsum_waves<LPR, VPL, TT, OT, SITE, MODE>())))
void k_segsum(const SegSumParams p)
{
    constexpr int kSegBlock = SegBlock<SITE>::threads;
    constexpr int kWaves = kSegBlock / 64;
    constexpr bool NT = SITE == SITE_KJT;  // streaming output
    constexpr int EPV = Elem<TT>::per_vec;
    constexpr int NACC = EPV * VPL;
    constexpr int ROWF = LPR * NACC;                      // floats of one (padded) row
    constexpr int OB = (OT == RECD_F32) ? EPV * 4 : 16;   // bytes a lane writes per vector
    constexpr int UNR = (VPL == 1) ? 8 : (VPL == 2 ? 4 : 2);
    constexpr int LL = ROWF <= 256 ? 4 : (ROWF <= 512 ? 2 : 1);  // long lists folded per barrier pair

    __shared__ int64_t s_loff[RECD_F_PER_LAUNCH + 1];
    __shared__ int64_t s_qpref[RECD_F_PER_LAUNCH + 1];
    __shared__ int64_t s_start[kMaxLB], s_end[kMaxLB], s_list[kMaxLB];
    __shared__ int s_feat[kMaxLB];
    __shared__ float s_part[LL][kWaves][ROWF];
    constexpr bool EXPAND = SITE == SITE_UNIQUE_EXPAND;
    static_assert(!EXPAND || kWaves == 1, "a finished row is in the registers of one wave");

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform, kept in a scalar register
    const int nq = p.nq;
    const int q = nq == 1 ? 0 : (int)(blockIdx.x % kNQ);
    const int64_t item0 = nq == 1 ? blockIdx.x : blockIdx.x / kNQ;
    const int64_t item_stride = nq == 1 ? gridDim.x : gridDim.x / kNQ;
    const int nslots = (p.F - q + nq - 1) / nq;  // features in my queue: q, q+nq, ...

    if constexpr (!EXPAND) {
    for (int f = tid; f <= p.F; f += kSegBlock)
        s_loff[f] = p.list_off ? p.list_off[f] : (int64_t)f * p.lists_per_feature;
    __syncthreads();
    if (wv == 0) {
        // exclusive prefix of my queue's per-feature list counts: two slots per lane
        const int k0 = 2 * lane, k1 = 2 * lane + 1;
        const int f0 = q + k0 * nq, f1 = q + k1 * nq;
        const int64_t c0 = k0 < nslots ? s_loff[f0 + 1] - s_loff[f0] : 0;
        const int64_t c1 = k1 < nslots ? s_loff[f1 + 1] - s_loff[f1] : 0;
        int64_t inc = c0 + c1;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int64_t x = __shfl_up(inc, d);
            if (lane >= d)
                inc += x;
        }
        const int64_t ex = inc - c0 - c1;
        if (k0 < nslots)
            s_qpref[k0] = ex;
        if (k1 < nslots)
            s_qpref[k1] = ex + c0;
        const int64_t all = __shfl(inc, 63);
        if (lane == 0)
            s_qpref[nslots] = all;
    }
    __syncthreads();
    }
    const int64_t total = EXPAND ? 0 : (p.count_dev ? *p.count_dev : s_qpref[nslots]);

    const int g = lane / LPR;   // lane group = which of the G rows of a load
    const int r = lane % LPR;   // 16-byte piece of the row
    const bool piece_ok = r < p.vecs_per_row || VPL > 1;
    const IdxT *values = static_cast<const IdxT *>(p.values);
    const uint32_t row_bytes = (uint32_t)p.D * (TT == RECD_F32 ? 4 : 2);
    // lanes beyond the row's last 16-byte piece (rows shorter than LPR pieces) read piece 0; they
    // never store
    const int lane_off = piece_ok ? r * 16 : 0;
    const int64_t out_row_bytes = (int64_t)p.D * (OT == RECD_F32 ? 4 : 2);
    const int lb = p.lb;

    auto fold_groups = [&](float *acc) {
#pragma unroll
        for (int s = LPR; s < 64; s <<= 1)
#pragma unroll
            for (int i = 0; i < NACC; i++)
                acc[i] = pool2<MODE>(acc[i], __shfl_xor(acc[i], s));
    };

    // A finished row: lanes of group 0 hold its NACC-element pieces in vals.
    auto finish_row = [&](int j, float *vals) {
        if (MODE == POOL_MEAN || MODE == POOL_MAX) {
            const int64_t len = s_end[j] - s_start[j];
#pragma unroll
            for (int i = 0; i < NACC; i++)
                vals[i] = len == 0 ? 0.f : (MODE == POOL_MEAN ? vals[i] / (float)len : vals[i]);
        }
        if ((SITE == SITE_GRAD_LISTS || SITE == SITE_GRAD_STREAM) && p.div_off) {
            const int64_t n = p.div_off[s_list[j] + 1] - p.div_off[s_list[j]];
            if (n > 0) {
#pragma unroll
                for (int i = 0; i < NACC; i++)
                    vals[i] = vals[i] / (float)n;
            }
        }
        if (g == 0 && piece_ok) {
            char *dst = static_cast<char *>(p.out) + s_list[j] * out_row_bytes;
#pragma unroll
            for (int w = 0; w < VPL; w++)
                store_row_piece<OT, EPV, NT>(dst + ((int64_t)w * LPR + r) * OB, vals + w * EPV);
        }
    };

    // One wave walks a whole list of more than 64 ids: the ids of the next chunk are fetched before
    // the rows of this one, so their latency hides behind the row loads.
    auto walk_long_list = [&](float (*acc)[NACC], const char *table, int64_t start, int64_t end) {
        int64_t base = start;
        int n = (int)(end - base < kChunk ? end - base : kChunk);
        uint32_t cur = lane < n ? (uint32_t)values[base + lane] : 0u;
        for (;;) {
            const int64_t nbase = base + kChunk;
            const bool more = nbase < end;
            const int nn = more ? (int)(end - nbase < kChunk ? end - nbase : kChunk) : 0;
            const uint32_t nxt = (more && lane < nn) ? (uint32_t)values[nbase + lane] : 0u;
            add_chunks<LPR, VPL, TT, IdxT, 1, UNR, MODE, SITE == SITE_GRAD_STREAM>(acc, &table, values, &base, &n,
                                                                                   row_bytes, lane, g, p.weights, &cur);
            if (!more)
                break;
            base = nbase;
            n = nn;
            cur = nxt;
        }
    };

    if constexpr (EXPAND) {
        // Work item = a run of the batch: adjacent rows of a feature that name the same unique list
        // (the samples of a session).  The wave of a list's first run sums the list, stores the row
        // to pooled and to every output row of the run; the runs of a list that comes back later in
        // the batch are left to the copy kernel that follows.  One load round trip brings the run's
        // entry, the start of the next run and the number of runs; no other index is read.
        // Queue q = blockIdx mod 8 (one XCD) takes a contiguous stretch of the runs, which are in
        // (feature, row) order, so a table's hot rows stay in one L2.
        const int64_t *ri = p.run_index;
        const int64_t per = p.runs_per_queue;
        const int qx = (int)(blockIdx.x % kNQ);
        const int64_t stride = gridDim.x / kNQ;
        for (int64_t item = blockIdx.x / kNQ;; item += stride) {
            const int64_t rr = item < per ? (int64_t)qx * per + item : (int64_t)kNQ * per + (item - per) * kNQ + qx;
            if (rr >= p.run_cap)
                break;
            int64_t word = 0;  // lanes 0..2: the entry, lane 3: first word of the next entry, lane 4: header
            if (lane < 4)
                word = ri[3 * (1 + rr) + lane];
            else if (lane == 4)
                word = ri[0];
            const uint32_t wlo = (uint32_t)(uint64_t)word, whi = (uint32_t)((uint64_t)word >> 32);
            auto lane64 = [&](int k) {
                return (int64_t)(((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)whi, k) << 32) |
                                 (uint32_t)__builtin_amdgcn_readlane((int)wlo, k));
            };
            if (rr >= lane64(4))
                break;  // runs beyond the last: so are all later items of this block
            const int64_t w0 = lane64(0);
            const uint32_t uf = (uint32_t)((uint64_t)w0 >> 32);
            const bool first_run = (uf >> 31) != 0;
            if (!first_run && !p.all_runs)
                continue;  // not the list's first run
            const uint32_t row0 = (uint32_t)(uint64_t)w0;
            const int64_t u = uf & 0x7fffffffu;
            const int64_t start = lane64(1);
            const int64_t len_ids = lane64(2);
            const uint32_t run_rows = (uint32_t)(uint64_t)lane64(3) - row0;
            const int f = (int)(row0 / (uint32_t)p.B) - p.feat_base;
            if (f < 0 || f >= p.F)
                continue;  // a feature of another launch
            const char *table = static_cast<const char *>(p.tables.p[f]) + lane_off;
            float acc[1][NACC];
#pragma unroll
            for (int i = 0; i < NACC; i++)
                acc[0][i] = pool_identity<MODE>();
            if (len_ids > kChunk) {
                walk_long_list(acc, table, start, start + len_ids);
            } else {
                const int n = (int)len_ids;
                add_chunks<LPR, VPL, TT, IdxT, 1, UNR, MODE, false>(acc, &table, values, &start, &n, row_bytes, lane,
                                                                    g, p.weights);
            }
            fold_groups(acc[0]);  // the butterfly leaves the finished row in every lane group
            if (piece_ok) {
                if (g == 0 && first_run) {
                    char *dst = static_cast<char *>(p.out) + u * out_row_bytes;
#pragma unroll
                    for (int w = 0; w < VPL; w++)
                        store_row_piece<OT, EPV, false>(dst + ((int64_t)w * LPR + r) * OB, acc[0] + w * EPV);
                }
                char *dst = static_cast<char *>(p.expanded) + (int64_t)row0 * out_row_bytes;
                for (uint32_t k = g; p.expanded && k < run_rows; k += 64 / LPR) {
#pragma unroll
                    for (int w = 0; w < VPL; w++)
                        store_row_piece<OT, EPV, true>(dst + (int64_t)k * out_row_bytes + ((int64_t)w * LPR + r) * OB,
                                                       acc[0] + w * EPV);
                }
            }
        }
        return;
    }

    for (int64_t item = item0; item * lb < total; item += item_stride) {
        const int64_t t0 = item * lb;
        const int cnt = (int)(total - t0 < lb ? total - t0 : lb);
        __syncthreads();  // the previous item no longer reads the shared arrays
        if (tid < cnt) {
            const int64_t t = t0 + tid;
            int lo = 0, hi = nslots;  // slot with s_qpref[slot] <= t < s_qpref[slot+1]
            while (hi - lo > 1) {
                const int mid = (lo + hi) >> 1;
                if (s_qpref[mid] <= t)
                    lo = mid;
                else
                    hi = mid;
            }
            const int f = q + lo * nq;
            const int64_t l = p.count_dev ? t : p.list_base + s_loff[f] + (t - s_qpref[lo]);
            s_feat[tid] = f;
            s_list[tid] = l;
            const int64_t start = p.offsets[l];
            s_start[tid] = start;
            s_end[tid] = p.ends ? p.ends[l] : (p.lens ? start + p.lens[l] : p.offsets[l + 1]);
        }
        __syncthreads();

        // ---- long lists (> 64 ids): the whole block; the list's 64-id chunks go to the waves
        //      round-robin, the wave partials are added in wave order -----------------------------
        int batch[LL];
        int nb = 0;
        for (int j = 0; j <= cnt; j++) {
            const bool is_long = j < cnt && s_end[j] - s_start[j] > kChunk;  // block-uniform
            if (is_long) {
                const int64_t start = uniform64(s_start[j]), end = uniform64(s_end[j]);
                const char *table = static_cast<const char *>(p.tables.p[s_feat[j]]) + lane_off;
                float acc[1][NACC];
#pragma unroll
                for (int i = 0; i < NACC; i++)
                    acc[0][i] = pool_identity<MODE>();
                if constexpr (kWaves == 1) {
                    walk_long_list(acc, table, start, end);
                } else {
                    for (int64_t base = start + (int64_t)wv * kChunk; base < end; base += kWaves * kChunk) {
                        const int n = (int)(end - base < kChunk ? end - base : kChunk);
                        add_chunks<LPR, VPL, TT, IdxT, 1, UNR, MODE, SITE == SITE_GRAD_STREAM>(
                            acc, &table, values, &base, &n, row_bytes, lane, g, p.weights);
                    }
                }
                fold_groups(acc[0]);
                if constexpr (kWaves == 1) {
                    finish_row(j, acc[0]);  // no other wave's partial to add
                } else {
                    if (g == 0) {
#pragma unroll
                        for (int w = 0; w < VPL; w++)
#pragma unroll
                            for (int i = 0; i < EPV; i++)
                                s_part[nb][wv][(w * LPR + r) * EPV + i] = acc[0][w * EPV + i];
                    }
                    batch[nb++] = j;
                }
            }
            if (nb == LL || (j == cnt && nb > 0)) {
                __syncthreads();
                for (int e = wv; e < nb; e += kWaves) {
                    float tot[NACC];
#pragma unroll
                    for (int w = 0; w < VPL; w++)
#pragma unroll
                        for (int i = 0; i < EPV; i++) {
                            const int x = (w * LPR + r) * EPV + i;
                            float t_ = s_part[e][0][x];
#pragma unroll
                            for (int w2 = 1; w2 < kWaves; w2++)
                                t_ = pool2<MODE>(t_, s_part[e][w2][x]);  // wave order
                            tot[w * EPV + i] = t_;
                        }
                    finish_row(batch[e], tot);
                }
                __syncthreads();
                nb = 0;
            }
        }

        // ---- short lists (one chunk at most): wave w takes lists w, w+4, ... of the item ----------
        for (int j = wv; j < cnt; j += kWaves) {
            const int64_t start = uniform64(s_start[j]);
            const int64_t len = uniform64(s_end[j]) - start;
            if (len > kChunk)
                continue;
            const char *table = static_cast<const char *>(p.tables.p[s_feat[j]]) + lane_off;
            const int n = (int)len;
            float acc[1][NACC];
#pragma unroll
            for (int i = 0; i < NACC; i++)
                acc[0][i] = pool_identity<MODE>();
            add_chunks<LPR, VPL, TT, IdxT, 1, UNR, MODE, SITE == SITE_GRAD_STREAM>(acc, &table, values, &start, &n,
                                                                                   row_bytes, lane, g, p.weights);
            fold_groups(acc[0]);
            finish_row(j, acc[0]);
        }
    }
}

template <int TT, int OT, typename IdxT, int SITE, int MODE = POOL_SUM>
bool launch_shape(hipStream_t st, int blocks, int vecs, const SegSumParams &p)
{
    const dim3 grid(blocks), block(SegBlock<SITE>::threads);
    if (vecs <= 8) hipLaunchKernelGGL((k_segsum<8, 1, TT, OT, IdxT, SITE, MODE>), grid, block, 0, st, p);
    else if (vecs <= 16) hipLaunchKernelGGL((k_segsum<16, 1, TT, OT, IdxT, SITE, MODE>), grid, block, 0, st, p);
    else if (vecs <= 32) hipLaunchKernelGGL((k_segsum<32, 1, TT, OT, IdxT, SITE, MODE>), grid, block, 0, st, p);
    else if (vecs <= 64) hipLaunchKernelGGL((k_segsum<64, 1, TT, OT, IdxT, SITE, MODE>), grid, block, 0, st, p);
    else if (vecs == 128) hipLaunchKernelGGL((k_segsum<64, 2, TT, OT, IdxT, SITE, MODE>), grid, block, 0, st, p);
    else if (vecs == 256) hipLaunchKernelGGL((k_segsum<64, 4, TT, OT, IdxT, SITE, MODE>), grid, block, 0, st, p);
    else return false;
    return true;
}

template <int SITE, int MODE = POOL_SUM>
bool launch_forward(hipStream_t st, int blocks, int v, const SegSumArgs &a, const SegSumParams &p)
{
    if (a.table_dt == RECD_F32 && a.out_dt == RECD_F32)
        return launch_shape<RECD_F32, RECD_F32, int64_t, SITE, MODE>(st, blocks, v, p);
    if (a.table_dt == RECD_F16 && a.out_dt == RECD_F16)
        return launch_shape<RECD_F16, RECD_F16, int64_t, SITE, MODE>(st, blocks, v, p);
    if (a.table_dt == RECD_F16 && a.out_dt == RECD_F32)
        return launch_shape<RECD_F16, RECD_F32, int64_t, SITE, MODE>(st, blocks, v, p);
    if (a.table_dt == RECD_BF16 && a.out_dt == RECD_BF16)
        return launch_shape<RECD_BF16, RECD_BF16, int64_t, SITE, MODE>(st, blocks, v, p);
    if (a.table_dt == RECD_BF16 && a.out_dt == RECD_F32)
        return launch_shape<RECD_BF16, RECD_F32, int64_t, SITE, MODE>(st, blocks, v, p);
    return false;
}

// ---- expand: out[f,b,:] = pooled[feat_uoff[f] + inverse[f,b], :]  (16-byte pieces) ------------
// A block copies kExpandRPT sweeps of (256 / vecs_per_row) consecutive output rows.  Every thread
// first loads the inverse entries of all its rows, then all its pooled pieces, then stores them
// with streaming (non-temporal) stores: the output is written once and never re-read here, while
// the pooled rows, shared by the consecutive samples of a session, should stay in L2.
// Rows per thread, measured at 1.05 M rows of 512 bytes (same buffers, back to back): 3: 106 us, 4: 94,
// 5: 92.5, 6: 90.5, 7: 93.5, 8: 98-100, 10: 100, 12: 103; blocks of 64, 128, 512 or 1024 threads
// instead of 256 are no faster at their best row counts (90.8-92 us), and occupancy limits do not
// help.  Fewer stores per wave reach memory in a more sequential order (a store-only kernel of this
// shape runs at 5.5 TB/s with 8 stores per thread and at 6.9 with one), more rows per thread hide
// the two dependent loads: six is where the two meet.
constexpr int kExpandRPT = 6;

template <bool TWO_FEATURES>
__global__ __launch_bounds__(kBlock) void k_expand(const u32x4 *__restrict__ pooled,
                                                   const int64_t *__restrict__ feat_uoff,
                                                   const int32_t *__restrict__ inverse,
                                                   u32x4 *__restrict__ out, uint32_t B,
                                                   uint32_t n_rows, int vecs_per_row)
{
    const uint32_t rows_per_sweep = kBlock / vecs_per_row;  // vecs_per_row <= 256
    const uint32_t piece = threadIdx.x % vecs_per_row;
    const uint32_t sub = threadIdx.x / vecs_per_row;
    if (sub >= rows_per_sweep)
        return;
    const uint32_t row0 = blockIdx.x * rows_per_sweep * kExpandRPT;
    // TWO_FEATURES: B >= rows per block, so the block's rows lie in features f0 and f0 + 1 only
    const uint32_t f0 = row0 / B;
    const uint32_t next_start = (f0 + 1) * B;
    const int64_t base0 = feat_uoff[f0];
    const int64_t base1 = TWO_FEATURES ? feat_uoff[f0 + (next_start < n_rows ? 1 : 0)] : 0;
    // loads use a clamped row so that none of them is conditional; only the store is predicated
    int32_t inv[kExpandRPT];
    uint32_t rows[kExpandRPT];
#pragma unroll
    for (int k = 0; k < kExpandRPT; k++) {
        const uint32_t row = row0 + k * rows_per_sweep + sub;
        rows[k] = row < n_rows ? row : n_rows - 1;
        inv[k] = inverse[rows[k]];
    }
    u32x4 v[kExpandRPT];
#pragma unroll
    for (int k = 0; k < kExpandRPT; k++) {
        int64_t base;
        if (TWO_FEATURES)
            base = rows[k] >= next_start ? base1 : base0;
        else
            base = feat_uoff[rows[k] / B];
        v[k] = pooled[(base + inv[k]) * vecs_per_row + piece];
    }
#pragma unroll
    for (int k = 0; k < kExpandRPT; k++) {
        const uint32_t row = row0 + k * rows_per_sweep + sub;
        if (row < n_rows)
            __builtin_nontemporal_store(v[k], &out[(int64_t)row * vecs_per_row + piece]);
    }
}

// ---- the rest of the expand after the fused lookup ---------------------------------------------
// Runs whose list was first seen earlier in the batch (the list came back after other rows): their
// output rows are copies of pooled[u].  A block takes 64 runs: its first wave lists the runs that
// are not first runs and numbers their rows, then the whole block copies them, a 16-byte piece per
// thread and step.  With session-clustered batches these are a few percent of the rows.
__global__ __launch_bounds__(kBlock) void k_expand_runs(const u32x4 *__restrict__ pooled,
                                                        const int64_t *__restrict__ run_index,
                                                        u32x4 *__restrict__ out, int vecs_per_row)
{
    __shared__ uint32_t s_row[64], s_src[64], s_off[65];
    __shared__ uint32_t s_cnt;
    const int tid = threadIdx.x, lane = tid & 63;
    const int64_t n_runs = run_index[0];
    const uint32_t vecs = (uint32_t)vecs_per_row;
    for (int64_t r0 = (int64_t)blockIdx.x * 64; r0 < n_runs; r0 += (int64_t)gridDim.x * 64) {
        __syncthreads();  // the previous round is done with the shared arrays
        if (tid < 64) {
            const int64_t rr = r0 + lane;
            uint32_t rows = 0, row = 0, u = 0;
            if (rr < n_runs) {
                const uint64_t w0 = (uint64_t)run_index[3 * (1 + rr)];
                const uint64_t w3 = (uint64_t)run_index[3 * (2 + rr)];
                row = (uint32_t)w0;
                u = (uint32_t)(w0 >> 32);
                rows = (u >> 31) ? 0u : (uint32_t)w3 - row;  // first runs were written by the lookup
                u &= 0x7fffffffu;
            }
            const uint64_t m = __ballot(rows != 0);
            uint32_t inc = rows;  // inclusive prefix of the rows to copy
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                const uint32_t x = __shfl_up(inc, d);
                if (lane >= d)
                    inc += x;
            }
            if (rows != 0) {
                const uint32_t k = (uint32_t)__popcll(m & ((1ull << lane) - 1));
                s_row[k] = row;
                s_src[k] = u;
                s_off[k] = inc - rows;
            }
            if (lane == 63) {
                s_cnt = (uint32_t)__popcll(m);
                s_off[__popcll(m)] = inc;
            }
        }
        __syncthreads();
        const uint32_t cnt = s_cnt;
        if (cnt == 0)
            continue;
        const uint32_t total = s_off[cnt] * vecs;
        for (uint32_t idx = tid; idx < total; idx += kBlock) {
            const uint32_t k = idx / vecs, piece = idx - k * vecs;
            uint32_t j = 0;  // the last listed run with s_off[j] <= k
#pragma unroll
            for (uint32_t st = 32; st >= 1; st >>= 1)
                if (j + st < cnt && s_off[j + st] <= k)
                    j += st;
            __builtin_nontemporal_store(pooled[(int64_t)s_src[j] * vecs + piece],
                                        &out[(int64_t)(s_row[j] + (k - s_off[j])) * vecs + piece]);
        }
    }
}

// err[0] |= 64: the run index is malformed (run count, row order, list positions)
__global__ void k_validate_runs(const int64_t *run_index, int64_t n_rows, int64_t B, int *err)
{
    const int64_t n_runs = run_index[0], U = run_index[1], M = run_index[2];
    if (n_runs < 0 || n_runs > n_rows || U < 0 || U > n_rows || M < 0) {
        if (blockIdx.x == 0 && threadIdx.x == 0)
            atomicOr(err, 64);
        return;
    }
    for (int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; r <= n_runs; r += (int64_t)gridDim.x * blockDim.x) {
        const uint64_t w0 = (uint64_t)run_index[3 * (1 + r)];
        const int64_t row = (uint32_t)w0, u = (uint32_t)(w0 >> 32) & 0x7fffffffu;
        const int64_t start = run_index[3 * (1 + r) + 1], n = run_index[3 * (1 + r) + 2];
        bool bad = false;
        if (r == n_runs) {
            bad = row != n_rows;
        } else {
            const int64_t next = (uint32_t)(uint64_t)run_index[3 * (2 + r)];
            // a run lies in one feature, the first run starts at row 0
            bad = row >= n_rows || next <= row || next > n_rows || (r == 0 && row != 0) ||
                  (next - 1) / B != row / B || u >= U || start < 0 || n < 0 || start > M || n > M - start;
        }
        if (bad)
            atomicOr(err, 64);
    }
}

// err[0] |= 2: an id of a first run lies outside its table (rows_f of the feature of launch f0 + f)
__global__ void k_validate_run_ids(const int64_t *run_index, const int64_t *values, int64_t B, int f,
                                   int64_t rows_f, int *err)
{
    const int64_t n_runs = run_index[0];
    for (int64_t r = blockIdx.x; r < n_runs; r += gridDim.x) {
        const uint64_t w0 = (uint64_t)run_index[3 * (1 + r)];
        if ((int64_t)((uint32_t)w0 / B) != f || !((w0 >> 63) & 1))
            continue;
        const int64_t start = run_index[3 * (1 + r) + 1], n = run_index[3 * (1 + r) + 2];
        for (int64_t t = threadIdx.x; t < n; t += blockDim.x)
            if (values[start + t] < 0 || values[start + t] >= rows_f)
                atomicOr(err, 2);
    }
}

// ---- a compute module on a grouped IKJT: element-wise sum over the features of a group ----------
// combined[group_uoff[g] + k, :] = sum over f in group g, feature order, of pooled[feat_uoff[f] + k, :]
// (fp32 accumulation, rounded once).  Thread = one 16-byte piece of one unique row of a group.
template <int TT>
__global__ __launch_bounds__(kBlock) void k_group_sum(const uint4 *__restrict__ pooled,
                                                      const int64_t *__restrict__ feat_uoff,
                                                      const int64_t *__restrict__ group_uoff,
                                                      const int32_t *__restrict__ group_off, int G,
                                                      int vecs, int64_t max_rows, void *__restrict__ out)
{
    __shared__ int64_t gu_s[RECD_MAX_FEATURES + 1];
    __shared__ int32_t go_s[RECD_MAX_FEATURES + 1];
    for (int i = threadIdx.x; i <= G; i += kBlock) {
        gu_s[i] = group_uoff[i];
        go_s[i] = group_off[i];
    }
    __syncthreads();
    const int rows_per_block = kBlock / vecs;
    const int piece = threadIdx.x % vecs, sub = threadIdx.x / vecs;
    if (sub >= rows_per_block)
        return;
    int64_t total = gu_s[G];
    if (total > max_rows)
        total = max_rows;
    constexpr int EPV = Elem<TT>::per_vec;
    for (int64_t r = (int64_t)blockIdx.x * rows_per_block + sub; r < total;
         r += (int64_t)gridDim.x * rows_per_block) {
        int g = 0;  // the last group with gu_s[g] <= r; r < gu_s[G], so it is not empty
#pragma unroll
        for (int s = RECD_MAX_FEATURES / 2; s >= 1; s >>= 1)
            if (g + s < G && gu_s[g + s] <= r)
                g += s;
        const int64_t k = r - gu_s[g];
        float acc[EPV] = {};
        for (int f = go_s[g]; f < go_s[g + 1]; f++)
            accumulate<TT>(acc, pooled[(feat_uoff[f] + k) * vecs + piece]);
        store_row_piece<TT, EPV, false>(static_cast<char *>(out) + (r * vecs + piece) * 16, acc);
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

// err[0] |= 16: a window of a partial IKJT leaves the stored values; |= 2: id outside its table
__global__ void k_validate_windows(const int64_t *p_values, int64_t P_cap, const int64_t *win_start,
                                   const int64_t *win_len, const int64_t *feat_uoff, int f,
                                   int64_t rows_f, int *err)
{
    const int64_t u0 = feat_uoff[f], u1 = feat_uoff[f + 1];
    for (int64_t u = u0 + blockIdx.x; u < u1; u += gridDim.x) {
        const int64_t s = win_start[u], n = win_len[u];
        if (s < 0 || n < 0 || s > P_cap || n > P_cap - s) {
            if (threadIdx.x == 0)
                atomicOr(err, 16);
            continue;
        }
        for (int64_t t = threadIdx.x; t < n; t += blockDim.x)
            if (p_values[s + t] < 0 || p_values[s + t] >= rows_f)
                atomicOr(err, 2);
    }
}

// err[0] |= 4: feat_uoff is not a prefix sum starting at 0, or an inverse entry is outside its
// feature's [0, U_f)
__global__ void k_validate_inverse(const int32_t *inverse, const int64_t *feat_uoff, int F, int64_t B,
                                   int *err)
{
    const int64_t n = (int64_t)F * B;
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i <= F && ((i == 0 && feat_uoff[0] != 0) || (i > 0 && feat_uoff[i] < feat_uoff[i - 1])))
        atomicOr(err, 4);
    if (i < n) {
        const int64_t f = i / B;
        const int64_t inv = inverse[i];
        if (inv < 0 || inv >= feat_uoff[f + 1] - feat_uoff[f])
            atomicOr(err, 4);
    }
}

} // namespace

// Checks a run index before the fused lookup reads through it.  Synchronises.
static recd_status validate_run_index(recd_ctx *ctx, int F, int64_t B, const int64_t *rows,
                                      const int64_t *u_values, const int64_t *run_index)
{
    RECD_TRY(recd_reserve(ctx, 512));
    int *err = reinterpret_cast<int *>(ctx->ws);
    RECD_HIP(ctx, hipMemsetAsync(err, 0, sizeof(int), ctx->stream));
    hipLaunchKernelGGL(k_validate_runs, dim3(256), dim3(256), 0, ctx->stream, run_index, (int64_t)F * B, B, err);
    ctx->host_pinned[0] = 0;
    RECD_HIP(ctx, hipMemcpyAsync(ctx->host_pinned, err, sizeof(int), hipMemcpyDeviceToHost, ctx->stream));
    RECD_HIP(ctx, hipStreamSynchronize(ctx->stream));
    if ((int)ctx->host_pinned[0] & 64)
        return recd_fail(ctx, RECD_EBOUNDS, "the run index is malformed");
    if (rows && u_values) {
        for (int f = 0; f < F; f++)
            hipLaunchKernelGGL(k_validate_run_ids, dim3(64), dim3(256), 0, ctx->stream, run_index, u_values, B, f,
                               rows[f], err);
        RECD_HIP(ctx, hipMemcpyAsync(ctx->host_pinned, err, sizeof(int), hipMemcpyDeviceToHost, ctx->stream));
        RECD_HIP(ctx, hipStreamSynchronize(ctx->stream));
        if ((int)ctx->host_pinned[0] & 2)
            return recd_fail(ctx, RECD_EBOUNDS, "an id lies outside its embedding table");
    }
    return RECD_OK;
}

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
    p.ends = a.ends;
    p.count_dev = a.count_dev;
    p.lens = a.lens;
    p.div_off = a.div_off;
    p.weights = a.weights;
    p.run_index = a.run_index;
    p.expanded = a.expanded;
    p.B = a.B;
    p.run_cap = (int64_t)a.F_all * a.B;
    p.feat_base = a.feat_base;
    p.runs_per_queue = 0;
    p.all_runs = a.all_runs;
    p.F = a.F;
    p.D = a.D;
    const int epv = a.table_dt == RECD_F32 ? 4 : 8;
    p.vecs_per_row = a.D / epv;
    // Launch shape.  Any grid is correct (blocks stride over their queue); these choices only
    // decide how well the chip is filled.
    const int64_t n = a.lists_bound > 0 ? a.lists_bound : 1;
    p.nq = (a.F >= kNQ && a.F % kNQ == 0 && !a.flat && !ctx->tune_flat && !a.count_dev) ? kNQ : 1;
    // lists per block: four-wave blocks (backward) take 4 to 16, single-wave blocks (forward) 1 to 4
    // (measured at 61 K unique lists and at 1.05 M KJT lists: 1 and 4)
    if (a.site == RECD_SITE_UNIQUE || a.site == RECD_SITE_KJT || a.site == RECD_SITE_UNIQUE_EXPAND)
        p.lb = n >= (512 << 10) ? 4 : (n >= (128 << 10) ? 2 : 1);
    else
        p.lb = n >= (512 << 10) ? 16 : (n >= (128 << 10) ? 8 : 4);
    if (ctx->tune_lb > 0)
        p.lb = ctx->tune_lb;
    if (a.count_dev)
        p.lb = 1;  // chunks of long segments: every list is long, one block per list
    const int64_t items = (n + p.lb - 1) / p.lb;
    int64_t nblk = p.nq == 1 ? items : kNQ * ((items + kNQ - 1) / kNQ + (items / kNQ) / 8 + 1);
    const int64_t cap = (int64_t)ctx->num_cu * 8 * (ctx->tune_gens > 0 ? ctx->tune_gens : 64);
    if (nblk > cap)
        nblk = cap / kNQ * kNQ;
    // a pass whose true list count lives on the device is usually far below the host bound: a
    // resident-sized grid that strides wastes no blocks
    if (a.count_dev && nblk > (int64_t)ctx->num_cu * 8)
        nblk = (int64_t)ctx->num_cu * 8;
    if (a.site == RECD_SITE_UNIQUE_EXPAND) {
        // one run per block; queue q of eight takes the runs [q * per, (q + 1) * per) of the host's
        // estimate first and shares whatever lies beyond it with the other queues
        p.lb = 1;
        p.nq = kNQ;
        p.runs_per_queue = (n + kNQ - 1) / kNQ;
        nblk = kNQ * (p.runs_per_queue + p.runs_per_queue / 16 + 1);
        if (nblk > cap)
            nblk = cap / kNQ * kNQ;
    }
    const int blocks = (int)nblk;
    bool ok = false;
    hipStream_t st = a.stream ? a.stream : ctx->stream;
    const int v = p.vecs_per_row;
    const bool fwd = !a.values_are_i32;
    const int slot = a.site == RECD_SITE_UNIQUE_EXPAND ? RECD_T_LOOKUP_EXPAND
                     : a.site == RECD_SITE_UNIQUE      ? RECD_T_LOOKUP
                     : a.site == RECD_SITE_KJT         ? RECD_T_KJT
                     : a.site == RECD_SITE_GRAD_STREAM ? RECD_T_GRAD_LISTS
                                                       : -1;
    if (slot >= 0)
        recd_time_begin(ctx, slot, st);
    if (a.site == RECD_SITE_UNIQUE && fwd && a.mode == POOL_SUM)
        ok = launch_forward<SITE_UNIQUE>(st, blocks, v, a, p);
    else if (a.site == RECD_SITE_KJT && fwd && a.mode == POOL_SUM)
        ok = launch_forward<SITE_KJT>(st, blocks, v, a, p);
    else if (a.site == RECD_SITE_UNIQUE_EXPAND && fwd && a.mode == POOL_SUM && a.run_index)
        ok = launch_forward<SITE_UNIQUE_EXPAND>(st, blocks, v, a, p);
    else if (a.site == RECD_SITE_UNIQUE && fwd && a.mode == POOL_MEAN)
        ok = launch_forward<SITE_UNIQUE, POOL_MEAN>(st, blocks, v, a, p);
    else if (a.site == RECD_SITE_KJT && fwd && a.mode == POOL_MEAN)
        ok = launch_forward<SITE_KJT, POOL_MEAN>(st, blocks, v, a, p);
    else if (a.site == RECD_SITE_UNIQUE && fwd && a.mode == POOL_MAX)
        ok = launch_forward<SITE_UNIQUE, POOL_MAX>(st, blocks, v, a, p);
    else if (a.site == RECD_SITE_KJT && fwd && a.mode == POOL_MAX)
        ok = launch_forward<SITE_KJT, POOL_MAX>(st, blocks, v, a, p);
    else if (a.site == RECD_SITE_UNIQUE && fwd && a.mode == POOL_WSUM && a.weights)
        ok = launch_forward<SITE_UNIQUE, POOL_WSUM>(st, blocks, v, a, p);
    else if (a.site == RECD_SITE_KJT && fwd && a.mode == POOL_WSUM && a.weights)
        ok = launch_forward<SITE_KJT, POOL_WSUM>(st, blocks, v, a, p);
    else if (a.site == RECD_SITE_GRAD_LISTS && a.values_are_i32 && a.table_dt == RECD_F32 &&
             a.out_dt == RECD_F32 && a.mode == POOL_SUM)
        ok = launch_shape<RECD_F32, RECD_F32, int32_t, SITE_GRAD_LISTS>(st, blocks, v, p);
    else if (a.site == RECD_SITE_GRAD_STREAM && a.values_are_i32 && a.table_dt == RECD_F32 &&
             a.out_dt == RECD_F32 && a.mode == POOL_SUM)
        ok = launch_shape<RECD_F32, RECD_F32, int32_t, SITE_GRAD_STREAM>(st, blocks, v, p);
    else if (a.site == RECD_SITE_GRAD_LISTS && a.values_are_i32 && a.table_dt == RECD_F32 &&
             a.out_dt == RECD_F32 && a.mode == POOL_WSUM && a.weights)
        ok = launch_shape<RECD_F32, RECD_F32, int32_t, SITE_GRAD_LISTS, POOL_WSUM>(st, blocks, v, p);
    if (slot >= 0)
        recd_time_end(ctx, slot, st);
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

// Checks an inverse index against feat_uoff (used by the expand and the backward).  Synchronises.
recd_status recd_validate_inverse(recd_ctx *ctx, int F, int64_t B, const int64_t *feat_uoff,
                                  const int32_t *inverse)
{
    RECD_TRY(recd_reserve(ctx, 512));
    int *err = reinterpret_cast<int *>(ctx->ws);
    RECD_HIP(ctx, hipMemsetAsync(err, 0, sizeof(int), ctx->stream));
    const int64_t n = (int64_t)F * B > F + 1 ? (int64_t)F * B : F + 1;
    hipLaunchKernelGGL(k_validate_inverse, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, ctx->stream,
                       inverse, feat_uoff, F, B, err);
    ctx->host_pinned[0] = 0;
    RECD_HIP(ctx, hipMemcpyAsync(ctx->host_pinned, err, sizeof(int), hipMemcpyDeviceToHost, ctx->stream));
    RECD_HIP(ctx, hipStreamSynchronize(ctx->stream));
    if ((int)ctx->host_pinned[0] & 4)
        return recd_fail(ctx, RECD_EBOUNDS, "inverse index or feat_uoff is malformed");
    return RECD_OK;
}

recd_status recd_validate_kjt_offsets(recd_ctx *ctx, int F, int64_t B, int64_t N, const int64_t *offsets)
{
    return validate_lists(ctx, F, nullptr, nullptr, offsets, nullptr, B, (int64_t)F * B, N);
}

recd_status recd_validate_kjt_lists(recd_ctx *ctx, int F, int64_t B, int64_t N, const int64_t *rows,
                                    const int64_t *values, const int64_t *offsets)
{
    if (!rows)
        return recd_fail(ctx, RECD_EINVAL, "validation needs rows[]");
    return validate_lists(ctx, F, rows, values, offsets, nullptr, B, (int64_t)F * B, N);
}

// Unique lists of an IKJT: feat_uoff[F] = U lives on the device and is fetched to size the offsets
// check; U must not exceed max_lists and, when M_cap >= 0, the ids must number at most M_cap.
recd_status recd_validate_unique_lists(recd_ctx *ctx, int F, const int64_t *rows,
                                       const int64_t *u_values, const int64_t *u_offsets,
                                       const int64_t *feat_uoff, int64_t max_lists, int64_t M_cap)
{
    if (!rows)
        return recd_fail(ctx, RECD_EINVAL, "validation needs rows[]");
    RECD_TRY(recd_reserve(ctx, 1024));
    int64_t *tmp = reinterpret_cast<int64_t *>(ctx->ws + 256);
    hipLaunchKernelGGL(k_read_i64, dim3(1), dim3(1), 0, ctx->stream, feat_uoff + F, tmp);
    RECD_HIP(ctx, hipMemcpyAsync(ctx->host_pinned + 1, tmp, 8, hipMemcpyDeviceToHost, ctx->stream));
    RECD_HIP(ctx, hipStreamSynchronize(ctx->stream));
    const int64_t U = ctx->host_pinned[1];
    if (U < 0 || U > max_lists)
        return recd_fail(ctx, RECD_ECAPACITY, "U=%lld exceeds max_lists=%lld", (long long)U,
                         (long long)max_lists);
    if (M_cap >= 0) {
        hipLaunchKernelGGL(k_read_i64, dim3(1), dim3(1), 0, ctx->stream, u_offsets + U, tmp);
        RECD_HIP(ctx, hipMemcpyAsync(ctx->host_pinned + 1, tmp, 8, hipMemcpyDeviceToHost, ctx->stream));
        RECD_HIP(ctx, hipStreamSynchronize(ctx->stream));
        const int64_t M = ctx->host_pinned[1];
        if (M < 0 || M > M_cap)
            return recd_fail(ctx, RECD_ECAPACITY, "M=%lld exceeds M_cap=%lld", (long long)M,
                             (long long)M_cap);
    }
    return validate_lists(ctx, F, rows, u_values, u_offsets, feat_uoff, 0, U, -1);
}

// weights: null, or one fp32 weight per id (then the pooling is the weighted sum, mode ignored)
static recd_status lookup_unique(recd_ctx *ctx, int mode, int F, int D, recd_dtype table_dt,
                                 recd_dtype out_dt, const void *const *tables, const int64_t *rows,
                                 const int64_t *u_values, const int64_t *u_offsets,
                                 const int64_t *feat_uoff, int64_t max_lists, void *pooled,
                                 const float *weights = nullptr)
{
    RECD_TRY(check_lookup_shape(ctx, F, D, table_dt, out_dt));
    RECD_TRY(recd_check_rows(ctx, F, rows));
    if (mode < 0 || mode > 2)
        return recd_fail(ctx, RECD_EINVAL, "unknown pooling mode %d", mode);
    if (weights)
        mode = POOL_WSUM;
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
    if (ctx->validate)
        RECD_TRY(recd_validate_unique_lists(ctx, F, rows, u_values, u_offsets, feat_uoff, max_lists, -1));
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
        a.lists_bound = max_lists;
        a.site = RECD_SITE_UNIQUE;
        a.mode = mode;
        a.weights = weights;
        a.out = pooled;
        RECD_TRY(recd_launch_segsum(ctx, a));
    }
    return RECD_OK;
}

static recd_status lookup_kjt(recd_ctx *ctx, int mode, int F, int64_t B, int D, recd_dtype table_dt,
                              recd_dtype out_dt, const void *const *tables, const int64_t *rows,
                              const int64_t *values, const int64_t *offsets, void *out,
                              const float *weights = nullptr)
{
    RECD_TRY(check_lookup_shape(ctx, F, D, table_dt, out_dt));
    RECD_TRY(recd_check_rows(ctx, F, rows));
    if (mode < 0 || mode > 2)
        return recd_fail(ctx, RECD_EINVAL, "unknown pooling mode %d", mode);
    if (weights)
        mode = POOL_WSUM;
    if (B < 0)
        return recd_fail(ctx, RECD_EINVAL, "B < 0");
    if (F == 0 || B == 0)
        return RECD_OK;
    if (!tables || !offsets || !out)  // values may be null when every list is empty (N = 0)
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
        a.lists_bound = (int64_t)a.F * B;
        a.site = RECD_SITE_KJT;
        a.mode = mode;
        a.weights = weights;
        a.out = out;
        RECD_TRY(recd_launch_segsum(ctx, a));
    }
    return RECD_OK;
}

extern "C" {

recd_status recd_pooled_lookup_unique(recd_ctx *ctx, int F, int D, recd_dtype table_dt,
                                      recd_dtype out_dt, const void *const *tables,
                                      const int64_t *rows, const int64_t *u_values,
                                      const int64_t *u_offsets, const int64_t *feat_uoff,
                                      int64_t max_lists, void *pooled)
{
    return lookup_unique(ctx, RECD_POOL_SUM, F, D, table_dt, out_dt, tables, rows, u_values, u_offsets,
                         feat_uoff, max_lists, pooled);
}

recd_status recd_kjt_pooled_lookup(recd_ctx *ctx, int F, int64_t B, int D, recd_dtype table_dt,
                                   recd_dtype out_dt, const void *const *tables,
                                   const int64_t *rows, const int64_t *values,
                                   const int64_t *offsets, void *out)
{
    return lookup_kjt(ctx, RECD_POOL_SUM, F, B, D, table_dt, out_dt, tables, rows, values, offsets, out);
}

// With no id there is no weight to read: a null weights pointer then selects the plain sum, which
// stores the same zeros.
recd_status recd_pooled_lookup_unique_weighted(recd_ctx *ctx, int F, int D, recd_dtype table_dt,
                                               recd_dtype out_dt, const void *const *tables,
                                               const int64_t *rows, const int64_t *u_values,
                                               const float *u_weights, const int64_t *u_offsets,
                                               const int64_t *feat_uoff, int64_t max_lists, void *pooled)
{
    if (ctx && u_values && !u_weights)
        return recd_fail(ctx, RECD_EINVAL, "null u_weights");
    return lookup_unique(ctx, RECD_POOL_SUM, F, D, table_dt, out_dt, tables, rows, u_values, u_offsets,
                         feat_uoff, max_lists, pooled, u_weights);
}

recd_status recd_kjt_pooled_lookup_weighted(recd_ctx *ctx, int F, int64_t B, int D, recd_dtype table_dt,
                                            recd_dtype out_dt, const void *const *tables,
                                            const int64_t *rows, const int64_t *values,
                                            const float *weights, const int64_t *offsets, void *out)
{
    if (ctx && values && !weights)
        return recd_fail(ctx, RECD_EINVAL, "null weights");
    return lookup_kjt(ctx, RECD_POOL_SUM, F, B, D, table_dt, out_dt, tables, rows, values, offsets, out,
                      weights);
}

recd_status recd_pooled_lookup_unique_mode(recd_ctx *ctx, recd_pooling mode, int F, int D,
                                           recd_dtype table_dt, recd_dtype out_dt,
                                           const void *const *tables, const int64_t *rows,
                                           const int64_t *u_values, const int64_t *u_offsets,
                                           const int64_t *feat_uoff, int64_t max_lists, void *pooled)
{
    return lookup_unique(ctx, (int)mode, F, D, table_dt, out_dt, tables, rows, u_values, u_offsets,
                         feat_uoff, max_lists, pooled);
}

recd_status recd_kjt_pooled_lookup_mode(recd_ctx *ctx, recd_pooling mode, int F, int64_t B, int D,
                                        recd_dtype table_dt, recd_dtype out_dt,
                                        const void *const *tables, const int64_t *rows,
                                        const int64_t *values, const int64_t *offsets, void *out)
{
    return lookup_kjt(ctx, (int)mode, F, B, D, table_dt, out_dt, tables, rows, values, offsets, out);
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
    if (ctx->validate)
        RECD_TRY(recd_validate_inverse(ctx, F, B, feat_uoff, inverse));
    const int vecs = (int)((size_t)D * elem_size(dt) / 16);
    const int64_t n_rows = (int64_t)F * B;
    const int64_t rows_per_block = (int64_t)(kBlock / vecs) * kExpandRPT;
    const int64_t blocks = (n_rows + rows_per_block - 1) / rows_per_block;
    if (blocks > 0x7fffffff)
        return recd_fail(ctx, RECD_EINVAL, "F*B too large");
    if (n_rows >= (int64_t)1 << 31)
        return recd_fail(ctx, RECD_EINVAL, "F*B must stay below 2^31");
    recd_time_begin(ctx, RECD_T_EXPAND, ctx->stream);
    if (B >= rows_per_block)
        hipLaunchKernelGGL(k_expand<true>, dim3((unsigned)blocks), dim3(kBlock), 0, ctx->stream,
                           static_cast<const u32x4 *>(pooled), feat_uoff, inverse,
                           static_cast<u32x4 *>(out), (uint32_t)B, (uint32_t)n_rows, vecs);
    else
        hipLaunchKernelGGL(k_expand<false>, dim3((unsigned)blocks), dim3(kBlock), 0, ctx->stream,
                           static_cast<const u32x4 *>(pooled), feat_uoff, inverse,
                           static_cast<u32x4 *>(out), (uint32_t)B, (uint32_t)n_rows, vecs);
    recd_time_end(ctx, RECD_T_EXPAND, ctx->stream);
    RECD_HIP(ctx, hipGetLastError());
    return RECD_OK;
}

static constexpr int64_t kAllRunsRows = 16384;

recd_status recd_pooled_lookup_expand(recd_ctx *ctx, int F, int64_t B, int D, recd_dtype table_dt,
                                      recd_dtype out_dt, const void *const *tables, const int64_t *rows,
                                      const int64_t *u_values, const int64_t *run_index, int64_t max_runs,
                                      void *pooled, void *out)
{
    RECD_TRY(check_lookup_shape(ctx, F, D, table_dt, out_dt));
    RECD_TRY(recd_check_rows(ctx, F, rows));
    if (B < 0 || max_runs < 0)
        return recd_fail(ctx, RECD_EINVAL, "B or max_runs < 0");
    const int64_t n_rows = (int64_t)F * B;
    if (n_rows >= (int64_t)1 << 31)
        return recd_fail(ctx, RECD_EINVAL, "F*B must stay below 2^31");
    if (n_rows == 0)
        return RECD_OK;
    if (max_runs == 0 || max_runs > n_rows)
        max_runs = n_rows;
    if (max_runs < F)
        max_runs = F;  // every feature of a batch with rows starts a run
    if (!tables || !run_index || !pooled)
        return recd_fail(ctx, RECD_EINVAL, "null pointer argument");  // u_values may be null when M = 0
    for (int f = 0; f < F; f++)
        if (!tables[f])
            return recd_fail(ctx, RECD_EINVAL, "tables[%d] is null", f);
    RECD_HIP(ctx, hipSetDevice(ctx->device));
    if (ctx->validate) {
        if (!rows)
            return recd_fail(ctx, RECD_EINVAL, "validation needs rows[]");
        RECD_TRY(validate_run_index(ctx, F, B, rows, u_values, run_index));
    }
    // A small batch is bound by its launches, not by its gathers: there every run sums its list
    // itself (the same ids in the same order: the same bits as a copy) and no copy pass follows.
    const int all_runs = out && ctx->small_path != 0 && n_rows <= kAllRunsRows;
    for (int f0 = 0; f0 < F; f0 += RECD_F_PER_LAUNCH) {
        SegSumArgs a{};
        a.F = F - f0 < RECD_F_PER_LAUNCH ? F - f0 : RECD_F_PER_LAUNCH;
        a.F_all = F;
        a.D = D;
        a.table_dt = table_dt;
        a.out_dt = out_dt;
        for (int f = 0; f < a.F; f++)
            a.tables.p[f] = tables[f0 + f];
        a.values = u_values;
        a.values_are_i32 = 0;
        a.lists_bound = max_runs;
        a.site = RECD_SITE_UNIQUE_EXPAND;
        a.mode = RECD_POOL_SUM;
        a.out = pooled;
        a.run_index = run_index;
        a.expanded = out;
        a.B = B;
        a.feat_base = f0;
        a.all_runs = all_runs;
        RECD_TRY(recd_launch_segsum(ctx, a));
    }
    if (all_runs || !out)
        return RECD_OK;
    const int vecs = (int)((size_t)D * elem_size(out_dt) / 16);
    int64_t cb = (max_runs + 63) / 64;
    if (cb > (int64_t)ctx->num_cu * 16)
        cb = (int64_t)ctx->num_cu * 16;
    recd_time_begin(ctx, RECD_T_UNCOVERED, ctx->stream);
    hipLaunchKernelGGL(k_expand_runs, dim3((unsigned)cb), dim3(kBlock), 0, ctx->stream,
                       static_cast<const u32x4 *>(pooled), run_index, static_cast<u32x4 *>(out), vecs);
    recd_time_end(ctx, RECD_T_UNCOVERED, ctx->stream);
    RECD_HIP(ctx, hipGetLastError());
    return RECD_OK;
}

recd_status recd_group_sum_unique(recd_ctx *ctx, int F, int G, int D, recd_dtype dt,
                                  const int32_t *group_off, const void *pooled,
                                  const int64_t *feat_uoff, const int64_t *group_uoff,
                                  int64_t max_rows, void *combined)
{
    RECD_TRY(check_lookup_shape(ctx, F, D, dt, dt));
    if (G < 0 || G > F || max_rows < 0)
        return recd_fail(ctx, RECD_EINVAL, "bad sizes G=%d max_rows=%lld", G, (long long)max_rows);
    if (!group_off || group_off[0] != 0 || group_off[G] != F)
        return recd_fail(ctx, RECD_EINVAL, "group_off must run from 0 to F");
    for (int g = 0; g < G; g++)
        if (group_off[g + 1] <= group_off[g])
            return recd_fail(ctx, RECD_EINVAL, "group %d is empty or group_off decreases", g);
    if (G == 0 || max_rows == 0)
        return RECD_OK;
    if (!pooled || !feat_uoff || !group_uoff || !combined)
        return recd_fail(ctx, RECD_EINVAL, "null pointer argument");
    RECD_HIP(ctx, hipSetDevice(ctx->device));
    const int32_t *go_dev = nullptr, *fg_dev = nullptr;
    RECD_TRY(recd_group_map(ctx, F, G, group_off, &go_dev, &fg_dev));
    const int vecs = (int)((size_t)D * elem_size(dt) / 16);
    if (vecs > kBlock)
        return recd_fail(ctx, RECD_EINVAL, "row too long");
    const int64_t rows_per_block = kBlock / vecs;
    int64_t blocks = (max_rows + rows_per_block - 1) / rows_per_block;
    if (blocks > (int64_t)ctx->num_cu * 32)
        blocks = (int64_t)ctx->num_cu * 32;
#define RECD_GS(TT)                                                                              \
    hipLaunchKernelGGL((k_group_sum<TT>), dim3((unsigned)blocks), dim3(kBlock), 0, ctx->stream,  \
                       static_cast<const uint4 *>(pooled), feat_uoff, group_uoff, go_dev, G, vecs, \
                       max_rows, combined)
    if (dt == RECD_F32)
        RECD_GS(RECD_F32);
    else if (dt == RECD_F16)
        RECD_GS(RECD_F16);
    else
        RECD_GS(RECD_BF16);
#undef RECD_GS
    RECD_HIP(ctx, hipGetLastError());
    return RECD_OK;
}

recd_status recd_pooled_lookup_partial(recd_ctx *ctx, int F, int D, recd_dtype table_dt,
                                       recd_dtype out_dt, const void *const *tables,
                                       const int64_t *rows, const int64_t *p_values, int64_t P_cap,
                                       const int64_t *win_start, const int64_t *win_len,
                                       const int64_t *feat_uoff, int64_t max_lists, void *pooled)
{
    RECD_TRY(check_lookup_shape(ctx, F, D, table_dt, out_dt));
    RECD_TRY(recd_check_rows(ctx, F, rows));
    if (max_lists < 0 || P_cap < 0)
        return recd_fail(ctx, RECD_EINVAL, "max_lists or P_cap < 0");
    if (F == 0 || max_lists == 0)
        return RECD_OK;
    if (!tables || !win_start || !win_len || !feat_uoff || !pooled || (P_cap > 0 && !p_values))
        return recd_fail(ctx, RECD_EINVAL, "null pointer argument");
    for (int f = 0; f < F; f++)
        if (!tables[f])
            return recd_fail(ctx, RECD_EINVAL, "tables[%d] is null", f);
    RECD_HIP(ctx, hipSetDevice(ctx->device));
    if (ctx->validate) {
        if (!rows)
            return recd_fail(ctx, RECD_EINVAL, "validation needs rows[]");
        RECD_TRY(recd_reserve(ctx, 1024));
        int64_t *tmp = reinterpret_cast<int64_t *>(ctx->ws + 256);
        hipLaunchKernelGGL(k_read_i64, dim3(1), dim3(1), 0, ctx->stream, feat_uoff + F, tmp);
        RECD_HIP(ctx, hipMemcpyAsync(ctx->host_pinned + 1, tmp, 8, hipMemcpyDeviceToHost, ctx->stream));
        RECD_HIP(ctx, hipStreamSynchronize(ctx->stream));
        const int64_t U = ctx->host_pinned[1];
        if (U < 0 || U > max_lists)
            return recd_fail(ctx, RECD_ECAPACITY, "U=%lld exceeds max_lists=%lld", (long long)U,
                             (long long)max_lists);
        int *err = reinterpret_cast<int *>(ctx->ws);
        RECD_HIP(ctx, hipMemsetAsync(err, 0, sizeof(int), ctx->stream));
        for (int f = 0; f < F; f++)
            hipLaunchKernelGGL(k_validate_windows, dim3(64), dim3(256), 0, ctx->stream, p_values, P_cap,
                               win_start, win_len, feat_uoff, f, rows[f], err);
        ctx->host_pinned[0] = 0;
        RECD_HIP(ctx, hipMemcpyAsync(ctx->host_pinned, err, sizeof(int), hipMemcpyDeviceToHost, ctx->stream));
        RECD_HIP(ctx, hipStreamSynchronize(ctx->stream));
        if ((int)ctx->host_pinned[0] & 16)
            return recd_fail(ctx, RECD_EBOUNDS, "a window leaves the stored values");
        if ((int)ctx->host_pinned[0] & 2)
            return recd_fail(ctx, RECD_EBOUNDS, "an id lies outside its embedding table");
    }
    for (int f0 = 0; f0 < F; f0 += RECD_F_PER_LAUNCH) {
        SegSumArgs a{};
        a.F = F - f0 < RECD_F_PER_LAUNCH ? F - f0 : RECD_F_PER_LAUNCH;
        a.D = D;
        a.table_dt = table_dt;
        a.out_dt = out_dt;
        for (int f = 0; f < a.F; f++)
            a.tables.p[f] = tables[f0 + f];
        a.values = p_values;
        a.values_are_i32 = 0;
        a.offsets = win_start;
        a.lens = win_len;
        a.list_off = feat_uoff + f0;
        a.lists_bound = max_lists;
        a.site = RECD_SITE_UNIQUE;
        a.mode = RECD_POOL_SUM;
        a.out = pooled;
        RECD_TRY(recd_launch_segsum(ctx, a));
    }
    return RECD_OK;
}

} // extern "C"
