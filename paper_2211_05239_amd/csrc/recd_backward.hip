// Backward of expand + pooled lookup on an IKJT, and row-wise Adagrad on the touched rows.
//
//   step A  g_u[u,:] = sum_{b : inverse[f,b] = u} grad_out[f,b,:]            (b ascending)
//   step B  G_f[r,:] = sum_{j : u_values[j] = r} g_u[list of j,:]            (j ascending)
// Each step is "group the contributions by destination, then sum every group in a fixed order":
// a stable least-significant-digit radix sort of (destination key, source row) pairs puts equal
// destinations next to each other with their sources still ascending, head flags + a scan number
// the groups, and the segmented gather-sum kernel of the forward pass adds each group's rows.
// There are no floating-point atomics, so two runs give bit-identical gradients.
//
// Radix sort pass (digits of up to 9 bits): per-tile digit histograms -> one block per digit scans its
// row of tile counts -> scatter (which first scans the digit totals itself).  Inside a tile every
// wave owns a contiguous run of keys and walks it 64 keys at a time: ballots tell each lane which
// lanes hold its digit (its rank among them), a per-wave running digit count in LDS gives the rank
// among the wave's earlier keys, and a prefix over the four waves completes the stable rank.
#include "recd_internal.h"

#include <algorithm>
#include <type_traits>

namespace {

constexpr int kSortThreads = 256;
constexpr int kIPT = 8;                       // keys per thread in a tile
constexpr int kTile = kSortThreads * kIPT;    // keys per tile
constexpr int kRadixMax = 512;                // digits of up to 9 bits
constexpr int kScanItems = 4;                 // items per thread in the generic scan
constexpr int kScanTile = 256 * kScanItems;

// ---------------------------------------------------------------- block-wide exclusive scan (uint32)
__device__ __forceinline__ uint32_t block_excl_scan_u32(uint32_t v, uint32_t &total)
{
    __shared__ uint32_t s_w[16];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    uint32_t inc = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        uint32_t x = __shfl_up(inc, d);
        if (lane >= d)
            inc += x;
    }
    __syncthreads();
    if (lane == 63)
        s_w[w] = inc;
    __syncthreads();
    uint32_t off = 0;
    total = 0;
    for (int i = 0; i < (int)(blockDim.x >> 6); i++) {
        if (i < w)
            off += s_w[i];
        total += s_w[i];
    }
    return off + inc - v;
}

// n may live on the device (n_dev != nullptr) or be given directly
__device__ __forceinline__ int64_t count_of(const int64_t *n_dev, int64_t n_host)
{
    return n_dev ? *n_dev : n_host;
}

__global__ __launch_bounds__(1024) void k_scan_small(uint32_t *a, int64_t n)
{
    uint32_t carry = 0;
    for (int64_t base = 0; base < n; base += 1024) {
        const int64_t i = base + threadIdx.x;
        const uint32_t v = i < n ? a[i] : 0;
        uint32_t total;
        const uint32_t e = block_excl_scan_u32(v, total);
        if (i < n)
            a[i] = carry + e;
        carry += total;
    }
}

// ---------------------------------------------------------------- stable LSD radix sort of pairs
template <typename KeyT>
__global__ __launch_bounds__(kSortThreads) void k_sort_hist(const KeyT *__restrict__ keys,
                                                            const int64_t *n_dev, int64_t n_host,
                                                            int shift, int dbits,
                                                            uint32_t *__restrict__ hist, int ntiles)
{
    __shared__ uint32_t s_h[kRadixMax];
    // every XCD takes a contiguous eighth of the tiles (see k_sort_scatter): the counters that
    // neighbouring tiles write lie next to each other in a digit's row
    const int tiles_per_xcd = (ntiles + 7) / 8;
    const int tile = (int)(blockIdx.x % 8) * tiles_per_xcd + (int)(blockIdx.x / 8);
    if (tile >= ntiles)
        return;
    const uint32_t radix = 1u << dbits;
    for (uint32_t d = threadIdx.x; d < radix; d += kSortThreads)
        s_h[d] = 0;
    __syncthreads();
    const int64_t n = count_of(n_dev, n_host);
    const int64_t base = (int64_t)tile * kTile;
#pragma unroll
    for (int k = 0; k < kIPT; k++) {
        const int64_t i = base + k * kSortThreads + threadIdx.x;
        if (i < n)
            atomicAdd(&s_h[(uint32_t)(keys[i] >> shift) & (radix - 1)], 1u);
    }
    __syncthreads();
    for (uint32_t d = threadIdx.x; d < radix; d += kSortThreads)
        hist[(int64_t)d * ntiles + tile] = s_h[d];
}

// one block per digit: in-place exclusive scan of the digit's row of tile counts; row total out
__global__ __launch_bounds__(256) void k_sort_rowscan(uint32_t *__restrict__ hist, int ntiles,
                                                      uint32_t *__restrict__ digit_total)
{
    uint32_t *row = hist + (int64_t)blockIdx.x * ntiles;
    uint32_t carry = 0;
    for (int base = 0; base < ntiles; base += 256) {
        const int i = base + threadIdx.x;
        const uint32_t v = i < ntiles ? row[i] : 0;
        uint32_t total;
        const uint32_t e = block_excl_scan_u32(v, total);
        if (i < ntiles)
            row[i] = carry + e;
        carry += total;
    }
    if (threadIdx.x == 0)
        digit_total[blockIdx.x] = carry;
}

template <typename KeyT>
__global__ __launch_bounds__(kSortThreads) void k_sort_scatter(
    const KeyT *__restrict__ kin, const uint32_t *__restrict__ pin, KeyT *__restrict__ kout,
    uint32_t *__restrict__ pout, const int64_t *n_dev, int64_t n_host, int shift, int dbits,
    const uint32_t *__restrict__ hist_scanned, const uint32_t *__restrict__ digit_total, int ntiles)
{
    constexpr int W = kSortThreads / 64;
    constexpr int kPerWave = 64 * kIPT;  // contiguous keys of one wave
    __shared__ uint32_t s_run[W][kRadixMax];  // per wave: keys seen so far per digit
    __shared__ uint32_t s_base[kRadixMax];    // where this tile's keys of a digit start in the output
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const uint32_t radix = 1u << dbits;
    const int64_t n = count_of(n_dev, n_host);
    // Blocks go to the XCDs in turn; every XCD takes a contiguous eighth of the tiles, so that the
    // short runs that neighbouring tiles append to one digit's output meet in one L2 and leave it
    // as whole lines.
    const int tiles_per_xcd = (ntiles + 7) / 8;
    const int tile = (int)(blockIdx.x % 8) * tiles_per_xcd + (int)(blockIdx.x / 8);
    const int64_t base = (int64_t)tile * kTile;
    if (tile >= ntiles || base >= n)
        return;  // whole block: nothing in this tile
    // digit bases = exclusive scan of the digit totals (two digits per thread), plus this tile's
    // offset inside the digit
    {
        const uint32_t d0 = 2 * tid, d1 = 2 * tid + 1;
        const uint32_t t0 = d0 < radix ? digit_total[d0] : 0, t1 = d1 < radix ? digit_total[d1] : 0;
        uint32_t total;
        const uint32_t e = block_excl_scan_u32(t0 + t1, total);
        if (d0 < radix)
            s_base[d0] = e + hist_scanned[(int64_t)d0 * ntiles + tile];
        if (d1 < radix)
            s_base[d1] = e + t0 + hist_scanned[(int64_t)d1 * ntiles + tile];
    }
    for (int i = tid; i < W * kRadixMax; i += kSortThreads)
        (&s_run[0][0])[i] = 0;
    __syncthreads();

    KeyT key[kIPT];
    uint32_t rank[kIPT];
    const uint64_t lt_mask = lane == 0 ? 0ull : (~0ull >> (64 - lane));
    const int64_t wbase = base + (int64_t)w * kPerWave;
#pragma unroll
    for (int k = 0; k < kIPT; k++) {
        const int64_t i = wbase + k * 64 + lane;
        const bool valid = i < n;
        key[k] = valid ? kin[i] : (KeyT)0;
        const uint32_t d = (uint32_t)(key[k] >> shift) & (radix - 1);
        uint64_t mask = __ballot(valid);
#pragma unroll
        for (int bit = 0; bit < 9; bit++) {
            if (bit < dbits) {  // uniform
                const bool one = (d >> bit) & 1u;
                const uint64_t bal = __ballot(one);
                mask &= one ? bal : ~bal;
            }
        }
        const uint32_t in_round = (uint32_t)__popcll(mask & lt_mask);
        // keys of this digit in the wave's earlier rounds; the first lane of each digit then adds
        // this round's count (same wave: the read above is complete before the write is issued)
        const uint32_t before = valid ? s_run[w][d] : 0;
        __builtin_amdgcn_wave_barrier();
        if (valid && in_round == 0)
            s_run[w][d] = before + (uint32_t)__popcll(mask);
        __builtin_amdgcn_wave_barrier();
        rank[k] = before + in_round;
    }
    __syncthreads();
    // s_run[w][d] now holds wave w's count of digit d: exclusive prefix over the waves
    for (uint32_t d = tid; d < radix; d += kSortThreads) {
        uint32_t run = 0;
#pragma unroll
        for (int ww = 0; ww < W; ww++) {
            const uint32_t c = s_run[ww][d];
            s_run[ww][d] = run;
            run += c;
        }
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < kIPT; k++) {
        const int64_t i = wbase + k * 64 + lane;
        if (i < n) {
            const uint32_t d = (uint32_t)(key[k] >> shift) & (radix - 1);
            const int64_t dst = (int64_t)s_base[d] + s_run[w][d] + rank[k];
            kout[dst] = key[k];
            pout[dst] = pin[i];
        }
    }
}

// Sorts (keys, pay) by the low `bits` bits of the key; returns through *kres/*pres which of the two
// buffer pairs holds the result.
template <typename KeyT>
recd_status radix_sort_pairs(recd_ctx *ctx, hipStream_t st, KeyT *k0, uint32_t *p0, KeyT *k1,
                             uint32_t *p1, const int64_t *n_dev, int64_t n_cap, int bits,
                             uint32_t *hist, uint32_t *bsum, KeyT **kres, uint32_t **pres)
{
    const int ntiles = (int)((n_cap + kTile - 1) / kTile);
    KeyT *ka = k0, *kb = k1;
    uint32_t *pa = p0, *pb = p1;
    // fewest passes with digits of at most 9 bits, digits as even as possible
    const int passes = (bits + 8) / 9;
    const int dbits = passes > 0 ? (bits + passes - 1) / passes : 0;
    for (int shift = 0; shift < bits && ntiles > 0; shift += dbits) {
        hipLaunchKernelGGL((k_sort_hist<KeyT>), dim3(8 * ((ntiles + 7) / 8)), dim3(kSortThreads), 0, st, ka, n_dev,
                           n_cap, shift, dbits, hist, ntiles);
        hipLaunchKernelGGL(k_sort_rowscan, dim3(1u << dbits), dim3(256), 0, st, hist, ntiles, bsum);
        hipLaunchKernelGGL((k_sort_scatter<KeyT>), dim3(8 * ((ntiles + 7) / 8)), dim3(kSortThreads), 0, st, ka, pa, kb,
                           pb, n_dev, n_cap, shift, dbits, hist, bsum, ntiles);
        KeyT *tk = ka; ka = kb; kb = tk;
        uint32_t *tp = pa; pa = pb; pb = tp;
    }
    RECD_HIP(ctx, hipGetLastError());
    *kres = ka;
    *pres = pa;
    return RECD_OK;
}

// ---------------------------------------------------------------- keys
// step A: destination = global unique-list index, source = row (f,b) of grad_out
__global__ void k_keys_rows(const int32_t *__restrict__ inverse, const int64_t *__restrict__ feat_uoff,
                            int64_t B, int64_t n_lists, uint32_t *__restrict__ keys,
                            uint32_t *__restrict__ pay, int64_t *n_out)
{
    const int64_t l = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (l == 0) {
        n_out[0] = n_lists;
        n_out[1] = 0;
    }
    if (l < n_lists) {
        keys[l] = (uint32_t)(feat_uoff[l / B] + inverse[l]);
        pay[l] = (uint32_t)l;
    }
}

// step B: destination = (feature, table row), source = unique list holding position j
template <typename KeyT, int SG>
__global__ __launch_bounds__(256) void k_keys_ids(const int64_t *__restrict__ u_values,
                                                  const int64_t *__restrict__ u_offsets,
                                                  const int64_t *__restrict__ feat_uoff, int F,
                                                  int row_bits, int64_t lists_cap, int64_t M_cap,
                                                  KeyT *__restrict__ keys, uint32_t *__restrict__ pay,
                                                  int64_t *n_out, int pay_positions,
                                                  uint32_t *__restrict__ pos_list = nullptr)
{
    const int s = threadIdx.x % SG;
    const int per_block = blockDim.x / SG;
    int64_t U = feat_uoff[F];
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        // never write past the caller's capacity; n_out[1] tells the host that M_cap was too small
        const int64_t M = u_offsets[U];
        n_out[0] = M < M_cap ? M : M_cap;
        n_out[1] = M > M_cap ? 1 : 0;
    }
    if (U > lists_cap)
        U = lists_cap;
    // the grid is sized by the caller's bound on U and strides, so any bound gives the same keys
    for (int64_t u = (int64_t)blockIdx.x * per_block + threadIdx.x / SG; u < U; u += (int64_t)gridDim.x * per_block) {
        int lo = 0, hi = F;  // feature of u: feat_uoff[f] <= u < feat_uoff[f+1]
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (feat_uoff[mid] <= u)
                lo = mid;
            else
                hi = mid;
        }
        const KeyT fkey = (KeyT)lo << row_bits;
        const int64_t j0 = u_offsets[u];
        const int64_t j1 = u_offsets[u + 1] < M_cap ? u_offsets[u + 1] : M_cap;
        for (int64_t j = j0 + s; j < j1; j += SG) {
            keys[j] = fkey | (KeyT)u_values[j];
            pay[j] = pay_positions ? (uint32_t)j : (uint32_t)u;  // source row of the later sum: g_emb[j] or g_u[u]
            if (pos_list)
                pos_list[j] = (uint32_t)u;
        }
    }
}

// Blocks of k_keys_ids for a caller's bound on U (at least one; never more than the lists there are).
static unsigned keys_ids_blocks(int64_t U_cap, int64_t n_lists, int SG, int block)
{
    int64_t lists = U_cap < n_lists ? U_cap : n_lists;
    if (lists < 1)
        lists = 1;
    const int per_block = block / SG;
    return (unsigned)((lists + per_block - 1) / per_block);
}

// Weighted lookup: the sort carried the position j of every entry.  Replace it by the entry's
// source row (the unique list of j) and fetch the entry's weight, both in sorted order, so that the
// segment sums read them as streams.
__global__ __launch_bounds__(256) void k_weight_payload(uint32_t *__restrict__ pay,
                                                        const uint32_t *__restrict__ pos_list,
                                                        const float *__restrict__ u_weights,
                                                        const int64_t *__restrict__ n_dev,
                                                        float *__restrict__ pay_w)
{
    const int64_t n = *n_dev;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (int64_t)gridDim.x * blockDim.x) {
        const uint32_t j = pay[i];
        pay_w[i] = u_weights[j];
        pay[i] = pos_list[j];
    }
}

// ---------------------------------------------------------------- step A from the batch's runs
// With session-clustered batches the rows that name one unique list come in runs of adjacent rows
// (the run index of the builder).  Grouping the rows by unique list then only needs the runs: keys =
// unique list of every run, payload = run number, the same stable sort (runs of a list stay in row
// order), and an expansion of the sorted runs into the row list that the sort of all F*B rows would
// have produced - the same rows in the same order, so the segment sums that follow are unchanged.
__global__ __launch_bounds__(256) void k_run_keys(const int64_t *__restrict__ run_index, int64_t runs_cap,
                                                  uint32_t *__restrict__ keys, uint32_t *__restrict__ pay,
                                                  int64_t *n_out)
{
    const int64_t all = run_index[0];
    const int64_t n = all < runs_cap ? all : runs_cap;
    const int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (r == 0) {
        n_out[0] = n;
        n_out[1] = all > runs_cap ? 1 : 0;  // the caller's bound on the runs was too small
    }
    if (r < n) {
        keys[r] = (uint32_t)((uint64_t)run_index[3 * (1 + r)] >> 32) & 0x7fffffffu;
        pay[r] = (uint32_t)r;
    }
}

// Sorted runs (ks = unique list, ps = run number).  EMIT = false: per tile, the number of lists that
// start in it and the rows of its runs.  EMIT = true, with both tile arrays scanned: seg_start of
// every list (in rows), list_off = {0, lists}, and the rows of every run written out in order.
template <bool EMIT>
__global__ __launch_bounds__(256) void k_run_rows(const uint32_t *__restrict__ ks, const uint32_t *__restrict__ ps,
                                                  const int64_t *__restrict__ run_index,
                                                  const int64_t *__restrict__ n_dev,
                                                  uint32_t *__restrict__ tile_heads,
                                                  uint32_t *__restrict__ tile_rows,
                                                  int64_t *__restrict__ seg_start,
                                                  int64_t *__restrict__ list_off, uint32_t *__restrict__ rows_out,
                                                  int64_t *long_count)
{
    const int64_t n = *n_dev;
    if (EMIT && blockIdx.x == 0 && threadIdx.x == 0) {
        long_count[0] = 0;
        long_count[1] = 0;
        if (n == 0) {
            seg_start[0] = 0;
            list_off[0] = 0;
            list_off[1] = 0;
        }
    }
    const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * kScanItems;
    uint32_t prev = (base > 0 && base <= n) ? ks[base - 1] : 0u;
    uint32_t head[kScanItems], row0[kScanItems], len[kScanItems];
    uint32_t hs = 0, rs = 0;
#pragma unroll
    for (int k = 0; k < kScanItems; k++) {
        const int64_t i = base + k;
        head[k] = 0;
        row0[k] = 0;
        len[k] = 0;
        if (i < n) {
            const uint32_t key = ks[i];
            const int64_t r = ps[i];
            head[k] = (i == 0 || key != prev) ? 1u : 0u;
            row0[k] = (uint32_t)(uint64_t)run_index[3 * (1 + r)];
            len[k] = (uint32_t)(uint64_t)run_index[3 * (2 + r)] - row0[k];
            prev = key;
        }
        hs += head[k];
        rs += len[k];
    }
    uint32_t th, tr;
    const uint32_t eh = block_excl_scan_u32(hs, th);
    const uint32_t er = block_excl_scan_u32(rs, tr);
    if (!EMIT) {
        if (threadIdx.x == 0) {
            tile_heads[blockIdx.x] = th;
            tile_rows[blockIdx.x] = tr;
        }
        return;
    }
    int64_t h = (int64_t)tile_heads[blockIdx.x] + eh;  // lists that start before this thread's runs
    int64_t at = (int64_t)tile_rows[blockIdx.x] + er;  // rows before them
#pragma unroll
    for (int k = 0; k < kScanItems; k++) {
        const int64_t i = base + k;
        if (i < n) {
            if (head[k])
                seg_start[h] = at;
            for (uint32_t t = 0; t < len[k]; t++)
                rows_out[at + t] = row0[k] + t;
            h += head[k];
            at += len[k];
            if (i == n - 1) {
                seg_start[h] = at;
                list_off[0] = 0;
                list_off[1] = h;
            }
        }
    }
}

// ---------------------------------------------------------------- segments of equal keys
// A head is an element whose key differs from its predecessor's (or the first element).  Numbering
// the heads is an exclusive scan of the head flags; the flags are recomputed from the keys where
// they are needed instead of being stored: k_head_count (heads per tile) -> k_scan_small (tile
// offsets) -> k_segments (segment number of every head, and what hangs on it).
template <typename KeyT>
__global__ __launch_bounds__(256) void k_head_count(const KeyT *__restrict__ keys, const int64_t *n_dev,
                                                    uint32_t *__restrict__ bsum, int64_t *long_count)
{
    const int64_t n = *n_dev;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        long_count[0] = 0;
        long_count[1] = 0;
    }
    const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * kScanItems;
    KeyT prev = (base > 0 && base <= n) ? keys[base - 1] : (KeyT)0;
    uint32_t s = 0;
#pragma unroll
    for (int k = 0; k < kScanItems; k++) {
        const int64_t i = base + k;
        if (i < n) {
            const KeyT key = keys[i];
            s += (i == 0 || key != prev) ? 1u : 0u;
            prev = key;
        }
    }
    uint32_t total;
    block_excl_scan_u32(s, total);
    if (threadIdx.x == 0)
        bsum[blockIdx.x] = total;
}

// bsum holds the exclusive scan of the per-tile head counts.  Heads record where their segment
// starts; the last element closes the list (seg_start[R] = n, list_off = {0, R}).  With
// row_bits >= 0 the key is (feature, row): also emit the row ids, the feature of every segment and
// the per-feature prefix of distinct-row counts.
template <typename KeyT>
__global__ __launch_bounds__(256) void k_segments(const KeyT *__restrict__ keys, const int64_t *n_dev,
                                                  const uint32_t *__restrict__ bsum,
                                                  int64_t *__restrict__ seg_start,
                                                  int64_t *__restrict__ list_off, int row_bits, int F,
                                                  int64_t *__restrict__ touched_rows,
                                                  int64_t *__restrict__ feat_roff,
                                                  int32_t *__restrict__ seg_feat)
{
    const int64_t n = *n_dev;
    if (n == 0) {
        if (blockIdx.x == 0 && threadIdx.x == 0) {
            seg_start[0] = 0;
            list_off[0] = 0;
            list_off[1] = 0;
            if (row_bits >= 0)
                for (int f = 0; f <= F; f++)
                    feat_roff[f] = 0;
        }
        return;
    }
    const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * kScanItems;
    const KeyT before = (base > 0 && base <= n) ? keys[base - 1] : (KeyT)0;
    KeyT key[kScanItems];
    uint32_t s = 0;
    {
        KeyT prev = before;
#pragma unroll
        for (int k = 0; k < kScanItems; k++) {
            const int64_t i = base + k;
            key[k] = i < n ? keys[i] : (KeyT)0;
            if (i < n)
                s += (i == 0 || key[k] != prev) ? 1u : 0u;
            prev = key[k];
        }
    }
    uint32_t total;
    int64_t sidx = (int64_t)bsum[blockIdx.x] + block_excl_scan_u32(s, total);  // heads before `base`
    KeyT prev = before;
#pragma unroll
    for (int k = 0; k < kScanItems; k++) {
        const int64_t i = base + k;
        if (i < n) {
            const bool head = i == 0 || key[k] != prev;
            if (head) {
                seg_start[sidx] = i;
                if (row_bits >= 0) {
                    touched_rows[sidx] = (int64_t)(key[k] & (((KeyT)1 << row_bits) - 1));
                    const int f = (int)(key[k] >> row_bits);
                    seg_feat[sidx] = f;
                    const int fprev = i == 0 ? -1 : (int)(prev >> row_bits);
                    for (int ff = fprev + 1; ff <= f; ff++)
                        feat_roff[ff] = sidx;
                }
            }
            if (i == n - 1) {
                const int64_t R = sidx + (head ? 1 : 0);
                seg_start[R] = n;
                list_off[0] = 0;
                list_off[1] = R;
                if (row_bits >= 0) {
                    const int f = (int)(key[k] >> row_bits);
                    for (int ff = f + 1; ff <= F; ff++)
                        feat_roff[ff] = R;
                }
            }
            sidx += head ? 1 : 0;
            prev = key[k];
        }
    }
}

// ---------------------------------------------------------------- row-wise Adagrad
// One 32-lane group per touched row k (rows of features [f0, f0+nf) only):
//   m[r] += mean_d G[k,d]^2 ;  W[r,d] -= lr * G[k,d] / (sqrt(m[r]) + eps)
struct OptPtrs {
    float *w[RECD_F_PER_LAUNCH];
    float *m[RECD_F_PER_LAUNCH];
};

__global__ __launch_bounds__(256) void k_adagrad(const float *__restrict__ grad_rows,
                                                 const int64_t *__restrict__ touched_rows,
                                                 const int64_t *__restrict__ feat_roff, int f0, int nf,
                                                 int D, OptPtrs ptrs, float lr, float eps)
{
    constexpr int SG = 32;
    const int s = threadIdx.x % SG;
    const int64_t k0 = feat_roff[f0], k1 = feat_roff[f0 + nf];
    const int vecs = D / 4;
    for (int64_t k = k0 + (int64_t)blockIdx.x * (256 / SG) + threadIdx.x / SG; k < k1;
         k += (int64_t)gridDim.x * (256 / SG)) {
        int lo = f0, hi = f0 + nf;
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (feat_roff[mid] <= k)
                lo = mid;
            else
                hi = mid;
        }
        const int64_t r = touched_rows[k];
        const float4 *g = reinterpret_cast<const float4 *>(grad_rows + k * D);
        float ss = 0.f;
        for (int v = s; v < vecs; v += SG) {
            const float4 x = g[v];
            ss += x.x * x.x;
            ss += x.y * x.y;
            ss += x.z * x.z;
            ss += x.w * x.w;
        }
#pragma unroll
        for (int m = SG / 2; m > 0; m >>= 1)
            ss += __shfl_xor(ss, m, SG);
        float *mp = ptrs.m[lo - f0] + r;
        const float mnew = *mp + ss / (float)D;
        const float scale = lr / (sqrtf(mnew) + eps);
        float4 *w = reinterpret_cast<float4 *>(ptrs.w[lo - f0] + r * D);
        for (int v = s; v < vecs; v += SG) {
            const float4 x = g[v];
            float4 y = w[v];
            y.x -= scale * x.x;
            y.y -= scale * x.y;
            y.z -= scale * x.z;
            y.w -= scale * x.w;
            w[v] = y;
        }
        // every lane has read *mp before any lane of the group overwrites it
        __builtin_amdgcn_wave_barrier();
        if (s == 0)
            *mp = mnew;
    }
}

// ---------------------------------------------------------------- row-gradient segment sum
// Step B has very many very short segments (a table row is named by a handful of unique lists, a
// few hot rows by thousands).  Here a group of LPR lanes owns a whole segment: G = 64/LPR segments
// advance side by side in one wave, each lane carries up to four 16-byte pieces of the row, no
// cross-lane fold is needed, and the Adagrad update of the destination row follows in the same
// lanes.  Segments longer than the cut (32 or 64 entries, see long_seg_cut) are only recorded; the block-cooperative gather-sum
// kernel sums them afterwards.  Order of additions inside a segment: ascending position.
struct RowSumParams {
    const float *table;        // g_u [U, D]
    const uint32_t *pay;       // sorted payload: unique-list index of every position
    const float *pay_w;        // weighted lookup: the weight of every sorted entry, else nullptr
    const int64_t *seg_start;  // [R+1]
    const int64_t *n_seg;      // device: R
    float *out;                // grad_rows [R, D] or nullptr
    int D;
    int pieces;                // D / 4
    // segments longer than long_seg entries are cut into chunks (work items) whose partial sums another
    // kernel computes; lseg_* describe the cut segments, item_* the chunks
    int64_t *long_count;       // [0] cut segments, [1] chunks
    int32_t *lseg_t, *lseg_first, *lseg_n;
    int64_t *item_start, *item_end;
    const float *partials;     // [chunks, D] (k_long_finalize)
    int long_seg;              // segments with more entries than this are the cut ones
};

// Tail of a row-gradient segment held by a lane group: acc = the segment's sum (piece w of lane r).
// Applies row-wise Adagrad to the destination row (operands fetched earlier into wreg/mreg) and/or
// stores the gradient row.
template <int LPR>
__device__ __forceinline__ void finish_segment(const RowSumParams &p, const OptAdagrad &opt, int64_t t,
                                               const float4 *acc, const float4 *wreg, float mreg,
                                               float *wrow, float *mp, const bool *piece, int r,
                                               bool update)
{
    constexpr int VPL = 4;
    if (update) {
        float ss = 0.f;
#pragma unroll
        for (int w = 0; w < VPL; w++)
            if (piece[w]) {
                ss += acc[w].x * acc[w].x;
                ss += acc[w].y * acc[w].y;
                ss += acc[w].z * acc[w].z;
                ss += acc[w].w * acc[w].w;
            }
#pragma unroll
        for (int s = 1; s < LPR; s <<= 1)
            ss += __shfl_xor(ss, s);
        const float mnew = mreg + ss / (float)p.D;
        const float scale = opt.lr / (sqrtf(mnew) + opt.eps);
#pragma unroll
        for (int w = 0; w < VPL; w++)
            if (piece[w]) {
                float4 x = wreg[w];
                x.x -= scale * acc[w].x;
                x.y -= scale * acc[w].y;
                x.z -= scale * acc[w].z;
                x.w -= scale * acc[w].w;
                {
                    typedef float f32x4s __attribute__((ext_vector_type(4)));
                    const f32x4s xo = {x.x, x.y, x.z, x.w};
                    __builtin_nontemporal_store(xo, reinterpret_cast<f32x4s *>(wrow) + w * LPR + r);
                }
            }
        if (r == 0)
            *mp = mnew;
    }
    if (p.out) {
        typedef float f32x4 __attribute__((ext_vector_type(4)));
        f32x4 *dst = reinterpret_cast<f32x4 *>(p.out + t * p.D);
#pragma unroll
        for (int w = 0; w < VPL; w++)
            if (piece[w]) {
                const f32x4 o = {acc[w].x, acc[w].y, acc[w].z, acc[w].w};
                __builtin_nontemporal_store(o, &dst[w * LPR + r]);
            }
    }
}

// Segments longer than p.long_seg entries are cut into chunks of 256 entries, or larger ones if that would
// give more than 64 chunks.  The cut depends on the segment's length only; the order in which
// segments and chunks are listed does not matter for the sums.
__global__ __launch_bounds__(256) void k_find_long(const RowSumParams p)
{
    const int64_t R = *p.n_seg;
    for (int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; k < R;
         k += (int64_t)gridDim.x * blockDim.x) {
        const int64_t start = p.seg_start[k], end = p.seg_start[k + 1];
        const int64_t len = end - start;
        if (len <= p.long_seg)
            continue;
        int64_t ch = 256;
        if ((len + ch - 1) / ch > 64)
            ch = (len + 63) / 64;
        const int nch = (int)((len + ch - 1) / ch);
        const int64_t first = (int64_t)atomicAdd(reinterpret_cast<unsigned long long *>(p.long_count + 1),
                                                 (unsigned long long)nch);
        const int64_t slot = (int64_t)atomicAdd(reinterpret_cast<unsigned long long *>(p.long_count), 1ull);
        p.lseg_t[slot] = (int32_t)k;
        p.lseg_first[slot] = (int32_t)first;
        p.lseg_n[slot] = nch;
        for (int c = 0; c < nch; c++) {
            p.item_start[first + c] = start + c * ch;
            p.item_end[first + c] = start + (c + 1) * ch < end ? start + (c + 1) * ch : end;
        }
    }
}

// FINALIZE = false: segments of at most p.long_seg entries are summed here (longer ones are skipped).
// FINALIZE = true: the "segments" are the cut ones; their entries are the chunk partial sums, in
// chunk order.
// WT (with FINALIZE = false): entry j contributes pay_w[j] times its source row.
template <int LPR, bool FINALIZE, bool WT = false>
__global__ __launch_bounds__(256) void k_segsum_rows(const RowSumParams p, const OptAdagrad opt)
{
    constexpr int G = 64 / LPR, VPL = 4;
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int g = lane / LPR, r = lane % LPR;
    const int64_t R = FINALIZE ? p.long_count[0] : *p.n_seg;
    const int per_block = (256 / 64) * G;
    const float4 *table = reinterpret_cast<const float4 *>(FINALIZE ? p.partials : p.table);
    bool piece[VPL];
#pragma unroll
    for (int w = 0; w < VPL; w++)
        piece[w] = w * LPR + r < p.pieces;

    // The segments are ordered by (feature, row) and their entries name rows of the source array that
    // belong to the same feature.  Blocks go to the XCDs in turn; every XCD takes a contiguous eighth
    // of the segments and its blocks stride through it side by side, so that the source rows an XCD
    // gathers at one time are a few features' worth and stay in its L2.
    // The few cut segments of the FINALIZE pass, and any grid that is not a multiple of 8 blocks, are
    // dealt to the blocks in turn instead.
    const bool by_xcd = !FINALIZE && gridDim.x % 8 == 0;
    const int64_t groups = (R + per_block - 1) / per_block;
    const int64_t per_xcd = (groups + 7) / 8;
    const int64_t g_first = by_xcd ? (int64_t)(blockIdx.x % 8) * per_xcd : 0;
    const int64_t g_count = by_xcd ? (per_xcd < groups - g_first ? per_xcd : groups - g_first) : groups;
    const int64_t g_step = by_xcd ? gridDim.x / 8 : gridDim.x;
    for (int64_t gi = by_xcd ? blockIdx.x / 8 : blockIdx.x; gi < g_count; gi += g_step) {
        const int64_t t0 = (g_first + gi) * per_block;
        const int64_t k = t0 + wv * G + g;
        int64_t t = k;       // destination segment
        int64_t start = 0;
        int n = 0;
        int f_seg = 0;
        int64_t row_seg = 0;
        if (k < R) {
            if (FINALIZE) {
                t = p.lseg_t[k];
                start = p.lseg_first[k];
                n = p.lseg_n[k];
            } else {
                // one round trip: where the segment lies, and (for the update) which row it is
                start = p.seg_start[k];
                const int64_t end = p.seg_start[k + 1];
                if (opt.n_feat > 0) {
                    f_seg = opt.seg_feat[k];
                    row_seg = opt.touched_rows[k];
                }
                const int64_t len = end - start;
                n = len <= p.long_seg ? (int)len : 0;  // longer segments were cut into chunks by k_find_long
            }
        }
        const bool mine = n > 0;  // uniform inside the lane group
        const bool update = mine && opt.n_feat > 0;
        // second round trip: the segment's entries (the first kPre * LPR of them, one load per lane
        // and LPR entries) together with the destination row and its accumulator
        constexpr int kPre = FINALIZE ? 0 : 4;
        uint32_t pre[kPre > 0 ? kPre : 1];
        float prew[kPre > 0 ? kPre : 1];
#pragma unroll
        for (int u = 0; u < kPre; u++) {
            const int idx = u * LPR + r;
            pre[u] = idx < n ? p.pay[start + idx] : 0u;
            prew[u] = (WT && idx < n) ? p.pay_w[start + idx] : 1.f;
        }
        float4 wreg[VPL];
        float mreg = 0.f;
        float *wrow = nullptr, *mp = nullptr;
        if (update) {
            if (FINALIZE) {
                f_seg = opt.seg_feat[t];
                row_seg = opt.touched_rows[t];
            }
            mp = opt.m[f_seg] + row_seg;
            wrow = opt.w[f_seg] + row_seg * p.D;
            mreg = *mp;
#pragma unroll
            for (int w = 0; w < VPL; w++)
                if (piece[w])
                {
                    typedef float f32x4l __attribute__((ext_vector_type(4)));
                    const f32x4l t = __builtin_nontemporal_load(reinterpret_cast<const f32x4l *>(wrow) + w * LPR + r);
                    wreg[w] = make_float4(t.x, t.y, t.z, t.w);
                }
        }
        float4 acc[VPL];
#pragma unroll
        for (int w = 0; w < VPL; w++)
            acc[w] = make_float4(0.f, 0.f, 0.f, 0.f);
        // one entry: the source row `id` (times wt) added to the segment's sum
        auto add_entry = [&](int64_t id, float wt) {
            float4 v[VPL];
#pragma unroll
            for (int w = 0; w < VPL; w++)
                if (piece[w])
                    v[w] = table[id * p.pieces + w * LPR + r];
#pragma unroll
            for (int w = 0; w < VPL; w++)
                if (piece[w]) {
                    if (WT) {
                        acc[w].x = __fmaf_rn(wt, v[w].x, acc[w].x);
                        acc[w].y = __fmaf_rn(wt, v[w].y, acc[w].y);
                        acc[w].z = __fmaf_rn(wt, v[w].z, acc[w].z);
                        acc[w].w = __fmaf_rn(wt, v[w].w, acc[w].w);
                    } else {
                        acc[w].x += v[w].x;
                        acc[w].y += v[w].y;
                        acc[w].z += v[w].z;
                        acc[w].w += v[w].w;
                    }
                }
        };
        // entries in ascending order: the fetched ones come out of the lane group's registers, any
        // further ones (cuts above kPre * LPR entries) are read one by one
        const int gbase = lane - r;
#pragma unroll
        for (int u = 0; u < kPre; u++) {
            const int cnt = n - u * LPR < LPR ? n - u * LPR : LPR;
            for (int ii = 0; ii < cnt; ii++) {
                const uint32_t id = __shfl(pre[u], gbase + ii);
                const float wt = WT ? __shfl(prew[u], gbase + ii) : 1.f;
                add_entry((int64_t)id, wt);
            }
        }
        for (int i = kPre * LPR; i < n; i++) {
            const int64_t j = start + i;
            add_entry(FINALIZE ? j : (int64_t)p.pay[j], WT ? p.pay_w[j] : 1.f);
        }
        if (mine)
            finish_segment<LPR>(p, opt, t, acc, wreg, mreg, wrow, mp, piece, r, update);
    }
}

// ---------------------------------------------------------------- max pooling: route g_u to the winners
// Backward of the max-pooled lookup: element d of g_u[u] belongs to the position of list u that holds
// the largest table element d (the first such position).  A group of LPR lanes owns a unique list
// (lane r: pieces r, r + LPR, ... of the row, 16 bytes each; one piece per lane up to 1 KiB rows):
// pass 1 walks the list's table rows, eight loads in flight per lane, and keeps the running
// maximum and its position per element, pass 2 writes one row per position,
// g_u[u] masked to the elements that position won, into emb[M, D].  The row-gradient segment sum
// then adds those rows per table row exactly as it does for the sequence path.
struct MaxTables {
    const float *w[RECD_F_PER_LAUNCH];
};

template <int LPR, int VPL>
__global__ __launch_bounds__(256) void k_max_route(const int64_t *__restrict__ u_values,
                                                   const int64_t *__restrict__ u_offsets,
                                                   const int64_t *__restrict__ feat_uoff, int f0, int nf,
                                                   MaxTables tabs, const float4 *__restrict__ g_u,
                                                   float4 *__restrict__ emb, int pieces, int64_t lists_cap,
                                                   int64_t m_cap)
{
    constexpr int G = 64 / LPR, US = 8 / VPL;  // US positions of a list in flight per lane
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int g = lane / LPR, r = lane % LPR;
    const int per_block = (256 / 64) * G;
    const int64_t u_lo = feat_uoff[f0];
    int64_t u_hi = feat_uoff[f0 + nf];
    u_hi = u_hi < lists_cap ? u_hi : lists_cap;
    bool piece[VPL];
#pragma unroll
    for (int w = 0; w < VPL; w++)
        piece[w] = w * LPR + r < pieces;
    for (int64_t u = u_lo + (int64_t)blockIdx.x * per_block + wv * G + g; u < u_hi;
         u += (int64_t)gridDim.x * per_block) {
        int lo = 0, hi = nf;  // feature of u inside [f0, f0 + nf)
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (feat_uoff[f0 + mid] <= u)
                lo = mid;
            else
                hi = mid;
        }
        const float4 *table = reinterpret_cast<const float4 *>(tabs.w[lo]);
        const int64_t j0 = u_offsets[u];
        int64_t j1 = u_offsets[u + 1];
        j1 = j1 < m_cap ? j1 : m_cap;
        float4 best[VPL];
        int4 arg[VPL];
#pragma unroll
        for (int w = 0; w < VPL; w++) {
            best[w] = make_float4(0.f, 0.f, 0.f, 0.f);
            arg[w] = make_int4(0, 0, 0, 0);
        }
        // pass 1: positions in ascending order, US rows in flight
        for (int64_t jb = j0; jb < j1; jb += US) {
            float4 v[US][VPL];
#pragma unroll
            for (int k = 0; k < US; k++) {
                const int64_t j = jb + k < j1 ? jb + k : j1 - 1;
                const int64_t id = u_values[j];
#pragma unroll
                for (int w = 0; w < VPL; w++)
                    if (piece[w])
                        v[k][w] = table[id * pieces + w * LPR + r];
            }
#pragma unroll
            for (int k = 0; k < US; k++)
                if (jb + k < j1) {
                    const int t = (int)(jb + k - j0);
#pragma unroll
                    for (int w = 0; w < VPL; w++)
                        if (piece[w]) {
                            const float4 x = v[k][w];
                            if (t == 0 || x.x > best[w].x) { best[w].x = x.x; arg[w].x = t; }
                            if (t == 0 || x.y > best[w].y) { best[w].y = x.y; arg[w].y = t; }
                            if (t == 0 || x.z > best[w].z) { best[w].z = x.z; arg[w].z = t; }
                            if (t == 0 || x.w > best[w].w) { best[w].w = x.w; arg[w].w = t; }
                        }
                }
        }
        // pass 2: one masked row per position
        float4 gu[VPL];
#pragma unroll
        for (int w = 0; w < VPL; w++)
            if (piece[w])
                gu[w] = g_u[u * pieces + w * LPR + r];
        for (int64_t j = j0; j < j1; j++) {
            const int t = (int)(j - j0);
#pragma unroll
            for (int w = 0; w < VPL; w++)
                if (piece[w]) {
                    float4 o;
                    o.x = arg[w].x == t ? gu[w].x : 0.f;
                    o.y = arg[w].y == t ? gu[w].y : 0.f;
                    o.z = arg[w].z == t ? gu[w].z : 0.f;
                    o.w = arg[w].w == t ? gu[w].w : 0.f;
                    {   // written once, read back once by the row-gradient sum: a streaming store
                        typedef float f32x4m __attribute__((ext_vector_type(4)));
                        const f32x4m ov = {o.x, o.y, o.z, o.w};
                        __builtin_nontemporal_store(ov, reinterpret_cast<f32x4m *>(emb) + j * pieces + w * LPR + r);
                    }
                }
        }
    }
}

__global__ void k_no_rows(int F, int64_t *feat_roff, int64_t *list_off)
{
    for (int f = threadIdx.x; f <= F; f += blockDim.x)
        feat_roff[f] = 0;
    if (threadIdx.x == 0) {
        list_off[0] = 0;
        list_off[1] = 0;
    }
}

int bits_for(uint64_t max_value)
{
    int b = 1;
    while (b < 64 && (max_value >> b) != 0)
        b++;
    return b;
}

// Buffers of one sort (the two sorts of a backward call run on two streams at the same time).
// ---------------------------------------------------------------- sequence path, step A
// g_emb[u_offsets[u] + t, :] = sum over the rows l (ascending) of unique list u of
// grad_out[offsets[l] + t, :].  The rows of u are ps[seg_start[u] .. seg_start[u+1]) (rows sorted by
// unique list; every list has at least one row, so segment number = list number).  A block owns
// LISTS consecutive unique lists and numbers their positions flat, so long and short lists load
// the threads alike.  The start offsets of up to 64 source rows per list are staged in LDS, so
// the inner loop is row loads only, eight in flight per thread (a thread = one 16-byte piece of
// one position); lists with more rows take further rounds that continue from the stored partial
// sum - the same additions in the same order.
template <int LISTS>
__global__ __launch_bounds__(256) void k_jagged_reduce(const float4 *__restrict__ grad_out,
                                                       const int64_t *__restrict__ offsets,
                                                       const uint32_t *__restrict__ ps,
                                                       const int64_t *__restrict__ seg_start,
                                                       const int64_t *__restrict__ n_seg,
                                                       const int64_t *__restrict__ u_offsets,
                                                       float4 *__restrict__ g_emb, int vecs,
                                                       int64_t n_rows, int64_t m_cap)
{
    static_assert(LISTS <= 64 && (LISTS & (LISTS - 1)) == 0, "one wave prepares the block's lists");
    constexpr int kRound = 64;  // source rows per list and round
    constexpr int kFly = 8;     // row loads in flight per thread
    __shared__ uint32_t rel_s[LISTS + 1];
    __shared__ int64_t pos_s[LISTS], seg_s[LISTS];
    __shared__ uint32_t cnt_s[LISTS];
    __shared__ uint32_t cmax_s;
    __shared__ int64_t off_s[LISTS][kRound];
    const int64_t U = *n_seg;
    const uint32_t rows_per_sweep = 256 / vecs;
    const uint32_t piece = threadIdx.x % vecs, sub = threadIdx.x / vecs;
    for (int64_t u0 = (int64_t)blockIdx.x * LISTS; u0 < U; u0 += (int64_t)gridDim.x * LISTS) {
        const uint32_t nl = U - u0 < LISTS ? (uint32_t)(U - u0) : (uint32_t)LISTS;
        __syncthreads();  // the previous lists are done with the shared arrays
        if (threadIdx.x < 64) {
            const uint32_t i = threadIdx.x;
            int64_t start = 0, s0 = 0;
            uint32_t len = 0, c = 0;
            if (i < nl) {
                start = u_offsets[u0 + i];
                len = (uint32_t)(u_offsets[u0 + i + 1] - start);
                s0 = seg_start[u0 + i];
                c = (uint32_t)(seg_start[u0 + i + 1] - s0);
            }
            uint32_t incl = len, cmax = c;
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                const uint32_t x = __shfl_up(incl, d);
                if (i >= (uint32_t)d)
                    incl += x;
                const uint32_t y = __shfl_xor(cmax, d);
                cmax = y > cmax ? y : cmax;
            }
            if (i < nl) {
                rel_s[i] = incl - len;
                pos_s[i] = start;
                seg_s[i] = s0;
                cnt_s[i] = c;
            }
            if (i == 63) {
                rel_s[nl] = incl;
                cmax_s = cmax;
            }
        }
        __syncthreads();
        const uint32_t total = rel_s[nl];
        const uint32_t cmax = cmax_s;
        for (uint32_t c0 = 0; c0 < cmax; c0 += kRound) {
            if (c0 > 0)
                __syncthreads();  // the previous round's offsets have been used
            for (uint32_t idx = threadIdx.x; idx < nl * kRound; idx += 256) {
                const uint32_t a = idx / kRound, i = idx % kRound;
                if (c0 + i < cnt_s[a])
                    off_s[a][i] = offsets[ps[seg_s[a] + c0 + i]];
            }
            __syncthreads();
            if (sub >= rows_per_sweep)
                continue;
            for (uint32_t r = sub; r < total; r += rows_per_sweep) {
                uint32_t a = 0;  // the last list with rel_s[a] <= r; r < rel_s[nl], so it is not empty
#pragma unroll
                for (uint32_t s = LISTS / 2; s >= 1; s >>= 1)
                    if (a + s < nl && rel_s[a + s] <= r)
                        a += s;
                const uint32_t c = cnt_s[a];
                if (c <= c0)
                    continue;  // this list has no rows left in this round
                const uint32_t n = c - c0 < (uint32_t)kRound ? c - c0 : (uint32_t)kRound;
                const int64_t t = r - rel_s[a];
                const int64_t j = pos_s[a] + t;
                if (j >= m_cap)
                    continue;
                float4 acc = c0 == 0 ? make_float4(0.f, 0.f, 0.f, 0.f) : g_emb[j * vecs + piece];
                for (uint32_t i = 0; i < n; i += kFly) {
                    float4 v[kFly];
#pragma unroll
                    for (int k = 0; k < kFly; k++) {
                        int64_t src = off_s[a][i + k < n ? i + k : n - 1] + t;
                        src = src < n_rows ? src : n_rows - 1;  // only a malformed IKJT gets here
                        {   // every gradient row is read once: a streaming load
                            typedef float f32x4g __attribute__((ext_vector_type(4)));
                            const f32x4g t4 = __builtin_nontemporal_load(
                                reinterpret_cast<const f32x4g *>(grad_out) + src * vecs + piece);
                            v[k] = make_float4(t4.x, t4.y, t4.z, t4.w);
                        }
                    }
#pragma unroll
                    for (int k = 0; k < kFly; k++)
                        if (i + k < n) {
                            acc.x += v[k].x;
                            acc.y += v[k].y;
                            acc.z += v[k].z;
                            acc.w += v[k].w;
                        }
                }
                g_emb[j * vecs + piece] = acc;
            }
        }
    }
}

struct SortSet {
    int64_t *n_dev;  // [0] number of pairs, [1] capacity-overflow flag
    void *k0, *k1;
    uint32_t *p0, *p1, *hist, *bsum;
};

struct BwdWs {
    SortSet a, b;
    // Segment numbering of step A (list_off, seg_start, long_count_a) and of step B (the _b arrays,
    // seg_feat, long_count and what follows): separate, the two are numbered on different streams.
    int64_t *list_off, *seg_start, *long_count_a;
    int64_t *list_off_b, *seg_start_b;
    int32_t *seg_feat, *lseg_t, *lseg_first, *lseg_n;
    int64_t *long_count, *item_start, *item_end;
    float *g_u, *partials;
    uint32_t *pos_list;  // weighted lookup: unique list of every position of u_values
    float *pay_w;        // weighted lookup: weight of every sorted entry of step B
    float *emb;          // max pooling: one masked gradient row per position of u_values [M, D]
    int long_seg;        // step B: segments with more entries are cut into chunks
    size_t bytes;
};

// Step B's lane groups walk a segment entry by entry, eight segments to a wave, so a wave lasts as
// long as its longest segment; segments with more entries than the context's cut
// (RECD_OPT_LONG_SEGMENT_CUT, default 32) go to the block-cooperative chunk passes on the side
// stream.  Measured at 2.2 M entries: 0.847 ms per step with 64, 0.838 with 32, 0.836 with 24 or 16;
// at 35 M entries (no deduplication), where the chunk passes are the larger part: 4.28 ms with 64,
// 4.55 with 32.
constexpr int kDefaultLongSeg = 32;

SortSet carve_sort(WsCarver &c, int64_t n, bool wide_keys)
{
    SortSet s;
    const int64_t ntiles = (n + kTile - 1) / kTile;
    const int64_t hist_n = (int64_t)kRadixMax * ntiles;
    s.n_dev = c.take<int64_t>(2);
    if (wide_keys) {
        s.k0 = c.take<uint64_t>(n);
        s.k1 = c.take<uint64_t>(n);
    } else {
        s.k0 = c.take<uint32_t>(n);
        s.k1 = c.take<uint32_t>(n);
    }
    s.p0 = c.take<uint32_t>(n);
    s.p1 = c.take<uint32_t>(n);
    s.hist = c.take<uint32_t>(hist_n);
    // block sums of the head-flag scan, and the digit totals of a sort pass
    s.bsum = c.take<uint32_t>((n + kScanTile - 1) / kScanTile + 1 + kRadixMax);
    return s;
}

BwdWs carve_bwd(char *base, int64_t n_lists, int64_t M_cap, int F, int D, int long_seg, bool with_emb = false)
{
    WsCarver c(base);
    BwdWs w;
    (void)c.take<char>(1024);  // the head of the workspace stays with the validation passes' flags
    const int64_t n_max = n_lists > M_cap ? n_lists : M_cap;
    int64_t u_cap = M_cap + F < n_lists ? M_cap + F : n_lists;
    w.a = carve_sort(c, n_lists, false);
    w.b = carve_sort(c, M_cap, true);
    w.list_off = c.take<int64_t>(2);
    w.long_count_a = c.take<int64_t>(2);
    w.seg_start = c.take<int64_t>(n_lists + 1);
    w.list_off_b = c.take<int64_t>(2);
    w.seg_start_b = c.take<int64_t>(M_cap + 1);
    w.seg_feat = c.take<int32_t>(M_cap);
    // cut segments (more than long_seg entries): at most n/(long_seg+1) of them, in at most
    // n/256 + n/(long_seg+1) chunks
    w.long_seg = long_seg;
    const int64_t lseg_cap = n_max / (w.long_seg + 1) + 16, item_cap = n_max / 256 + n_max / (w.long_seg + 1) + 16;
    w.lseg_t = c.take<int32_t>(lseg_cap);
    w.lseg_first = c.take<int32_t>(lseg_cap);
    w.lseg_n = c.take<int32_t>(lseg_cap);
    w.long_count = c.take<int64_t>(2);
    w.item_start = c.take<int64_t>(item_cap);
    w.item_end = c.take<int64_t>(item_cap);
    w.partials = c.take<float>((size_t)item_cap * D);
    w.g_u = c.take<float>((size_t)u_cap * D);
    w.pos_list = c.take<uint32_t>(M_cap);
    w.pay_w = c.take<float>(M_cap);
    w.emb = with_emb ? c.take<float>((size_t)M_cap * D) : nullptr;
    w.bytes = c.off;
    return w;
}

// Segments of equal keys in the sorted keys ks: seg_start, list_off = {0, R} and, for (feature, row)
// keys, the row ids, the feature of every segment and feat_roff.
// (row_bits < 0: step A's arrays; row_bits >= 0: step B's.)
struct SegBufs {
    int64_t *seg_start, *list_off, *long_count;
};

SegBufs seg_bufs(const BwdWs &w, int row_bits)
{
    return row_bits < 0 ? SegBufs{w.seg_start, w.list_off, w.long_count_a}
                        : SegBufs{w.seg_start_b, w.list_off_b, w.long_count};
}

template <typename KeyT>
recd_status number_segments(recd_ctx *ctx, hipStream_t st, const BwdWs &w, const SortSet &set, const KeyT *ks,
                            int64_t n_cap, int row_bits, int F, int64_t *touched_rows, int64_t *feat_roff)
{
    const SegBufs sb = seg_bufs(w, row_bits);
    const unsigned tiles = (unsigned)((n_cap + kScanTile - 1) / kScanTile > 0 ? (n_cap + kScanTile - 1) / kScanTile : 1);
    hipLaunchKernelGGL((k_head_count<KeyT>), dim3(tiles), dim3(256), 0, st, ks, set.n_dev, set.bsum,
                       sb.long_count);
    hipLaunchKernelGGL(k_scan_small, dim3(1), dim3(1024), 0, st, set.bsum, (int64_t)tiles);
    hipLaunchKernelGGL((k_segments<KeyT>), dim3(tiles), dim3(256), 0, st, ks, set.n_dev, set.bsum,
                       sb.seg_start, sb.list_off, row_bits, F, touched_rows, feat_roff, w.seg_feat);
    RECD_HIP(ctx, hipGetLastError());
    return RECD_OK;
}

// What the row-gradient kernels of step B need to know about its segments.
RowSumParams row_params(const BwdWs &w, const uint32_t *ps, const float *pay_w, const void *table, int D, void *out)
{
    RowSumParams rp;
    rp.table = static_cast<const float *>(table);
    rp.pay = ps;
    rp.pay_w = pay_w;
    rp.seg_start = w.seg_start_b;
    rp.n_seg = w.list_off_b + 1;
    rp.out = static_cast<float *>(out);
    rp.D = D;
    rp.pieces = D / 4;
    rp.long_count = w.long_count;
    rp.lseg_t = w.lseg_t;
    rp.lseg_first = w.lseg_first;
    rp.lseg_n = w.lseg_n;
    rp.item_start = w.item_start;
    rp.item_end = w.item_end;
    rp.partials = w.partials;
    rp.long_seg = w.long_seg;
    return rp;
}

// Step B's segments need the sorted keys only, not the result of step A: numbered, and the long
// ones cut into chunks, on the stream the sort ran on.
template <typename KeyT>
recd_status prepare_rows(recd_ctx *ctx, hipStream_t st, const BwdWs &w, const SortSet &set, const KeyT *ks,
                         int64_t n_cap, int64_t seg_bound, int row_bits, int F, int64_t *touched_rows,
                         int64_t *feat_roff, hipEvent_t numbered = nullptr)
{
    RECD_TRY(number_segments<KeyT>(ctx, st, w, set, ks, n_cap, row_bits, F, touched_rows, feat_roff));
    // the sum of the short segments needs nothing of what follows: whoever waits for `numbered`
    // instead of the end of this stream's work starts it one kernel earlier
    if (numbered)
        RECD_HIP(ctx, hipEventRecord(numbered, st));
    const RowSumParams rp = row_params(w, nullptr, nullptr, nullptr, 4, nullptr);
    int64_t fblk = (seg_bound + 255) / 256;
    if (fblk > (int64_t)ctx->num_cu * 8)
        fblk = (int64_t)ctx->num_cu * 8;
    hipLaunchKernelGGL(k_find_long, dim3((unsigned)(fblk < 1 ? 1 : fblk)), dim3(256), 0, st, rp);
    RECD_HIP(ctx, hipGetLastError());
    return RECD_OK;
}

// Step A: segments of equal keys in the sorted pairs (ks, ps) of `set`, then the sum of every
// segment's rows (the block-cooperative gather-sum kernel handles any segment length).
recd_status segment_and_sum_lists(recd_ctx *ctx, const BwdWs &w, const SortSet &set, const uint32_t *ks,
                                  const uint32_t *ps, int64_t n_cap, int64_t seg_bound, int F,
                                  const void *table, int D, void *out, const int64_t *div_off)
{
    RECD_TRY(number_segments<uint32_t>(ctx, ctx->stream, w, set, ks, n_cap, -1, F, nullptr, nullptr));
    SegSumArgs a{};
    a.site = RECD_SITE_GRAD_STREAM;  // every grad_out row is read exactly once
    a.F = 1;
    a.D = D;
    a.table_dt = RECD_F32;
    a.out_dt = RECD_F32;
    a.tables.p[0] = table;
    a.values = ps;
    a.values_are_i32 = 1;
    a.offsets = w.seg_start;
    a.list_off = w.list_off;
    a.lists_bound = seg_bound;
    a.flat = 1;
    a.out = out;
    a.div_off = div_off;
    return recd_launch_segsum(ctx, a);
}

// Step B after prepare_rows: short segments (at most long_seg entries) by one lane group each, the cut
// ones by the block-cooperative kernel on the side stream next to them; optimizer fused.
recd_status sum_rows(recd_ctx *ctx, const BwdWs &w, const uint32_t *ps, int64_t n_cap, int64_t seg_bound,
                     const void *table, int D, void *out, int64_t *touched_rows, const OptAdagrad *opt,
                     const float *pay_w)
{
    hipStream_t st = ctx->stream;
    const RowSumParams rp = row_params(w, ps, pay_w, table, D, out);
    OptAdagrad o;
    if (opt)
        o = *opt;
    else
        o.n_feat = 0;
    o.touched_rows = touched_rows;
    o.seg_feat = w.seg_feat;
    const int P = rp.pieces;
    const int lpr = P <= 16 ? 4 : (P <= 32 ? 8 : (P <= 64 ? 16 : (P <= 128 ? 32 : 64)));
    const int per_block = 4 * (64 / lpr);
    int64_t nblk = (seg_bound + per_block - 1) / per_block;
    const int64_t cap = (int64_t)ctx->num_cu * 64;
    if (nblk > cap)
        nblk = cap;
    nblk = (nblk + 7) / 8 * 8;  // the kernel deals its blocks to 8 XCDs
    if (nblk < 8)
        nblk = 8;
    const dim3 block(256);
    auto launch_rows = [&](auto fin, auto wt, unsigned nb, hipStream_t stream) {
        constexpr bool FIN = decltype(fin)::value, WT = decltype(wt)::value;
        const dim3 grid(nb);
        switch (lpr) {
        case 4: hipLaunchKernelGGL((k_segsum_rows<4, FIN, WT>), grid, block, 0, stream, rp, o); break;
        case 8: hipLaunchKernelGGL((k_segsum_rows<8, FIN, WT>), grid, block, 0, stream, rp, o); break;
        case 16: hipLaunchKernelGGL((k_segsum_rows<16, FIN, WT>), grid, block, 0, stream, rp, o); break;
        case 32: hipLaunchKernelGGL((k_segsum_rows<32, FIN, WT>), grid, block, 0, stream, rp, o); break;
        default: hipLaunchKernelGGL((k_segsum_rows<64, FIN, WT>), grid, block, 0, stream, rp, o); break;
        }
    };
    // 1. on the side stream: partial sum of every chunk of the cut segments (block-cooperative
    //    gather-sum, one block per chunk), then the chunk partials added in chunk order and the same
    //    update / store as for short segments.  Long and short segments name different rows.
    hipStream_t side = ctx->side_stream;
    RECD_HIP(ctx, hipEventRecord(ctx->ev_fork, st));
    RECD_HIP(ctx, hipStreamWaitEvent(side, ctx->ev_fork, 0));
    SegSumArgs c{};
    c.site = RECD_SITE_GRAD_LISTS;
    c.F = 1;
    c.D = D;
    c.table_dt = RECD_F32;
    c.out_dt = RECD_F32;
    c.tables.p[0] = table;
    c.values = ps;
    c.values_are_i32 = 1;
    c.flat = 1;
    c.offsets = w.item_start;
    c.ends = w.item_end;
    c.count_dev = w.long_count + 1;
    c.lists_bound = n_cap / 256 + n_cap / (w.long_seg + 1) + 1;
    c.out = w.partials;
    c.stream = side;
    if (pay_w) {  // the chunk partials carry the weights; adding the partials does not
        c.mode = 3;
        c.weights = pay_w;
    }
    RECD_TRY(recd_launch_segsum(ctx, c));
    launch_rows(std::true_type(), std::false_type(), (unsigned)((ctx->num_cu + 7) / 8 * 8), side);
    RECD_HIP(ctx, hipGetLastError());
    RECD_HIP(ctx, hipEventRecord(ctx->ev_join, side));
    // 2. short segments summed and updated
    recd_time_begin(ctx, RECD_T_GRAD_ROWS, st);
    if (pay_w)
        launch_rows(std::false_type(), std::true_type(), (unsigned)nblk, st);
    else
        launch_rows(std::false_type(), std::false_type(), (unsigned)nblk, st);
    recd_time_end(ctx, RECD_T_GRAD_ROWS, st);
    RECD_HIP(ctx, hipGetLastError());
    RECD_HIP(ctx, hipStreamWaitEvent(st, ctx->ev_join, 0));
    return RECD_OK;
}

} // namespace

size_t recd_backward_workspace(int F, int64_t B, int64_t M_cap, int D)
{
    return carve_bwd(nullptr, (int64_t)F * B, M_cap, F, D, kDefaultLongSeg).bytes;
}

// The fused update reads and writes a table row (and its accumulator) once per (feature, row)
// segment, from different lane groups and two streams at the same time: two features must not name
// the same table or the same accumulator array.
static recd_status check_distinct_tables(recd_ctx *ctx, int F, void *const *tables, float *const *state)
{
    if (!tables)
        return RECD_OK;
    std::vector<const void *> t(tables, tables + F), m(state, state + F);
    std::sort(t.begin(), t.end());
    std::sort(m.begin(), m.end());
    for (int f = 1; f < F; f++)
        if (t[f] == t[f - 1] || m[f] == m[f - 1])
            return recd_fail(ctx, RECD_EINVAL,
                             "tables[] and adagrad_state[] must each hold pairwise distinct pointers "
                             "(one table per feature)");
    return RECD_OK;
}

// Backward of the pooled path (seq = false: grad_out is [F,B,D]) and of the sequence path (seq =
// true: grad_out is [N,D], one row per KJT position; kjt_offsets, N and grad_emb are used).
// mean: the pooled path averaged, so g_u[u] is divided by the length of unique list u (every
// segment of step A is one unique list, in order: each has at least one row).
// u_weights: the pooled path's lookup was the weighted sum: position j hands u_weights[j] * g_u on.
// max_tables: the pooled path's lookup was the maximum over these fp32 tables: element d of g_u
// goes to the position that won it (k_max_route), then step B adds per-position rows.
static recd_status backward_common(recd_ctx *ctx, bool seq, bool mean, int F, int64_t B, int64_t N, int D,
                                   const float *grad_out, const int64_t *kjt_offsets,
                                   const int32_t *inverse, const int64_t *feat_uoff,
                                   const int64_t *u_values, const float *u_weights,
                                   const void *const *max_tables, const int64_t *u_offsets,
                                   const int64_t *rows, int64_t U_cap, int64_t M_cap, float *grad_emb,
                                   int64_t *touched_rows, int64_t *feat_roff, float *grad_rows,
                                   void *const *tables, float *const *adagrad_state, float lr,
                                   float eps, int64_t *host_R)
{
    if (!ctx)
        return RECD_EINVAL;
    if (seq && (N < 0 || N >= (int64_t)1 << 31 || !kjt_offsets || (M_cap > 0 && !grad_emb)))
        return recd_fail(ctx, RECD_EINVAL, "sequence backward: bad N or null offsets / grad_emb");
    if (F < 0 || F > RECD_MAX_FEATURES || B < 0 || M_cap < 0 || U_cap < 0)
        return recd_fail(ctx, RECD_EINVAL, "bad sizes");
    if (U_cap > (int64_t)F * B)
        U_cap = (int64_t)F * B;
    if (D <= 0 || D % 4 != 0 || (size_t)D * 4 > RECD_MAX_ROW_BYTES ||
        (D * 4 / 16 > 64 && D * 4 / 16 != 128 && D * 4 / 16 != 256))
        return recd_fail(ctx, RECD_EINVAL, "unsupported D=%d", D);
    const int64_t n_lists = (int64_t)F * B;
    if (n_lists >= (int64_t)1 << 31 || M_cap >= (int64_t)1 << 31)
        return recd_fail(ctx, RECD_EINVAL, "F*B and M_cap must stay below 2^31");
    if (!feat_roff || !feat_uoff || !u_offsets || (F > 0 && !rows))
        return recd_fail(ctx, RECD_EINVAL, "null pointer argument");
    if (n_lists > 0 && ((!grad_out && !(seq && N == 0)) || !inverse))
        return recd_fail(ctx, RECD_EINVAL, "null pointer argument");
    if (M_cap > 0 && (!u_values || !touched_rows))
        return recd_fail(ctx, RECD_EINVAL, "null pointer argument");
    if (M_cap > 0 && !grad_rows && !(tables && F <= RECD_F_PER_LAUNCH))
        return recd_fail(ctx, RECD_EINVAL,
                         "grad_rows may be NULL only with the optimizer and at most %d features",
                         RECD_F_PER_LAUNCH);
    if ((tables == nullptr) != (adagrad_state == nullptr))
        return recd_fail(ctx, RECD_EINVAL, "tables and adagrad_state must be given together");
    RECD_TRY(recd_check_rows(ctx, F, rows));
    int64_t max_rows = 1;
    for (int f = 0; f < F; f++) {
        if (rows[f] <= 0)
            return recd_fail(ctx, RECD_EINVAL, "rows[%d] <= 0", f);
        if (rows[f] > max_rows)
            max_rows = rows[f];
        if (tables && (!tables[f] || !adagrad_state[f]))
            return recd_fail(ctx, RECD_EINVAL, "tables[%d] or adagrad_state[%d] is null", f, f);
    }
    RECD_TRY(check_distinct_tables(ctx, F, tables, adagrad_state));
    RECD_HIP(ctx, hipSetDevice(ctx->device));
    if (ctx->validate && n_lists > 0)
        RECD_TRY(recd_validate_inverse(ctx, F, B, feat_uoff, inverse));
    const bool maxmode = max_tables != nullptr;
    ctx->plan.valid = false;  // this call reuses the workspace a plan would live in
    RECD_TRY(recd_reserve(ctx, carve_bwd(nullptr, n_lists, M_cap, F, D, ctx->long_seg_cut, maxmode).bytes));
    const BwdWs w = carve_bwd(ctx->ws, n_lists, M_cap, F, D, ctx->long_seg_cut, maxmode);
    hipStream_t st = ctx->stream;

    if (n_lists == 0 || M_cap == 0) {
        // no id anywhere: no row is touched
        hipLaunchKernelGGL(k_no_rows, dim3(1), dim3(64), 0, st, F, feat_roff, w.list_off);
        RECD_HIP(ctx, hipGetLastError());
        if (host_R) {
            RECD_HIP(ctx, hipStreamSynchronize(st));
            host_R[0] = 0;
        }
        return RECD_OK;
    }

    // Row-wise Adagrad runs inside the row-gradient segment sum while the sum is still in
    // registers; with more features than one launch carries it runs as a kernel of its own.
    const bool fused = tables != nullptr && F <= RECD_F_PER_LAUNCH;
    OptAdagrad oa;
    oa.n_feat = 0;
    if (fused) {
        oa.n_feat = F;
        for (int f = 0; f < F; f++) {
            oa.w[f] = static_cast<float *>(tables[f]);
            oa.m[f] = adagrad_state[f];
        }
        oa.lr = lr;
        oa.eps = eps;
    }
    const int row_bits = bits_for((uint64_t)(max_rows - 1));
    const int bits_b = row_bits + bits_for((uint64_t)(F > 1 ? F - 1 : 1));
    const int bits_a = bits_for((uint64_t)(U_cap > 1 ? U_cap - 1 : 1));
    const bool wide = bits_b > 32;

    // The sort of step B needs nothing from step A: it runs on the side stream meanwhile, forked from
    // the point before step A.  Step A's launches are issued first: its chain is the longer one, and
    // while the host issues the side stream's fifteen short launches the main stream would idle.
    hipStream_t side = ctx->side_stream;
    RECD_HIP(ctx, hipEventRecord(ctx->ev_fork, st));
    // ---- step A: group rows (f,b) by unique list, sum grad_out rows into g_u --------------------
    {
        uint32_t *k0 = static_cast<uint32_t *>(w.a.k0), *k1 = static_cast<uint32_t *>(w.a.k1), *ks, *ps;
        hipLaunchKernelGGL(k_keys_rows, dim3((unsigned)((n_lists + 255) / 256)), dim3(256), 0, st,
                           inverse, feat_uoff, B, n_lists, k0, w.a.p0, w.a.n_dev);
        RECD_TRY(radix_sort_pairs<uint32_t>(ctx, st, k0, w.a.p0, k1, w.a.p1, w.a.n_dev, n_lists, bits_a,
                                            w.a.hist, w.a.bsum, &ks, &ps));
        if (!seq) {
            RECD_TRY(segment_and_sum_lists(ctx, w, w.a, ks, ps, n_lists, U_cap, F, grad_out, D, w.g_u,
                                           mean ? u_offsets : nullptr));
        } else {
            RECD_TRY(number_segments<uint32_t>(ctx, st, w, w.a, ks, n_lists, -1, F, nullptr, nullptr));
            // lists per block: about 128 positions
            const double avg = (double)M_cap / (double)(U_cap > 0 ? U_cap : 1);
            int lists = 1;
            while (lists < 64 && 2.0 * lists * avg <= 192.0)
                lists *= 2;
            int64_t blocks = (U_cap + lists - 1) / lists;
            if (blocks > (int64_t)ctx->num_cu * 64)
                blocks = (int64_t)ctx->num_cu * 64;
            if (blocks < 1)
                blocks = 1;
#define RECD_JR(L)                                                                                    \
    hipLaunchKernelGGL((k_jagged_reduce<L>), dim3((unsigned)blocks), dim3(256), 0, st,                 \
                       reinterpret_cast<const float4 *>(grad_out), kjt_offsets, ps, w.seg_start,       \
                       w.list_off + 1, u_offsets, reinterpret_cast<float4 *>(grad_emb), D / 4, N, M_cap)
            switch (lists) {
            case 1: RECD_JR(1); break;
            case 2: RECD_JR(2); break;
            case 4: RECD_JR(4); break;
            case 8: RECD_JR(8); break;
            case 16: RECD_JR(16); break;
            case 32: RECD_JR(32); break;
            default: RECD_JR(64); break;
            }
#undef RECD_JR
            RECD_HIP(ctx, hipGetLastError());
        }
    }
    if (maxmode) {
        const int P = D / 4;  // 16-byte pieces of a row: up to 64 one per lane, else 128 or 256
        const int lpr = P <= 4 ? 4 : (P <= 8 ? 8 : (P <= 16 ? 16 : (P <= 32 ? 32 : 64)));
        const int vpl = P <= 64 ? 1 : (P == 128 ? 2 : 4);
        const int per_block = 4 * (64 / lpr);
        for (int f0 = 0; f0 < F; f0 += RECD_F_PER_LAUNCH) {
            MaxTables mt;
            const int nf = F - f0 < RECD_F_PER_LAUNCH ? F - f0 : RECD_F_PER_LAUNCH;
            for (int f = 0; f < nf; f++)
                mt.w[f] = static_cast<const float *>(max_tables[f0 + f]);
            int64_t nblk = (U_cap + per_block - 1) / per_block;
            if (nblk > (int64_t)ctx->num_cu * 64)
                nblk = (int64_t)ctx->num_cu * 64;
            const dim3 grid((unsigned)(nblk < 1 ? 1 : nblk)), block(256);
#define RECD_MR(L, V)                                                                                    \
    hipLaunchKernelGGL((k_max_route<L, V>), grid, block, 0, st, u_values, u_offsets, feat_uoff, f0, nf, mt,  \
                       reinterpret_cast<const float4 *>(w.g_u), reinterpret_cast<float4 *>(w.emb), P, U_cap, \
                       M_cap)
            if (vpl == 4) RECD_MR(64, 4);
            else if (vpl == 2) RECD_MR(64, 2);
            else if (lpr == 4) RECD_MR(4, 1);
            else if (lpr == 8) RECD_MR(8, 1);
            else if (lpr == 16) RECD_MR(16, 1);
            else if (lpr == 32) RECD_MR(32, 1);
            else RECD_MR(64, 1);
#undef RECD_MR
        }
        RECD_HIP(ctx, hipGetLastError());
    }
    // ---- step B's keys, sort and segment numbering on the side stream ------------------------------
    RECD_HIP(ctx, hipStreamWaitEvent(side, ctx->ev_fork, 0));
    void *ks_b = nullptr;
    uint32_t *ps_b = nullptr;
    {
        constexpr int SG = 16;
        const unsigned kb = keys_ids_blocks(U_cap, n_lists, SG, 256);
        if (!wide) {
            uint32_t *k0 = static_cast<uint32_t *>(w.b.k0), *k1 = static_cast<uint32_t *>(w.b.k1), *ks;
            hipLaunchKernelGGL((k_keys_ids<uint32_t, SG>), dim3(kb), dim3(256), 0, side, u_values,
                               u_offsets, feat_uoff, F, row_bits, n_lists, M_cap, k0, w.b.p0, w.b.n_dev,
                               (seq || u_weights || maxmode) ? 1 : 0, u_weights ? w.pos_list : nullptr);
            RECD_TRY(radix_sort_pairs<uint32_t>(ctx, side, k0, w.b.p0, k1, w.b.p1, w.b.n_dev, M_cap, bits_b,
                                                w.b.hist, w.b.bsum, &ks, &ps_b));
            ks_b = ks;
        } else {
            uint64_t *k0 = static_cast<uint64_t *>(w.b.k0), *k1 = static_cast<uint64_t *>(w.b.k1), *ks;
            hipLaunchKernelGGL((k_keys_ids<uint64_t, SG>), dim3(kb), dim3(256), 0, side, u_values,
                               u_offsets, feat_uoff, F, row_bits, n_lists, M_cap, k0, w.b.p0, w.b.n_dev,
                               (seq || u_weights || maxmode) ? 1 : 0, u_weights ? w.pos_list : nullptr);
            RECD_TRY(radix_sort_pairs<uint64_t>(ctx, side, k0, w.b.p0, k1, w.b.p1, w.b.n_dev, M_cap, bits_b,
                                                w.b.hist, w.b.bsum, &ks, &ps_b));
            ks_b = ks;
        }
        if (u_weights) {
            int64_t wb = (M_cap + 255) / 256;
            if (wb > (int64_t)ctx->num_cu * 16)
                wb = (int64_t)ctx->num_cu * 16;
            hipLaunchKernelGGL(k_weight_payload, dim3((unsigned)(wb < 1 ? 1 : wb)), dim3(256), 0, side, ps_b,
                               w.pos_list, u_weights, w.b.n_dev, w.pay_w);
        }
        RECD_HIP(ctx, hipGetLastError());
        // the segments of step B (row ids, per-feature counts, chunks of the long ones) as well
        if (!wide)
            RECD_TRY(prepare_rows<uint32_t>(ctx, side, w, w.b, static_cast<const uint32_t *>(ks_b), M_cap, M_cap,
                                            row_bits, F, touched_rows, feat_roff));
        else
            RECD_TRY(prepare_rows<uint64_t>(ctx, side, w, w.b, static_cast<const uint64_t *>(ks_b), M_cap, M_cap,
                                            row_bits, F, touched_rows, feat_roff));
        RECD_HIP(ctx, hipEventRecord(ctx->ev_join, side));
    }
    const float *b_table = seq ? grad_emb : (maxmode ? w.emb : w.g_u);
    // ---- step B: group unique-id positions by (feature, row), sum g_u rows into grad_rows --------
    RECD_HIP(ctx, hipStreamWaitEvent(st, ctx->ev_join, 0));
    RECD_TRY(sum_rows(ctx, w, ps_b, M_cap, M_cap, b_table, D, grad_rows, touched_rows, fused ? &oa : nullptr,
                      u_weights ? w.pay_w : nullptr));
    // ---- optimizer -------------------------------------------------------------------------------
    if (tables && !fused) {
        for (int f0 = 0; f0 < F; f0 += RECD_F_PER_LAUNCH) {
            OptPtrs ptrs;
            const int nf = F - f0 < RECD_F_PER_LAUNCH ? F - f0 : RECD_F_PER_LAUNCH;
            for (int f = 0; f < nf; f++) {
                ptrs.w[f] = static_cast<float *>(tables[f0 + f]);
                ptrs.m[f] = adagrad_state[f0 + f];
            }
            hipLaunchKernelGGL(k_adagrad, dim3(ctx->num_cu * 8), dim3(256), 0, st, grad_rows,
                               touched_rows, feat_roff, f0, nf, D, ptrs, lr, eps);
        }
        RECD_HIP(ctx, hipGetLastError());
    }
    if (host_R) {
        RECD_HIP(ctx, hipMemcpyAsync(ctx->host_pinned, w.list_off_b + 1, sizeof(int64_t),
                                     hipMemcpyDeviceToHost, st));
        RECD_HIP(ctx, hipMemcpyAsync(ctx->host_pinned + 1, w.b.n_dev + 1, sizeof(int64_t),
                                     hipMemcpyDeviceToHost, st));
        RECD_HIP(ctx, hipStreamSynchronize(st));
        host_R[0] = ctx->host_pinned[0];
        if (ctx->host_pinned[1])
            return recd_fail(ctx, RECD_ECAPACITY, "M_cap=%lld is smaller than M", (long long)M_cap);
    }
    return RECD_OK;
}

// ---------------------------------------------------------------- planned backward
// The backward's grouping work (keys, sorts, segment numbering of both steps) depends on the IKJT
// only, not on the gradient.  recd_backward_plan runs it on the two side streams, starting where the
// IKJT's build ended, so that it overlaps the forward calls (which are bandwidth-bound, while the
// plan is a chain of short latency-bound kernels); recd_backward_apply then waits for the plan on the
// main stream and runs the two segment sums with the fused update.  Same kernels, same inputs, same
// results as the one-call form.
// run_index: null, or the batch's run index (then step A's grouping sorts the runs, at most
// runs_cap of them, instead of all F*B rows)
static recd_status plan_common(recd_ctx *ctx, int F, int64_t B, int D, const int32_t *inverse,
                               const int64_t *feat_uoff, const int64_t *u_values, const int64_t *u_offsets,
                               const int64_t *rows, int64_t U_cap, int64_t M_cap, const int64_t *run_index,
                               int64_t runs_cap, int64_t *touched_rows, int64_t *feat_roff)
{
    if (!ctx)
        return RECD_EINVAL;
    ctx->plan.valid = false;
    if (run_index && runs_cap < 0)
        return recd_fail(ctx, RECD_EINVAL, "runs_cap < 0");
    if (F < 0 || F > RECD_MAX_FEATURES || B < 0 || M_cap < 0 || U_cap < 0)
        return recd_fail(ctx, RECD_EINVAL, "bad sizes");
    if (U_cap > (int64_t)F * B)
        U_cap = (int64_t)F * B;
    if (D <= 0 || D % 4 != 0 || (size_t)D * 4 > RECD_MAX_ROW_BYTES ||
        (D * 4 / 16 > 64 && D * 4 / 16 != 128 && D * 4 / 16 != 256))
        return recd_fail(ctx, RECD_EINVAL, "unsupported D=%d", D);
    const int64_t n_lists = (int64_t)F * B;
    if (n_lists >= (int64_t)1 << 31 || M_cap >= (int64_t)1 << 31)
        return recd_fail(ctx, RECD_EINVAL, "F*B and M_cap must stay below 2^31");
    if (!feat_roff || !feat_uoff || !u_offsets || (F > 0 && !rows) || (n_lists > 0 && !inverse) ||
        (M_cap > 0 && (!u_values || !touched_rows)))
        return recd_fail(ctx, RECD_EINVAL, "null pointer argument");
    RECD_TRY(recd_check_rows(ctx, F, rows));
    int64_t max_rows = 1;
    for (int f = 0; f < F; f++) {
        if (rows[f] <= 0)
            return recd_fail(ctx, RECD_EINVAL, "rows[%d] <= 0", f);
        if (rows[f] > max_rows)
            max_rows = rows[f];
    }
    RECD_HIP(ctx, hipSetDevice(ctx->device));
    if (ctx->validate && n_lists > 0)
        RECD_TRY(recd_validate_inverse(ctx, F, B, feat_uoff, inverse));
    // the side streams may start at the end of the build only if nothing on the stream has used the
    // workspace since (this call's own reservation does not count)
    const bool ws_idle_since_build = !ctx->ws_used_since_build;
    RECD_TRY(recd_reserve(ctx, carve_bwd(nullptr, n_lists, M_cap, F, D, ctx->long_seg_cut).bytes));
    const BwdWs w = carve_bwd(ctx->ws, n_lists, M_cap, F, D, ctx->long_seg_cut);
    recd_ctx::BackwardPlan &pl = ctx->plan;
    pl.F = F;
    pl.B = B;
    pl.D = D;
    pl.U_cap = U_cap;
    pl.M_cap = M_cap;
    pl.u_offsets = u_offsets;
    pl.touched_rows = touched_rows;
    pl.feat_roff = feat_roff;
    pl.ws = ctx->ws;
    pl.empty = n_lists == 0 || M_cap == 0;
    hipStream_t st = ctx->stream, sa = ctx->side_stream2, sb = ctx->side_stream;
    // Where the side streams may start: at the end of the build that produced this IKJT if it is the
    // context's most recent one, else at the main stream's current position.
    hipEvent_t from = ctx->ev_fork;
    if (ctx->build_valid && ws_idle_since_build && ctx->built_inverse == inverse &&
        ctx->built_u_values == u_values && n_lists > 0)
        from = ctx->ev_built;
    else
        RECD_HIP(ctx, hipEventRecord(ctx->ev_fork, st));
    RECD_HIP(ctx, hipStreamWaitEvent(sa, from, 0));
    RECD_HIP(ctx, hipStreamWaitEvent(sb, from, 0));
    if (!pl.empty) {
        const int row_bits = bits_for((uint64_t)(max_rows - 1));
        const int bits_b = row_bits + bits_for((uint64_t)(F > 1 ? F - 1 : 1));
        const int bits_a = bits_for((uint64_t)(U_cap > 1 ? U_cap - 1 : 1));
        pl.row_bits = row_bits;
        pl.wide = bits_b > 32;
        auto chain_a = [&]() -> recd_status {
        // step A's grouping on the second side stream
        if (run_index) {
            // the runs sorted by unique list, then written out as the rows they stand for
            if (runs_cap > n_lists || runs_cap == 0)
                runs_cap = n_lists;
            uint32_t *k0 = static_cast<uint32_t *>(w.a.k0), *k1 = static_cast<uint32_t *>(w.a.k1), *ks, *ps;
            hipLaunchKernelGGL(k_run_keys, dim3((unsigned)((runs_cap + 255) / 256)), dim3(256), 0, sa, run_index,
                               runs_cap, k0, w.a.p0, w.a.n_dev);
            RECD_TRY(radix_sort_pairs<uint32_t>(ctx, sa, k0, w.a.p0, k1, w.a.p1, w.a.n_dev, runs_cap, bits_a,
                                                w.a.hist, w.a.bsum, &ks, &ps));
            const unsigned tiles = (unsigned)((runs_cap + kScanTile - 1) / kScanTile);
            uint32_t *rows_out = ps == w.a.p0 ? w.a.p1 : w.a.p0;
            hipLaunchKernelGGL((k_run_rows<false>), dim3(tiles), dim3(256), 0, sa, ks, ps, run_index, w.a.n_dev,
                               w.a.bsum, w.a.hist, w.seg_start, w.list_off, rows_out, w.long_count_a);
            hipLaunchKernelGGL(k_scan_small, dim3(1), dim3(1024), 0, sa, w.a.bsum, (int64_t)tiles);
            hipLaunchKernelGGL(k_scan_small, dim3(1), dim3(1024), 0, sa, w.a.hist, (int64_t)tiles);
            hipLaunchKernelGGL((k_run_rows<true>), dim3(tiles), dim3(256), 0, sa, ks, ps, run_index, w.a.n_dev,
                               w.a.bsum, w.a.hist, w.seg_start, w.list_off, rows_out, w.long_count_a);
            RECD_HIP(ctx, hipGetLastError());
            pl.ks_a = ks;
            pl.ps_a = rows_out;
        } else {
            uint32_t *k0 = static_cast<uint32_t *>(w.a.k0), *k1 = static_cast<uint32_t *>(w.a.k1), *ks, *ps;
            hipLaunchKernelGGL(k_keys_rows, dim3((unsigned)((n_lists + 255) / 256)),
                               dim3(256), 0, sa, inverse,
                               feat_uoff, B, n_lists, k0, w.a.p0, w.a.n_dev);
            RECD_TRY(radix_sort_pairs<uint32_t>(ctx, sa, k0, w.a.p0, k1, w.a.p1, w.a.n_dev, n_lists, bits_a,
                                                w.a.hist, w.a.bsum, &ks, &ps));
            RECD_TRY(number_segments<uint32_t>(ctx, sa, w, w.a, ks, n_lists, -1, F, nullptr, nullptr));
            pl.ks_a = ks;
            pl.ps_a = ps;
        }
        return RECD_OK;
        };
        auto chain_b = [&]() -> recd_status {
        // step B's grouping on the first
        {
            constexpr int SG = 16;
            const unsigned kb = keys_ids_blocks(U_cap, n_lists, SG, 256);
            if (!pl.wide) {
                uint32_t *k0 = static_cast<uint32_t *>(w.b.k0), *k1 = static_cast<uint32_t *>(w.b.k1), *ks, *ps;
                hipLaunchKernelGGL((k_keys_ids<uint32_t, SG>), dim3(kb), dim3(256), 0, sb, u_values, u_offsets,
                                   feat_uoff, F, row_bits, n_lists, M_cap, k0, w.b.p0, w.b.n_dev, 0, nullptr);
                RECD_TRY(radix_sort_pairs<uint32_t>(ctx, sb, k0, w.b.p0, k1, w.b.p1, w.b.n_dev, M_cap, bits_b,
                                                    w.b.hist, w.b.bsum, &ks, &ps));
                RECD_TRY(prepare_rows<uint32_t>(ctx, sb, w, w.b, ks, M_cap, M_cap, row_bits, F, touched_rows,
                                                feat_roff, ctx->ev_plan_rows));
                pl.ps_b = ps;
            } else {
                uint64_t *k0 = static_cast<uint64_t *>(w.b.k0), *k1 = static_cast<uint64_t *>(w.b.k1), *ks;
                uint32_t *ps;
                hipLaunchKernelGGL((k_keys_ids<uint64_t, SG>), dim3(kb), dim3(256), 0, sb, u_values, u_offsets,
                                   feat_uoff, F, row_bits, n_lists, M_cap, k0, w.b.p0, w.b.n_dev, 0, nullptr);
                RECD_TRY(radix_sort_pairs<uint64_t>(ctx, sb, k0, w.b.p0, k1, w.b.p1, w.b.n_dev, M_cap, bits_b,
                                                    w.b.hist, w.b.bsum, &ks, &ps));
                RECD_TRY(prepare_rows<uint64_t>(ctx, sb, w, w.b, ks, M_cap, M_cap, row_bits, F, touched_rows,
                                                feat_roff, ctx->ev_plan_rows));
                pl.ps_b = ps;
            }
        }
        return RECD_OK;
        };
        // The host issues one chain after the other: the longer one first.  Sorting all F*B rows makes
        // step A's chain the longer one; from the run index it is a fraction of step B's.
        if (run_index) {
            RECD_TRY(chain_b());
            RECD_TRY(chain_a());
        } else {
            RECD_TRY(chain_a());
            RECD_TRY(chain_b());
        }
        RECD_HIP(ctx, hipGetLastError());
    }
    RECD_HIP(ctx, hipEventRecord(ctx->ev_plan_a, sa));
    RECD_HIP(ctx, hipEventRecord(ctx->ev_plan_b, sb));
    pl.pending = true;
    pl.valid = true;
    return RECD_OK;
}

extern "C" recd_status recd_backward_plan(recd_ctx *ctx, int F, int64_t B, int D, const int32_t *inverse,
                                          const int64_t *feat_uoff, const int64_t *u_values,
                                          const int64_t *u_offsets, const int64_t *rows, int64_t U_cap,
                                          int64_t M_cap, int64_t *touched_rows, int64_t *feat_roff)
{
    return plan_common(ctx, F, B, D, inverse, feat_uoff, u_values, u_offsets, rows, U_cap, M_cap, nullptr, 0,
                       touched_rows, feat_roff);
}

extern "C" recd_status recd_backward_plan_runs(recd_ctx *ctx, int F, int64_t B, int D, const int32_t *inverse,
                                               const int64_t *feat_uoff, const int64_t *u_values,
                                               const int64_t *u_offsets, const int64_t *rows, int64_t U_cap,
                                               int64_t M_cap, const int64_t *run_index, int64_t runs_cap,
                                               int64_t *touched_rows, int64_t *feat_roff)
{
    if (ctx && !run_index && (int64_t)F * B > 0)
        return recd_fail(ctx, RECD_EINVAL, "null run_index");
    return plan_common(ctx, F, B, D, inverse, feat_uoff, u_values, u_offsets, rows, U_cap, M_cap, run_index,
                       runs_cap, touched_rows, feat_roff);
}

extern "C" recd_status recd_backward_apply(recd_ctx *ctx, recd_pooling mode, const float *grad_out,
                                           float *grad_rows, void *const *tables,
                                           float *const *adagrad_state, float lr, float eps,
                                           int64_t *host_R)
{
    if (!ctx)
        return RECD_EINVAL;
    recd_ctx::BackwardPlan &pl = ctx->plan;
    if (!pl.valid || pl.ws != ctx->ws)
        return recd_fail(ctx, RECD_EINVAL,
                         "no valid plan: recd_backward_plan must be the context's last workspace-using call");
    pl.valid = false;
    if (mode != RECD_POOL_SUM && mode != RECD_POOL_MEAN)
        return recd_fail(ctx, RECD_EINVAL, "planned backward: pooling mode %d is not supported", (int)mode);
    const int F = pl.F, D = pl.D;
    const int64_t B = pl.B, n_lists = (int64_t)F * B, M_cap = pl.M_cap;
    if (n_lists > 0 && !grad_out)
        return recd_fail(ctx, RECD_EINVAL, "null grad_out");
    if ((tables == nullptr) != (adagrad_state == nullptr))
        return recd_fail(ctx, RECD_EINVAL, "tables and adagrad_state must be given together");
    if (M_cap > 0 && !grad_rows && !(tables && F <= RECD_F_PER_LAUNCH))
        return recd_fail(ctx, RECD_EINVAL,
                         "grad_rows may be NULL only with the optimizer and at most %d features",
                         RECD_F_PER_LAUNCH);
    for (int f = 0; f < F && tables; f++)
        if (!tables[f] || !adagrad_state[f])
            return recd_fail(ctx, RECD_EINVAL, "tables[%d] or adagrad_state[%d] is null", f, f);
    RECD_TRY(check_distinct_tables(ctx, F, tables, adagrad_state));
    RECD_HIP(ctx, hipSetDevice(ctx->device));
    hipStream_t st = ctx->stream;
    const BwdWs w = carve_bwd(ctx->ws, n_lists, M_cap, F, D, ctx->long_seg_cut);
    RECD_HIP(ctx, hipStreamWaitEvent(st, ctx->ev_plan_a, 0));
    if (pl.empty) {
        RECD_HIP(ctx, hipStreamWaitEvent(st, ctx->ev_plan_b, 0));
        pl.pending = false;
        hipLaunchKernelGGL(k_no_rows, dim3(1), dim3(64), 0, st, F, pl.feat_roff, w.list_off_b);
        RECD_HIP(ctx, hipGetLastError());
        if (host_R) {
            RECD_HIP(ctx, hipStreamSynchronize(st));
            host_R[0] = 0;
        }
        return RECD_OK;
    }
    const bool fused = tables != nullptr && F <= RECD_F_PER_LAUNCH;
    OptAdagrad oa;
    oa.n_feat = 0;
    if (fused) {
        oa.n_feat = F;
        for (int f = 0; f < F; f++) {
            oa.w[f] = static_cast<float *>(tables[f]);
            oa.m[f] = adagrad_state[f];
        }
        oa.lr = lr;
        oa.eps = eps;
    }
    // step A's sum over the planned segments
    {
        SegSumArgs a{};
        a.site = RECD_SITE_GRAD_STREAM;
        a.F = 1;
        a.D = D;
        a.table_dt = RECD_F32;
        a.out_dt = RECD_F32;
        a.tables.p[0] = grad_out;
        a.values = pl.ps_a;
        a.values_are_i32 = 1;
        a.offsets = w.seg_start;
        a.list_off = w.list_off;
        a.lists_bound = pl.U_cap;
        a.flat = 1;
        a.out = w.g_u;
        a.div_off = mode == RECD_POOL_MEAN ? pl.u_offsets : nullptr;
        RECD_TRY(recd_launch_segsum(ctx, a));
    }
    // Step B's grouping may still be running next to the sum above.  The cut of the long segments,
    // the last kernel of that chain, is needed only by the chunk passes, which sum_rows enqueues on
    // the same side stream behind it; the stream joins that side stream at the end of sum_rows.
    RECD_HIP(ctx, hipStreamWaitEvent(st, ctx->ev_plan_rows, 0));
    RECD_TRY(sum_rows(ctx, w, pl.ps_b, M_cap, M_cap, w.g_u, D, grad_rows, pl.touched_rows, fused ? &oa : nullptr,
                      nullptr));
    pl.pending = false;  // the stream now waits for everything the plan enqueued
    if (tables && !fused) {
        for (int f0 = 0; f0 < F; f0 += RECD_F_PER_LAUNCH) {
            OptPtrs ptrs;
            const int nf = F - f0 < RECD_F_PER_LAUNCH ? F - f0 : RECD_F_PER_LAUNCH;
            for (int f = 0; f < nf; f++) {
                ptrs.w[f] = static_cast<float *>(tables[f0 + f]);
                ptrs.m[f] = adagrad_state[f0 + f];
            }
            hipLaunchKernelGGL(k_adagrad, dim3(ctx->num_cu * 8), dim3(256), 0, st, grad_rows, pl.touched_rows,
                               pl.feat_roff, f0, nf, D, ptrs, lr, eps);
        }
        RECD_HIP(ctx, hipGetLastError());
    }
    if (host_R) {
        RECD_HIP(ctx, hipMemcpyAsync(ctx->host_pinned, w.list_off_b + 1, sizeof(int64_t), hipMemcpyDeviceToHost, st));
        RECD_HIP(ctx, hipMemcpyAsync(ctx->host_pinned + 1, w.b.n_dev + 1, sizeof(int64_t), hipMemcpyDeviceToHost,
                                     st));
        RECD_HIP(ctx, hipMemcpyAsync(ctx->host_pinned + 2, w.a.n_dev + 1, sizeof(int64_t), hipMemcpyDeviceToHost,
                                     st));
        RECD_HIP(ctx, hipStreamSynchronize(st));
        host_R[0] = ctx->host_pinned[0];
        if (ctx->host_pinned[1])
            return recd_fail(ctx, RECD_ECAPACITY, "M_cap=%lld is smaller than M", (long long)M_cap);
        if (ctx->host_pinned[2])
            return recd_fail(ctx, RECD_ECAPACITY, "runs_cap is smaller than the number of runs");
    }
    return RECD_OK;
}

extern "C" recd_status recd_backward_dedup(recd_ctx *ctx, int F, int64_t B, int D,
                                           const float *grad_out, const int32_t *inverse,
                                           const int64_t *feat_uoff, const int64_t *u_values,
                                           const int64_t *u_offsets, const int64_t *rows,
                                           int64_t U_cap, int64_t M_cap, int64_t *touched_rows,
                                           int64_t *feat_roff, float *grad_rows, void *const *tables,
                                           float *const *adagrad_state, float lr, float eps,
                                           int64_t *host_R)
{
    return backward_common(ctx, false, false, F, B, 0, D, grad_out, nullptr, inverse, feat_uoff, u_values,
                           nullptr, nullptr, u_offsets, rows, U_cap, M_cap, nullptr, touched_rows, feat_roff, grad_rows, tables,
                           adagrad_state, lr, eps, host_R);
}

extern "C" recd_status recd_backward_dedup_mode(recd_ctx *ctx, recd_pooling mode, int F, int64_t B, int D,
                                                const float *grad_out, const int32_t *inverse,
                                                const int64_t *feat_uoff, const int64_t *u_values,
                                                const int64_t *u_offsets, const int64_t *rows,
                                                int64_t U_cap, int64_t M_cap, int64_t *touched_rows,
                                                int64_t *feat_roff, float *grad_rows, void *const *tables,
                                                float *const *adagrad_state, float lr, float eps,
                                                int64_t *host_R)
{
    if (!ctx)
        return RECD_EINVAL;
    if (mode != RECD_POOL_SUM && mode != RECD_POOL_MEAN)
        return recd_fail(ctx, RECD_EINVAL,
                         "backward: pooling mode %d is not supported (sum and mean are)", (int)mode);
    return backward_common(ctx, false, mode == RECD_POOL_MEAN, F, B, 0, D, grad_out, nullptr, inverse,
                           feat_uoff, u_values, nullptr, nullptr, u_offsets, rows, U_cap, M_cap, nullptr, touched_rows,
                           feat_roff, grad_rows, tables, adagrad_state, lr, eps, host_R);
}

extern "C" recd_status recd_backward_sequence_dedup(recd_ctx *ctx, int F, int64_t B, int64_t N, int D,
                                                    const float *grad_out, const int64_t *offsets,
                                                    const int32_t *inverse, const int64_t *feat_uoff,
                                                    const int64_t *u_values, const int64_t *u_offsets,
                                                    const int64_t *rows, int64_t U_cap, int64_t M_cap,
                                                    float *grad_emb, int64_t *touched_rows,
                                                    int64_t *feat_roff, float *grad_rows,
                                                    void *const *tables, float *const *adagrad_state,
                                                    float lr, float eps, int64_t *host_R)
{
    return backward_common(ctx, true, false, F, B, N, D, grad_out, offsets, inverse, feat_uoff, u_values, nullptr,
                           nullptr, u_offsets, rows, U_cap, M_cap, grad_emb, touched_rows, feat_roff, grad_rows, tables,
                           adagrad_state, lr, eps, host_R);
}

extern "C" recd_status recd_backward_dedup_weighted(recd_ctx *ctx, int F, int64_t B, int D,
                                                    const float *grad_out, const int32_t *inverse,
                                                    const int64_t *feat_uoff, const int64_t *u_values,
                                                    const float *u_weights, const int64_t *u_offsets,
                                                    const int64_t *rows, int64_t U_cap, int64_t M_cap,
                                                    int64_t *touched_rows, int64_t *feat_roff,
                                                    float *grad_rows, void *const *tables,
                                                    float *const *adagrad_state, float lr, float eps,
                                                    int64_t *host_R)
{
    if (!ctx)
        return RECD_EINVAL;
    if (M_cap > 0 && !u_weights)
        return recd_fail(ctx, RECD_EINVAL, "null u_weights");
    return backward_common(ctx, false, false, F, B, 0, D, grad_out, nullptr, inverse, feat_uoff, u_values,
                           M_cap > 0 ? u_weights : nullptr, nullptr, u_offsets, rows, U_cap, M_cap, nullptr,
                           touched_rows, feat_roff, grad_rows, tables, adagrad_state, lr, eps, host_R);
}

extern "C" recd_status recd_backward_dedup_max(recd_ctx *ctx, int F, int64_t B, int D,
                                               const float *grad_out, const int32_t *inverse,
                                               const int64_t *feat_uoff, const int64_t *u_values,
                                               const int64_t *u_offsets, const int64_t *rows,
                                               int64_t U_cap, int64_t M_cap,
                                               const void *const *lookup_tables, int64_t *touched_rows,
                                               int64_t *feat_roff, float *grad_rows, void *const *tables,
                                               float *const *adagrad_state, float lr, float eps,
                                               int64_t *host_R)
{
    if (!ctx)
        return RECD_EINVAL;
    if (F > 0 && !lookup_tables)
        return recd_fail(ctx, RECD_EINVAL, "null lookup_tables");
    for (int f = 0; f < F; f++)
        if (!lookup_tables[f])
            return recd_fail(ctx, RECD_EINVAL, "lookup_tables[%d] is null", f);
    return backward_common(ctx, false, false, F, B, 0, D, grad_out, nullptr, inverse, feat_uoff, u_values,
                           nullptr, M_cap > 0 && F > 0 ? lookup_tables : nullptr, u_offsets, rows, U_cap, M_cap,
                           nullptr, touched_rows, feat_roff, grad_rows, tables, adagrad_state, lr, eps, host_R);
}

size_t recd_build_workspace(int F, int64_t B);

extern "C" recd_status recd_workspace_bytes(int F, int64_t B, int64_t N, int D, size_t *out_bytes)
{
    if (!out_bytes || F < 0 || B < 0 || N < 0 || D <= 0)
        return RECD_EINVAL;
    const size_t a = recd_build_workspace(F, B);
    const size_t b = recd_backward_workspace(F, B, N, D);
    *out_bytes = (a > b ? a : b) + 4096;
    return RECD_OK;
}
