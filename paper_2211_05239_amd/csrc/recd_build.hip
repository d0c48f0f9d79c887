// KJT -> IKJT builder (paper Sec. 4.2): which rows of a feature hold exactly the same list?
//
// Steps, all on the device, no host round trip:
//   hash+insert  a group of SG lanes per list.  A list equal to its predecessor in the batch (the
//                common case once a session's samples are adjacent, Sec. 4.1) is only marked as a
//                follower.  Any other list is a run head: its 64-bit hash (position-salted sum of mixed
//                ids, so lanes hash strided pairs of ids and add) is inserted by open addressing into a
//                per-feature table whose slots hold (hash tag, sample index).  A slot belongs to one
//                list *content*: a newcomer whose tag matches compares its list element by element
//                with the slot's current sample and, if equal, lowers the slot's sample index with
//                an atomic min; if not, it probes on.  Hash collisions therefore never merge lists.
//   flags        a run head is a first occurrence iff its slot's final sample index is its own;
//                per-block sums of (first, first*len) and the last run head of the block.
//   scan         exclusive scan of those over all F*B lists in (f,b) order: the unique-list number
//                and the position of its ids in u_values, both in first-occurrence order, and for
//                followers the run head they copy (rep[f,b] = rep of the head = smallest b' with the
//                same list).
//   emit         inverse[f,b] = number[rep] - number[f,0]; first occurrences copy their ids.
// The atomic min makes the result independent of insertion order: integer outputs are canonical.
#include "recd_internal.h"

namespace {

constexpr uint64_t kEmpty = ~0ull;
constexpr int kScanBlock = 1024;

__device__ __forceinline__ uint64_t mix64(uint64_t x)
{
    x ^= x >> 30;
    x *= 0xbf58476d1ce4e5b9ull;
    x ^= x >> 27;
    x *= 0x94d049bb133111ebull;
    x ^= x >> 31;
    return x;
}

// One list element's share of the list hash: cheaper than mix64 (one 64-bit multiply; the
// multiplies are most of the insert kernel's arithmetic), enough because the per-list sum of the
// terms goes through mix64 once more and an exact comparison follows every tag match anyway.
__device__ __forceinline__ uint64_t hash_term(uint64_t x)
{
    x ^= x >> 31;
    x *= 0xbf58476d1ce4e5b9ull;
    return x ^ (x >> 29);
}

__global__ void k_copy_i64(const int64_t *src, int64_t *dst) { *dst = *src; }

__global__ void k_fill_u64(uint64_t *p, int64_t n, uint64_t v)
{
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (int64_t)gridDim.x * blockDim.x)
        p[i] = v;
}

// Lists per lane group and launch: the group's lists are consecutive, and the first loads of all of
// them are issued together so that one group keeps several memory requests in flight.
constexpr int kLPG = 1;
constexpr int kHU = 2;   // strides of the long-list loop whose loads are issued together
constexpr int kFirst = 3;  // strides of a list loaded up front
// Threads per block of the insert kernel: one wave.  Lists of 1 to 256 ids finish at different times
// and a block's wave slots are free again only when its last wave is done (0.158 -> 0.149 ms).
constexpr int kHashBlock = 64;
// two adjacent ids; lists start on 8-byte boundaries only (global loads need no more)
typedef long long id2 __attribute__((ext_vector_type(2), aligned(8)));

// An id and (WT) the bit pattern of its weight as one hash input.
template <bool WT>
__device__ __forceinline__ uint64_t hash_item(int64_t id, uint32_t wbits)
{
    return WT ? (uint64_t)id + (uint64_t)wbits * 0xc2b2ae3d27d4eb4full : (uint64_t)id;
}

// WT: the lists carry one weight per id (wbits: their bit patterns); two lists are the same only if
// the weights agree too, so they enter the hash and every comparison.
template <int SG, bool WT>
__global__ __launch_bounds__(kHashBlock) void k_hash_insert(const int64_t *__restrict__ values,
                                                     const uint32_t *__restrict__ wbits,
                                                     const int64_t *__restrict__ offsets, int64_t B,
                                                     int64_t n_lists, uint64_t *table,
                                                     uint32_t cap_mask, int32_t *__restrict__ slot_of,
                                                     int weak_hash)
{
    const int s = threadIdx.x % SG;
    // Blocks go to the eight XCDs in turn; every XCD takes a contiguous eighth of the lists, so that
    // the predecessor of a block's first list, and the cache lines that neighbouring lists share,
    // were fetched by the block before it through the same L2 (with neighbouring blocks on different
    // XCDs the kernel fetched 1.3 times the ids from memory).
    const int64_t per_xcd = ((int64_t)gridDim.x + 7) / 8;
    const int64_t blk = (int64_t)(blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
    const int64_t l0 = (blk * (kHashBlock / SG) + threadIdx.x / SG) * kLPG;
    if (blk >= (int64_t)gridDim.x || l0 >= n_lists)
        return;  // whole lane group leaves together

    // offsets of rows l0-1 .. l0+kLPG (clamped to the array)
    int64_t off[kLPG + 2];
#pragma unroll
    for (int k = 0; k < kLPG + 2; k++) {
        int64_t i = l0 - 1 + k;
        i = i < 0 ? 0 : (i > n_lists ? n_lists : i);
        off[k] = offsets[i];
    }
    int64_t start[kLPG], len[kLPG], pstart[kLPG];
    int follows[kLPG];
    bool live[kLPG];
    uint64_t h[kLPG];
#pragma unroll
    for (int k = 0; k < kLPG; k++) {
        const int64_t l = l0 + k;
        live[k] = l < n_lists;
        start[k] = off[k + 1];
        len[k] = live[k] ? off[k + 2] - off[k + 1] : 0;
        pstart[k] = off[k];
        // the previous row of the same feature ends where this one starts
        follows[k] = live[k] && (l % B) != 0 && (start[k] - pstart[k]) == len[k];
        h[k] = 0;
    }
    // A lane takes two adjacent ids (and weights) per stride, one 16-byte load; a stride of the
    // group covers 2 * SG ids.  The hash is a position-salted sum, so which lane adds which id does
    // not matter.  The first kFirst strides of every list and of its predecessor are loaded up
    // front, all in flight together; longer lists continue kHU strides per trip.
    auto load2 = [&](const int64_t *base, int64_t t, int64_t n, bool on, int64_t &a, int64_t &b) {
        a = 0;
        b = 0;
        if (on && t + 1 < n) {
            const id2 p = *reinterpret_cast<const id2 *>(base + t);
            a = p.x;
            b = p.y;
        } else if (on && t < n) {
            a = base[t];
        }
    };
    auto loadw2 = [&](const uint32_t *base, int64_t t, int64_t n, bool on, uint32_t &a, uint32_t &b) {
        a = 0;
        b = 0;
        if (WT && on && t < n)
            a = base[t];
        if (WT && on && t + 1 < n)
            b = base[t + 1];
    };
    auto fold2 = [&](int k, int64_t t, int64_t a, int64_t b, int64_t pa, int64_t pb, uint32_t wa, uint32_t wb,
                     uint32_t pwa, uint32_t pwb) {
        // position salt (t + 1) * phi from the low 32 bits of the position (one 32 x 64-bit product;
        // it only has to be the same for equal lists)
        const uint64_t salt = (uint64_t)(uint32_t)(t + 1) * 0x9e3779b97f4a7c15ull;
        if (t < len[k]) {
            follows[k] &= pa == a && pwa == wa;
            h[k] += hash_term(hash_item<WT>(a, wa) + salt);
        }
        if (t + 1 < len[k]) {
            follows[k] &= pb == b && pwb == wb;
            h[k] += hash_term(hash_item<WT>(b, wb) + salt + 0x9e3779b97f4a7c15ull);
        }
    };
    int64_t va[kLPG][kFirst], vb[kLPG][kFirst], pa[kLPG][kFirst], pb[kLPG][kFirst];
    uint32_t wa[kLPG][kFirst], wb[kLPG][kFirst], pwa[kLPG][kFirst], pwb[kLPG][kFirst];
#pragma unroll
    for (int k = 0; k < kLPG; k++)
#pragma unroll
        for (int u = 0; u < kFirst; u++) {
            const int64_t t = 2 * s + u * 2 * SG;
            load2(values + start[k], t, len[k], true, va[k][u], vb[k][u]);
            load2(values + pstart[k], t, len[k], follows[k], pa[k][u], pb[k][u]);
            loadw2(wbits + start[k], t, len[k], true, wa[k][u], wb[k][u]);
            loadw2(wbits + pstart[k], t, len[k], follows[k], pwa[k][u], pwb[k][u]);
        }
#pragma unroll
    for (int k = 0; k < kLPG; k++) {
#pragma unroll
        for (int u = 0; u < kFirst; u++)
            fold2(k, 2 * s + u * 2 * SG, va[k][u], vb[k][u], pa[k][u], pb[k][u], wa[k][u], wb[k][u], pwa[k][u],
                  pwb[k][u]);
        for (int64_t t0 = 2 * s + kFirst * 2 * SG; t0 < len[k]; t0 += kHU * 2 * SG) {
            int64_t xa[kHU], xb[kHU], qa[kHU], qb[kHU];
            uint32_t ya[kHU], yb[kHU], za[kHU], zb[kHU];
#pragma unroll
            for (int u = 0; u < kHU; u++) {
                const int64_t t = t0 + u * 2 * SG;
                load2(values + start[k], t, len[k], true, xa[u], xb[u]);
                load2(values + pstart[k], t, len[k], follows[k], qa[u], qb[u]);
                loadw2(wbits + start[k], t, len[k], true, ya[u], yb[u]);
                loadw2(wbits + pstart[k], t, len[k], follows[k], za[u], zb[u]);
            }
#pragma unroll
            for (int u = 0; u < kHU; u++)
                fold2(k, t0 + u * 2 * SG, xa[u], xb[u], qa[u], qb[u], ya[u], yb[u], za[u], zb[u]);
        }
    }
#pragma unroll
    for (int m = SG / 2; m > 0; m >>= 1)
#pragma unroll
        for (int k = 0; k < kLPG; k++) {
            h[k] += __shfl_xor((unsigned long long)h[k], m, SG);
            follows[k] &= __shfl_xor(follows[k], m, SG);
        }

#pragma unroll
    for (int k = 0; k < kLPG; k++) {
        if (!live[k])
            continue;
        const int64_t l = l0 + k;
        if (follows[k]) {  // same list as the previous row: no table traffic at all
            if (s == 0)
                slot_of[l] = -1;
            continue;
        }
        const int64_t f = l / B;
        const int64_t b = l - f * B;
        uint64_t hh = mix64(h[k] ^ ((uint64_t)len[k] * 0xd6e8feb86659fd93ull + 1ull));
        if (weak_hash)
            hh = (uint64_t)len[k];  // test hook: only the exact comparison separates lists
        const uint64_t tag = hh >> 32;
        const uint64_t mine = (tag << 32) | (uint64_t)b;
        uint64_t *tab = table + (uint64_t)f * ((uint64_t)cap_mask + 1);
        uint32_t slot = (uint32_t)hh & cap_mask;
        // The table has at least 2*B slots per feature, so an empty slot or the list's own class
        // is met.
        for (;;) {
            unsigned long long old = 0;
            if (s == 0)
                old = atomicCAS(reinterpret_cast<unsigned long long *>(&tab[slot]), kEmpty, mine);
            old = __shfl(old, 0, SG);
            if (old == kEmpty)
                break;
            if ((old >> 32) == tag) {
                const int64_t ol = f * B + (int64_t)(old & 0xffffffffull);
                const int64_t ostart = offsets[ol];
                int eq = (offsets[ol + 1] - ostart) == len[k];
                if (eq)
                    for (int64_t t = s; t < len[k]; t += SG)
                        if (values[start[k] + t] != values[ostart + t] ||
                            (WT && wbits[start[k] + t] != wbits[ostart + t])) {
                            eq = 0;
                            break;
                        }
#pragma unroll
                for (int m = SG / 2; m > 0; m >>= 1)
                    eq &= __shfl_xor(eq, m, SG);
                if (eq) {
                    if (s == 0)
                        atomicMin(reinterpret_cast<unsigned long long *>(&tab[slot]), mine);
                    break;
                }
            }
            slot = (slot + 1) & cap_mask;
        }
        if (s == 0)
            slot_of[l] = (int32_t)slot;
    }
}

// Block-wide scan of (a, b, c): exclusive sums of a and b, and for c the maximum over the threads
// up to and including this one.  Totals (sum a, sum b, max c) are returned to every thread.
__device__ __forceinline__ void block_scan3(int64_t a, int64_t b, int64_t c, int64_t &ea, int64_t &eb,
                                            int64_t &ic, int64_t &ta, int64_t &tb, int64_t &tc)
{
    __shared__ int64_t s_a[kScanBlock / 64], s_b[kScanBlock / 64], s_c[kScanBlock / 64];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    int64_t ia = a, ib = b;
    ic = c;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int64_t xa = __shfl_up(ia, d), xb = __shfl_up(ib, d), xc = __shfl_up(ic, d);
        if (lane >= d) {
            ia += xa;
            ib += xb;
            ic = xc > ic ? xc : ic;
        }
    }
    __syncthreads();  // protect the shared arrays against the previous use
    if (lane == 63) {
        s_a[w] = ia;
        s_b[w] = ib;
        s_c[w] = ic;
    }
    __syncthreads();
    int64_t oa = 0, ob = 0;
    ta = 0;
    tb = 0;
    tc = -1;
    for (int i = 0; i < (int)(blockDim.x >> 6); i++) {
        if (i < w) {
            oa += s_a[i];
            ob += s_b[i];
            ic = s_c[i] > ic ? s_c[i] : ic;
        }
        ta += s_a[i];
        tb += s_b[i];
        tc = s_c[i] > tc ? s_c[i] : tc;
    }
    ea = oa + ia - a;
    eb = ob + ib - b;
}

// The scan of the numbering kernels, made of ballots: per thread two flags (first occurrence, run
// head), the length of a first occurrence and the row of a run head.  Exclusive counts of the flags
// and the nearest head at or before the thread come from wave ballots (no data moves between lanes);
// only the lengths take a shuffle scan.  Totals of the block are returned to every thread.
struct ListScan {
    int64_t firsts_before, heads_before, len_before;  // exclusive, inside the block
    int64_t head_row;                                  // nearest run head at or before the thread, -1: none yet
    int64_t firsts, heads, len, last_head;             // block totals
};

template <bool TOTALS_ONLY>
__device__ __forceinline__ ListScan block_scan_lists(bool first, bool head, int64_t flen, int64_t row)
{
    __shared__ uint32_t s_first[kScanBlock / 64], s_heads[kScanBlock / 64];
    __shared__ int64_t s_len[kScanBlock / 64], s_last[kScanBlock / 64];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const uint64_t mf = __ballot(first), mh = __ballot(head);
    const uint64_t le = lane == 63 ? ~0ull : ((1ull << (lane + 1)) - 1), lt = le >> 1;
    ListScan r;
    int64_t il = flen;  // inclusive sum of the lengths in the wave
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int64_t x = TOTALS_ONLY ? __shfl_xor(il, d) : __shfl_up(il, d);
        if (TOTALS_ONLY || lane >= d)
            il += x;
    }
    // row of the wave's lane k = row - lane + k
    const uint64_t hb = mh & le;
    r.head_row = hb ? row - lane + (63 - __builtin_clzll(hb)) : -1;
    __syncthreads();  // the shared arrays are free again
    if (lane == 63) {
        s_first[w] = (uint32_t)__popcll(mf);
        s_heads[w] = (uint32_t)__popcll(mh);
        s_len[w] = il;  // lane 63 holds the wave's sum in either mode
        s_last[w] = mh ? row - 63 + (63 - __builtin_clzll(mh)) : -1;
    }
    __syncthreads();
    r.firsts_before = __popcll(mf & lt);
    r.heads_before = __popcll(mh & lt);
    r.len_before = il - flen;
    r.firsts = r.heads = r.len = 0;
    r.last_head = -1;
    int64_t prev_last = -1;  // last head of the waves before this one (rows grow with the wave)
    for (int i = 0; i < (int)(blockDim.x >> 6); i++) {
        if (i < w) {
            r.firsts_before += s_first[i];
            r.heads_before += s_heads[i];
            r.len_before += s_len[i];
            prev_last = s_last[i] > prev_last ? s_last[i] : prev_last;
        }
        r.firsts += s_first[i];
        r.heads += s_heads[i];
        r.len += s_len[i];
        r.last_head = s_last[i] > r.last_head ? s_last[i] : r.last_head;
    }
    if (r.head_row < 0)
        r.head_row = prev_last;
    return r;
}

__global__ __launch_bounds__(kScanBlock) void k_flags(const int64_t *__restrict__ offsets, int64_t B,
                                                      int64_t n_lists,
                                                      const uint64_t *__restrict__ table,
                                                      uint32_t cap_mask,
                                                      const int32_t *__restrict__ slot_of,
                                                      int64_t *__restrict__ bs_cnt,
                                                      int64_t *__restrict__ bs_len,
                                                      int64_t *__restrict__ bs_head)
{
    const int64_t l = (int64_t)blockIdx.x * kScanBlock + threadIdx.x;
    int64_t first = 0, flen = 0, head = -1;
    if (l < n_lists) {
        const int32_t slot = slot_of[l];
        if (slot >= 0) {
            head = l;
            const int64_t f = l / B, b = l - f * B;
            const uint64_t e = table[(uint64_t)f * ((uint64_t)cap_mask + 1) + (uint32_t)slot];
            if ((int64_t)(e & 0xffffffffull) == b) {
                first = 1;
                flen = offsets[l + 1] - offsets[l];
            }
        }
    }
    // two counts ride in one sum: first occurrences in the low half, run heads in the high half
    // (both stay below 2^31)
    const ListScan sc = block_scan_lists<true>(first != 0, head >= 0, flen, l);
    if (threadIdx.x == 0) {
        bs_cnt[blockIdx.x] = sc.firsts + (sc.heads << 32);
        bs_len[blockIdx.x] = sc.len;
        bs_head[blockIdx.x] = sc.last_head;
    }
}

// one block, in place: exclusive sums of a and b, exclusive running maximum of c (-1 before the
// first entry)
__global__ __launch_bounds__(kScanBlock) void k_scan_blocks(int64_t *a, int64_t *b, int64_t *c, int64_t n)
{
    int64_t ca = 0, cb = 0, cc = -1;
    for (int64_t base = 0; base < n; base += kScanBlock) {
        const int64_t i = base + threadIdx.x;
        const int64_t va = i < n ? a[i] : 0, vb = i < n ? b[i] : 0, vc = i < n ? c[i] : -1;
        int64_t ea, eb, ic, ta, tb, tc;
        block_scan3(va, vb, vc, ea, eb, ic, ta, tb, tc);
        // exclusive maximum: shift the inclusive one by one thread
        int64_t prev = __shfl_up(ic, 1);
        __shared__ int64_t s_last[kScanBlock / 64];
        if ((threadIdx.x & 63) == 63)
            s_last[threadIdx.x >> 6] = ic;
        __syncthreads();
        if ((threadIdx.x & 63) == 0)
            prev = threadIdx.x == 0 ? -1 : s_last[(threadIdx.x >> 6) - 1];
        __syncthreads();
        if (i < n) {
            a[i] = ca + ea;
            b[i] = cb + eb;
            c[i] = prev > cc ? prev : cc;
        }
        ca += ta;
        cb += tb;
        cc = tc > cc ? tc : cc;
    }
}

__global__ __launch_bounds__(kScanBlock) void k_number(const int64_t *__restrict__ offsets, int64_t B,
                                                       int64_t n_lists, int F,
                                                       const uint64_t *__restrict__ table,
                                                       uint32_t cap_mask,
                                                       const int32_t *__restrict__ slot_of,
                                                       const int64_t *__restrict__ bs_cnt,
                                                       const int64_t *__restrict__ bs_len,
                                                       const int64_t *__restrict__ bs_head,
                                                       int32_t *__restrict__ rep,
                                                       int32_t *__restrict__ number,
                                                       int32_t *__restrict__ src_of,
                                                       int64_t *__restrict__ u_offsets,
                                                       int64_t *__restrict__ feat_uoff,
                                                       int64_t *__restrict__ counts,
                                                       int64_t *mailbox, int64_t seq,
                                                       int32_t *__restrict__ hrank = nullptr,
                                                       int64_t *__restrict__ run_index = nullptr)
{
    const int64_t l = (int64_t)blockIdx.x * kScanBlock + threadIdx.x;
    int64_t first = 0, flen = 0, head = -1, b = -1, f = 0, my_rep = -1;
    if (l < n_lists) {
        f = l / B;
        b = l - f * B;
        const int32_t slot = slot_of[l];
        if (slot >= 0) {
            head = l;
            const uint64_t e = table[(uint64_t)f * ((uint64_t)cap_mask + 1) + (uint32_t)slot];
            my_rep = (int64_t)(e & 0xffffffffull);
            if (my_rep == b) {
                first = 1;
                flen = offsets[l + 1] - offsets[l];
            }
        }
    }
    const ListScan sc = block_scan_lists<false>(first != 0, head >= 0, flen, l);
    // What the blocks before this one hold: the block's first wave adds up the per-block sums of
    // k_flags itself (a few thousand values from L2) instead of a one-block scan kernel in between.
    __shared__ int64_t s_carry[3];
    if (threadIdx.x < 64) {
        int64_t pa = 0, pb = 0, pc = -1;
        for (int64_t i = threadIdx.x; i < (int64_t)blockIdx.x; i += 64) {
            pa += bs_cnt[i];
            pb += bs_len[i];
            pc = bs_head[i] > pc ? bs_head[i] : pc;
        }
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            pa += __shfl_xor(pa, d);
            pb += __shfl_xor(pb, d);
            const int64_t x = __shfl_xor(pc, d);
            pc = x > pc ? x : pc;
        }
        if (threadIdx.x == 0) {
            s_carry[0] = pa;
            s_carry[1] = pb;
            s_carry[2] = pc;
        }
    }
    __syncthreads();
    const int64_t carry_cnt = s_carry[0], carry_len = s_carry[1], carry_head = s_carry[2];
    const int64_t ea = sc.firsts_before + (sc.heads_before << 32), eb = sc.len_before, ic = sc.head_row;
    if (l < n_lists) {
        const int64_t packed = carry_cnt + ea;   // first occurrences | run heads before l
        if (hrank)
            hrank[l] = head >= 0 ? (int32_t)(packed >> 32) : -1;
        if (head < 0) {
            // follower: copy the representative of the run head (the nearest head at or before l;
            // row 0 of a feature is always a head, so the run never leaves the feature)
            const int64_t hl = ic > carry_head ? ic : carry_head;
            const uint64_t e = table[(uint64_t)f * ((uint64_t)cap_mask + 1) + (uint32_t)slot_of[hl]];
            my_rep = (int64_t)(e & 0xffffffffull);
        }
        rep[l] = (int32_t)my_rep;
        const int64_t num = packed & 0xffffffffll;  // unique lists before (f,b), all features
        const int64_t pos = carry_len + eb;  // their ids
        number[l] = (int32_t)num;
        if (first) {
            u_offsets[num] = pos;
            src_of[num] = (int32_t)l;
        }
        if (b == 0)
            feat_uoff[f] = num;
        if (l == n_lists - 1) {
            const int64_t U = num + first, M = pos + flen;
            u_offsets[U] = M;
            feat_uoff[F] = U;
            const int64_t n_runs = (packed >> 32) + (head >= 0);  // runs of adjacent rows with one list
            counts[0] = U;
            counts[1] = M;
            counts[2] = n_runs;
            if (run_index) {
                // header {runs, U, M} and the closing entry (a run ends where the next one starts)
                run_index[0] = n_runs;
                run_index[1] = U;
                run_index[2] = M;
                run_index[3 * (1 + n_runs)] = n_lists;
                run_index[3 * (1 + n_runs) + 1] = M;
                run_index[3 * (1 + n_runs) + 2] = 0;
            }
            if (mailbox) {
                // U and M are final here: the host may have them while the last builder kernel still
                // copies ids (values first, the sequence number last, each visible to the host
                // before the next)
                mailbox[0] = U;
                mailbox[1] = M;
                mailbox[2] = n_runs;
                __threadfence_system();
                mailbox[7] = seq;
                __threadfence_system();
            }
        }
    }
}

// Last builder kernel, two kinds of blocks in one launch:
//   blocks [0, inv_blocks): one thread per row, inverse[f,b] = number[rep] - number[f,0];
//   the others: one group of SG lanes per *unique* list (source row recorded by k_number), striding
//   until the device-side count U is reached, copy the list's ids into u_values.
template <int SG>
__global__ __launch_bounds__(256) void k_emit(const int64_t *__restrict__ values,
                                              const int64_t *__restrict__ offsets, int64_t B,
                                              int64_t n_lists, const int32_t *__restrict__ rep,
                                              const int32_t *__restrict__ number,
                                              const int32_t *__restrict__ src_of,
                                              const int64_t *__restrict__ u_offsets,
                                              const int64_t *__restrict__ counts,
                                              int64_t *__restrict__ u_values,
                                              int32_t *__restrict__ inverse, unsigned inv_blocks,
                                              const uint32_t *__restrict__ wbits = nullptr,
                                              uint32_t *__restrict__ u_wbits = nullptr,
                                              unsigned fill_blocks = 0, uint64_t *fill = nullptr,
                                              int64_t fill_n = 0, const int32_t *__restrict__ hrank = nullptr,
                                              int64_t *__restrict__ run_index = nullptr)
{
    if (blockIdx.x < fill_blocks) {
        // the hash tables are no longer needed: leave them empty for the next build
        for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < fill_n; i += (int64_t)fill_blocks * 256)
            fill[i] = kEmpty;
        return;
    }
    const unsigned bid = blockIdx.x - fill_blocks;
    if (bid < inv_blocks) {
        const int64_t l = (int64_t)bid * 256 + threadIdx.x;
        if (l < n_lists) {
            const int64_t f = l / B;
            const int32_t u = number[f * B + rep[l]];
            inverse[l] = u - number[f * B];
            if (run_index && hrank[l] >= 0) {
                // run entry: {row | (unique list, first-occurrence flag) << 32, ids at, ids}
                int64_t *e = run_index + 3 * (1 + (int64_t)hrank[l]);
                const uint32_t uf = (uint32_t)u | (rep[l] == (int32_t)(l - f * B) ? 0x80000000u : 0u);
                e[0] = (int64_t)(((uint64_t)uf << 32) | (uint32_t)l);
                e[1] = u_offsets[u];
                e[2] = offsets[l + 1] - offsets[l];
            }
        }
        return;
    }
    const int s = threadIdx.x % SG;
    const int64_t U = counts[0];
    const int64_t stride = (int64_t)(gridDim.x - fill_blocks - inv_blocks) * (256 / SG);
    for (int64_t u = (int64_t)(bid - inv_blocks) * (256 / SG) + threadIdx.x / SG; u < U;
         u += stride) {
        const int64_t l = src_of[u];
        const int64_t start = offsets[l], len = offsets[l + 1] - start;
        const int64_t dst = u_offsets[u];
        for (int64_t t = s; t < len; t += SG)
            u_values[dst + t] = values[start + t];
        if (wbits)  // the weights of a weighted KJT travel with the ids
            for (int64_t t = s; t < len; t += SG)
                u_wbits[dst + t] = wbits[start + t];
    }
}

// ---- small batches: the whole builder in one launch ---------------------------------------------
// Up to kSmallB rows per feature: one block per feature does what the four kernels above do, with
// the feature's hash table and per-row arrays in LDS.  The blocks meet once: every block publishes
// its counts (unique lists, runs, ids) in two self-describing 64-bit words and then reads those of
// the features before it, which were dispatched earlier and never wait for a later block.  The last
// block to arrive adds up the batch's totals, publishes them and clears the words for the next
// launch.  A wait is bounded; a block whose wait expires numbers from zero (every write stays inside
// the outputs) and the totals are published as -1.
// The outputs are the canonical ones (first-occurrence numbering), the same as the general path's.
constexpr int kSmallB = 1024;
constexpr int kSmallThreads = 1024;
constexpr int kSmallSpinLimit = 1 << 20;
constexpr int64_t kSmallIds = 1 << 20;  // beyond this the general path's parallelism wins
constexpr uint32_t kSmallEmpty = 0xffffffffu;
constexpr uint64_t kSmallValid = 1ull << 63;

// Wave 0: sums of the published words of features [0, n); false if a word did not arrive in time.
__device__ __forceinline__ bool small_gather(const uint64_t *agg, int n, int lane, int spin_limit, int64_t &u,
                                             int64_t &r, int64_t &m)
{
    u = r = m = 0;
    int ok = spin_limit >= 0;  // a negative limit makes every wait expire (test hook)
    for (int i = lane; i < n; i += 64) {
        uint64_t w0 = 0, w1 = 0;
        int spins = 0;
        for (;;) {
            w0 = __hip_atomic_load(agg + 2 * i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            w1 = __hip_atomic_load(agg + 2 * i + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if ((w0 & kSmallValid) && (w1 & kSmallValid))
                break;
            if (++spins > spin_limit) {
                ok = 0;
                break;
            }
            __builtin_amdgcn_s_sleep(2);
        }
        if (ok) {
            u += (int64_t)(w0 & 0xffffull);
            r += (int64_t)((w0 >> 16) & 0xffffull);
            m += (int64_t)(w1 & ~kSmallValid);
        }
    }
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        u += __shfl_xor(u, d);
        r += __shfl_xor(r, d);
        m += __shfl_xor(m, d);
        ok &= __shfl_xor(ok, d);
    }
    return ok != 0;
}

// Inclusive sums over the wave's lanes: shifts inside the rows of 16 lanes (data-parallel primitives,
// no LDS traffic), then the totals of the rows before the lane's own.
__device__ __forceinline__ uint32_t wave_scan_add(uint32_t x, int lane)
{
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x111, 0xf, 0xf, false);  // row_shr:1
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x112, 0xf, 0xf, false);  // row_shr:2
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x114, 0xf, 0xf, false);  // row_shr:4
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x118, 0xf, 0xf, false);  // row_shr:8
    const uint32_t t0 = (uint32_t)__builtin_amdgcn_readlane((int)x, 15), t1 = (uint32_t)__builtin_amdgcn_readlane((int)x, 31),
                   t2 = (uint32_t)__builtin_amdgcn_readlane((int)x, 47);
    const int row = lane >> 4;
    return x + (row >= 1 ? t0 : 0u) + (row >= 2 ? t1 : 0u) + (row >= 3 ? t2 : 0u);
}

// The same inside one row of 16 lanes only (lanes 0..15 of a wave hold the 16 values).
__device__ __forceinline__ uint32_t row_scan_add(uint32_t x)
{
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x111, 0xf, 0xf, false);
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x112, 0xf, 0xf, false);
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x114, 0xf, 0xf, false);
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x118, 0xf, 0xf, false);
    return x;
}
__device__ __forceinline__ int row_scan_max(int x)
{
    int y = __builtin_amdgcn_update_dpp(-1, x, 0x111, 0xf, 0xf, false);
    x = y > x ? y : x;
    y = __builtin_amdgcn_update_dpp(-1, x, 0x112, 0xf, 0xf, false);
    x = y > x ? y : x;
    y = __builtin_amdgcn_update_dpp(-1, x, 0x114, 0xf, 0xf, false);
    x = y > x ? y : x;
    y = __builtin_amdgcn_update_dpp(-1, x, 0x118, 0xf, 0xf, false);
    return y > x ? y : x;
}

// agg: 2 words per feature, then the arrival counter and the failure mark; all zero between launches.
// A feature's ids are one contiguous stretch of `values`: up to kSmallStage of them are brought into
// LDS with one round of coalesced loads, and hashing, comparing and copying read them there (longer
// stretches are read from memory each time).  Small kernels run at low clocks, so the instruction
// count matters here: 32-bit hashing (the exact comparison decides anyway), ballots and lane shifts
// for the scans, one barrier per phase.
constexpr int kSmallStage = 16384;

template <int SG>
__global__ __launch_bounds__(kSmallThreads) void k_build_small(const int64_t *__restrict__ values,
                                                               const int64_t *__restrict__ offsets, int B, int F,
                                                               uint32_t cap_mask, int weak_hash, int spin_limit,
                                                               uint64_t *agg, int64_t *__restrict__ u_values,
                                                               int64_t *__restrict__ u_offsets,
                                                               int32_t *__restrict__ inverse,
                                                               int64_t *__restrict__ feat_uoff,
                                                               int64_t *__restrict__ counts, int64_t *mailbox,
                                                               int64_t seq, int64_t *__restrict__ run_index)
{
    __shared__ int64_t s_ids[kSmallStage];
    __shared__ uint32_t s_tab[2 * kSmallB];
    __shared__ uint32_t s_off[kSmallB + 1], s_pos[kSmallB];  // a row's ids start at s_off, relative to the feature
    __shared__ int16_t s_slot[kSmallB];
    __shared__ uint16_t s_num[kSmallB], s_src[kSmallB];
    __shared__ uint32_t s_wcnt[kSmallThreads / 64], s_wlen[kSmallThreads / 64];
    __shared__ int s_wlast[kSmallThreads / 64];
    __shared__ int64_t s_base[4];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int f = blockIdx.x;
    const int64_t l0 = (int64_t)f * B;

    // offsets of the feature's rows (one load per thread), the empty table
    const int64_t fstart = offsets[l0];
    for (int i = tid; i <= B; i += kSmallThreads)
        s_off[i] = (uint32_t)(offsets[l0 + i] - fstart);
    for (int i = tid; i <= (int)cap_mask; i += kSmallThreads)
        s_tab[i] = kSmallEmpty;
    __syncthreads();
    const int n_ids = (int)s_off[B];
    const bool staged = n_ids <= kSmallStage;
    const int64_t *gids = values + fstart;
    if (staged) {
        for (int i0 = tid; i0 < n_ids; i0 += 8 * kSmallThreads) {
            int64_t v[8];
#pragma unroll
            for (int k = 0; k < 8; k++) {
                const int i = i0 + k * kSmallThreads;
                v[k] = i < n_ids ? gids[i] : 0;
            }
#pragma unroll
            for (int k = 0; k < 8; k++) {
                const int i = i0 + k * kSmallThreads;
                if (i < n_ids)
                    s_ids[i] = v[k];
            }
        }
        __syncthreads();
    }

    // ---- hash + insert: SG lanes per row, all rows of the feature at once ---------------------------
    // id(i): the feature's i-th id, from LDS or from memory
    auto insert_rows = [&](auto id) {
        const int s = tid % SG;
        const int b = tid / SG;
        if (b >= B)
            return;
        const int start = (int)s_off[b], len = (int)s_off[b + 1] - start;
        const int pstart = b > 0 ? (int)s_off[b - 1] : start;
        int follows = b > 0 && (start - pstart) == len;
        uint32_t h = 0;
        for (int t0 = s; t0 < len; t0 += 4 * SG) {
            int64_t v[4], q[4];
#pragma unroll
            for (int k = 0; k < 4; k++) {
                const int t = t0 + k * SG;
                v[k] = t < len ? id(start + t) : 0;
                q[k] = (follows && t < len) ? id(pstart + t) : v[k];
            }
#pragma unroll
            for (int k = 0; k < 4; k++) {
                const int t = t0 + k * SG;
                if (t < len) {
                    follows &= q[k] == v[k];
                    // position-salted sum of mixed ids: which lane adds which id does not matter
                    uint32_t x = (uint32_t)v[k] ^ ((uint32_t)((uint64_t)v[k] >> 32) * 0x9e3779b1u);
                    x = (x + (uint32_t)(t + 1) * 0x7feb352du) * 0x85ebca6bu;
                    h += x ^ (x >> 15);
                }
            }
        }
#pragma unroll
        for (int m = SG / 2; m > 0; m >>= 1) {
            h += __shfl_xor(h, m, SG);
            follows &= __shfl_xor(follows, m, SG);
        }
        if (follows) {
            if (s == 0)
                s_slot[b] = -1;
            return;
        }
        uint32_t hh = h ^ ((uint32_t)len * 0xc2b2ae35u + 1u);
        hh ^= hh >> 16;
        hh *= 0x85ebca6bu;
        hh ^= hh >> 13;
        hh *= 0xc2b2ae35u;
        hh ^= hh >> 16;
        if (weak_hash)
            hh = (uint32_t)len;  // test hook: only the exact comparison separates lists
        const uint32_t tag = hh >> 11;                     // 21 bits
        const uint32_t mine = (tag << 10) | (uint32_t)b;  // below 2^31: never the empty mark
        uint32_t slot = hh & cap_mask;
        // at least 2 * B slots: an empty slot or the list's own class is met
        for (;;) {
            uint32_t old = 0;
            if (s == 0)
                old = atomicCAS(&s_tab[slot], kSmallEmpty, mine);
            old = __shfl(old, 0, SG);
            if (old == kSmallEmpty)
                break;
            if ((old >> 10) == tag) {
                const int ob = (int)(old & 1023u);
                const int ostart = (int)s_off[ob];
                int eq = ((int)s_off[ob + 1] - ostart) == len;
                if (eq)
                    for (int t = s; t < len; t += SG)
                        if (id(start + t) != id(ostart + t)) {
                            eq = 0;
                            break;
                        }
#pragma unroll
                for (int m = SG / 2; m > 0; m >>= 1)
                    eq &= __shfl_xor(eq, m, SG);
                if (eq) {
                    if (s == 0)
                        atomicMin(&s_tab[slot], mine);
                    break;
                }
            }
            slot = (slot + 1) & cap_mask;
        }
        if (s == 0)
            s_slot[b] = (int16_t)slot;
    };
    if (staged)
        insert_rows([&](int i) { return s_ids[i]; });
    else
        insert_rows([&](int i) { return gids[i]; });
    __syncthreads();

    // ---- numbering inside the feature: one row per thread -----------------------------------------
    const int b = tid;
    bool first = false, head = false;
    int my_rep = -1, my_len = 0, my_slot = -1;
    if (b < B) {
        my_slot = s_slot[b];
        my_len = (int)(s_off[b + 1] - s_off[b]);
        if (my_slot >= 0) {
            head = true;
            my_rep = (int)(s_tab[my_slot] & 1023u);
            first = my_rep == b;
        }
    }
    const uint64_t mf = __ballot(first), mh = __ballot(head);
    const uint64_t le = lane == 63 ? ~0ull : ((1ull << (lane + 1)) - 1), lt = le >> 1;
    const uint32_t ilen = wave_scan_add(first ? (uint32_t)my_len : 0u, lane);  // inclusive in the wave
    const uint64_t hb = mh & le;
    int head_row = hb ? b - lane + (63 - __builtin_clzll(hb)) : -1;  // nearest head at or before me in the wave
    if (lane == 63) {
        s_wcnt[wv] = (uint32_t)__popcll(mf) | ((uint32_t)__popcll(mh) << 16);
        s_wlen[wv] = ilen;
        s_wlast[wv] = mh ? b - 63 + (63 - __builtin_clzll(mh)) : -1;
    }
    __syncthreads();
    // every wave scans the 16 wave totals itself (lanes 0..15): no second barrier
    const int wl = lane & 15;
    const uint32_t wc_i = row_scan_add(s_wcnt[wl]), wn_i = row_scan_add(s_wlen[wl]);
    const int wh_i = row_scan_max(s_wlast[wl]);
    const uint32_t tot_cnt = (uint32_t)__builtin_amdgcn_readlane((int)wc_i, 15);
    const uint32_t tot_len = (uint32_t)__builtin_amdgcn_readlane((int)wn_i, 15);
    uint32_t pre_cnt = 0, pre_len = 0;
    int pre_last = -1;
    if (wv > 0) {
        pre_cnt = (uint32_t)__builtin_amdgcn_readlane((int)wc_i, wv - 1);
        pre_len = (uint32_t)__builtin_amdgcn_readlane((int)wn_i, wv - 1);
        pre_last = __builtin_amdgcn_readlane(wh_i, wv - 1);
    }
    const uint32_t firsts_before = (pre_cnt & 0xffffu) + (uint32_t)__popcll(mf & lt);
    const uint32_t heads_before = (pre_cnt >> 16) + (uint32_t)__popcll(mh & lt);
    const uint32_t len_before = pre_len + ilen - (first ? (uint32_t)my_len : 0u);
    const uint32_t n_first = tot_cnt & 0xffffu, n_heads = tot_cnt >> 16;
    if (head_row < 0)
        head_row = pre_last;
    if (b < B) {
        if (!head)  // follower: the representative of its run head (row 0 is always a head)
            my_rep = (int)(s_tab[s_slot[head_row]] & 1023u);
        if (first) {
            s_num[b] = (uint16_t)firsts_before;
            s_pos[b] = len_before;
            s_src[firsts_before] = (uint16_t)b;
        }
    }
    if (tid == 0) {
        __hip_atomic_store(agg + 2 * f, kSmallValid | ((uint64_t)n_heads << 16) | (uint64_t)n_first,
                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(agg + 2 * f + 1, kSmallValid | (uint64_t)tot_len, __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();  // s_num is complete
    // what needs no other feature's counts goes out while they travel
    uint32_t lu = 0;
    if (b < B) {
        lu = s_num[my_rep];
        inverse[l0 + b] = (int32_t)lu;
    }

    // ---- the features before this one ----------------------------------------------------------------
    bool ok = true;
    if (wv == 0) {
        int64_t bu, br, bm;
        ok = small_gather(agg, f, lane, spin_limit, bu, br, bm);
        if (!ok)
            bu = br = bm = 0;
        if (lane == 0) {
            s_base[0] = bu;
            s_base[1] = br;
            s_base[2] = bm;
        }
    }
    __syncthreads();
    const int64_t base_u = s_base[0], base_r = s_base[1], base_m = s_base[2];

    // ---- emit ---------------------------------------------------------------------------------------------
    if (b < B) {
        if (first)
            u_offsets[base_u + lu] = base_m + s_pos[b];
        if (b == 0)
            feat_uoff[f] = base_u;
        if (run_index && head) {
            int64_t *e = run_index + 3 * (1 + base_r + heads_before);
            const uint32_t uf = (uint32_t)(base_u + lu) | (first ? 0x80000000u : 0u);
            e[0] = (int64_t)(((uint64_t)uf << 32) | (uint32_t)(l0 + b));
            e[1] = base_m + s_pos[my_rep];
            e[2] = (int64_t)my_len;
        }
    }
    auto copy_lists = [&](auto id) {
        constexpr int CG = 8;  // lanes per copied list
        for (int k = tid / CG; k < (int)n_first; k += kSmallThreads / CG) {
            const int sb = s_src[k];
            const int start = (int)s_off[sb], len = (int)s_off[sb + 1] - start;
            const int64_t dst = base_m + s_pos[sb];
            for (int t = tid % CG; t < len; t += CG)
                u_values[dst + t] = id(start + t);
        }
    };
    if (staged)
        copy_lists([&](int i) { return s_ids[i]; });
    else
        copy_lists([&](int i) { return gids[i]; });

    // ---- arrival: the last block adds up the batch and leaves the words clear -----------------------------
    if (wv == 0) {
        uint64_t *arrived = agg + 2 * (size_t)F;
        unsigned long long before = 0;
        if (lane == 0) {
            if (!ok)
                __hip_atomic_store(agg + 2 * (size_t)F + 1, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            // my words and my reads of the others' lie before the arrival
            before = __hip_atomic_fetch_add(arrived, 1ull, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
        }
        before = __shfl(before, 0);
        if (before == (unsigned long long)(F - 1)) {
            int64_t U, R, M;
            bool all = small_gather(agg, F, lane, spin_limit, U, R, M);
            const uint64_t failed = __hip_atomic_load(agg + 2 * (size_t)F + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            all = all && failed == 0;
            for (int i = lane; i < 2 * F + 2; i += 64)
                __hip_atomic_store(agg + i, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (lane == 0) {
                if (all) {
                    u_offsets[U] = M;
                    feat_uoff[F] = U;
                    if (run_index) {
                        run_index[0] = R;
                        run_index[1] = U;
                        run_index[2] = M;
                        run_index[3 * (1 + R)] = (int64_t)F * B;
                        run_index[3 * (1 + R) + 1] = M;
                        run_index[3 * (1 + R) + 2] = 0;
                    }
                } else {
                    U = R = M = -1;
                    if (run_index)
                        run_index[0] = 0;  // no runs: the one-pass lookup does nothing
                }
                counts[0] = U;
                counts[1] = M;
                counts[2] = R;
                if (mailbox) {
                    // every word carries the build's sequence number: the host needs no ordering between them
                    const uint64_t tag = (uint64_t)RECD_MAILBOX_TAG_BIT | ((uint64_t)seq & (RECD_MAILBOX_TAG_BIT - 1));
                    mailbox[0] = (int64_t)((tag << 40) | ((uint64_t)U & 0xffffffffffull));
                    mailbox[1] = (int64_t)((tag << 40) | ((uint64_t)M & 0xffffffffffull));
                    mailbox[2] = (int64_t)((tag << 40) | ((uint64_t)R & 0xffffffffffull));
                }
            }
        }
    }
}

__global__ void k_empty_ikjt(int F, int64_t *u_offsets, int64_t *feat_uoff, int64_t *counts)
{
    for (int f = threadIdx.x; f <= F; f += blockDim.x)
        feat_uoff[f] = 0;
    if (threadIdx.x == 0) {
        u_offsets[0] = 0;
        counts[0] = 0;
        counts[1] = 0;
        counts[2] = 0;
    }
}

// ---- grouped IKJT (Sec. 4.2 "Grouped IKJTs") ---------------------------------------------------
// One inverse per group of consecutive features: the item is the row b of group g, i.e. the tuple
// of the lists (f,b) over the group's features.  Same scheme as above with the tuple in the place
// of the list: a row equal to its predecessor in every feature is a follower; run heads are hashed
// over all their lists (feature-salted) and meet in a per-group table; a tag match is followed by
// an exact comparison of the whole tuple.
template <int SG>
__global__ __launch_bounds__(256) void k_group_hash_insert(const int64_t *__restrict__ values,
                                                           const int64_t *__restrict__ offsets,
                                                           int64_t B, int64_t n_items,
                                                           const int32_t *__restrict__ group_off,
                                                           uint64_t *table, uint32_t cap_mask,
                                                           int32_t *__restrict__ slot_of, int weak_hash)
{
    const int s = threadIdx.x % SG;
    const int64_t item = (int64_t)blockIdx.x * (256 / SG) + threadIdx.x / SG;
    if (item >= n_items)
        return;  // whole lane group leaves together
    const int64_t g = item / B, b = item - g * B;
    const int f0 = group_off[g], f1 = group_off[g + 1];
    int follows = b != 0;
    uint64_t h = 0;
    int64_t total_len = 0;
    for (int f = f0; f < f1; f++) {
        const int64_t l = (int64_t)f * B + b;
        const int64_t o1 = offsets[l], len = offsets[l + 1] - o1;
        const int64_t o0 = b != 0 ? offsets[l - 1] : o1;
        follows &= (o1 - o0) == len;  // same for all lanes
        const uint64_t salt = (uint64_t)(f - f0 + 1) * 0xc2b2ae3d27d4eb4full;
        for (int64_t t = s; t < len; t += SG) {
            const int64_t x = values[o1 + t];
            if (follows)
                follows &= values[o0 + t] == x;
            h += mix64((uint64_t)x + (uint64_t)(t + 1) * 0x9e3779b97f4a7c15ull + salt);
        }
        if (s == 0)
            h += mix64((uint64_t)len * 0xd6e8feb86659fd93ull + salt + 1ull);
        total_len += len;
    }
#pragma unroll
    for (int m = SG / 2; m > 0; m >>= 1) {
        h += __shfl_xor((unsigned long long)h, m, SG);
        follows &= __shfl_xor(follows, m, SG);
    }
    if (follows) {
        if (s == 0)
            slot_of[item] = -1;
        return;
    }
    uint64_t hh = mix64(h);
    if (weak_hash)
        hh = (uint64_t)total_len;  // test hook: only the exact comparison separates tuples
    const uint64_t tag = hh >> 32;
    const uint64_t mine = (tag << 32) | (uint64_t)b;
    uint64_t *tab = table + (uint64_t)g * ((uint64_t)cap_mask + 1);
    uint32_t slot = (uint32_t)hh & cap_mask;
    // at least 2*B slots per group: an empty slot or the tuple's own class is met
    for (;;) {
        unsigned long long old = 0;
        if (s == 0)
            old = atomicCAS(reinterpret_cast<unsigned long long *>(&tab[slot]), kEmpty, mine);
        old = __shfl(old, 0, SG);
        if (old == kEmpty)
            break;
        if ((old >> 32) == tag) {
            const int64_t ob = (int64_t)(old & 0xffffffffull);
            int eq = 1;
            for (int f = f0; f < f1 && eq; f++) {  // eq is the same in all lanes at the loop test
                const int64_t l = (int64_t)f * B + b, ol = (int64_t)f * B + ob;
                const int64_t o1 = offsets[l], len = offsets[l + 1] - o1, oo = offsets[ol];
                eq = (offsets[ol + 1] - oo) == len;
                if (eq)
                    for (int64_t t = s; t < len; t += SG)
                        if (values[o1 + t] != values[oo + t]) {
                            eq = 0;
                            break;
                        }
#pragma unroll
                for (int m = SG / 2; m > 0; m >>= 1)
                    eq &= __shfl_xor(eq, m, SG);
            }
            if (eq) {
                if (s == 0)
                    atomicMin(reinterpret_cast<unsigned long long *>(&tab[slot]), mine);
                break;
            }
        }
        slot = (slot + 1) & cap_mask;
    }
    if (s == 0)
        slot_of[item] = (int32_t)slot;
}

// Feature-level compaction of a grouped IKJT: list (f,b) is stored iff row b is the representative
// of its slot in f's group.  Pass 1 (NUMBER = false): per-block sums of (stored, stored * length).
// Pass 2 (NUMBER = true), after the scan of the block sums: positions of the stored lists.
template <bool NUMBER>
__global__ __launch_bounds__(kScanBlock) void k_group_compact(const int64_t *__restrict__ offsets,
                                                              int64_t B, int64_t n_lists, int F,
                                                              const int32_t *__restrict__ feat_group,
                                                              const int32_t *__restrict__ rep_g,
                                                              const int32_t *__restrict__ inverse_g,
                                                              int64_t *__restrict__ bs_cnt,
                                                              int64_t *__restrict__ bs_len,
                                                              int64_t *__restrict__ bs_head,
                                                              int32_t *__restrict__ src_of,
                                                              int64_t *__restrict__ u_offsets,
                                                              int64_t *__restrict__ feat_uoff,
                                                              int32_t *__restrict__ inverse_f,
                                                              int64_t *__restrict__ counts)
{
    const int64_t l = (int64_t)blockIdx.x * kScanBlock + threadIdx.x;
    int64_t first = 0, flen = 0, f = 0, b = -1, item = 0;
    if (l < n_lists) {
        f = l / B;
        b = l - f * B;
        item = (int64_t)feat_group[f] * B + b;
        if (rep_g[item] == b) {
            first = 1;
            flen = offsets[l + 1] - offsets[l];
        }
    }
    int64_t ea, eb, ic, ta, tb, tc;
    block_scan3(first, flen, -1, ea, eb, ic, ta, tb, tc);
    if (!NUMBER) {
        if (threadIdx.x == 0) {
            bs_cnt[blockIdx.x] = ta;
            bs_len[blockIdx.x] = tb;
            bs_head[blockIdx.x] = -1;
        }
        return;
    }
    if (l < n_lists) {
        const int64_t num = bs_cnt[blockIdx.x] + ea;
        const int64_t pos = bs_len[blockIdx.x] + eb;
        if (first) {
            u_offsets[num] = pos;
            src_of[num] = (int32_t)l;
        }
        if (b == 0)
            feat_uoff[f] = num;
        if (inverse_f)
            inverse_f[l] = inverse_g[item];
        if (l == n_lists - 1) {
            const int64_t U = num + first, M = pos + flen;
            u_offsets[U] = M;
            feat_uoff[F] = U;
            counts[0] = U;
            counts[1] = M;
        }
    }
}

__global__ void k_empty_grouped(int F, int G, int64_t *u_offsets, int64_t *feat_uoff, int64_t *group_uoff,
                                int64_t *counts, int64_t *counts_g)
{
    for (int f = threadIdx.x; f <= F; f += blockDim.x)
        feat_uoff[f] = 0;
    for (int g = threadIdx.x; g <= G; g += blockDim.x)
        group_uoff[g] = 0;
    if (threadIdx.x == 0) {
        u_offsets[0] = 0;
        counts[0] = counts[1] = 0;
        counts_g[0] = counts_g[1] = 0;
    }
}

// ---- partial IKJT (Sec. 7 "Supporting Partial IKJTs") ------------------------------------------
// The slots are the IKJT's (same duplicates, same first-occurrence numbering); what changes is the
// storage: a slot whose first row directly follows a row holding the previous slot's list may
// continue that list - with k the largest overlap of the previous list's tail and the new list's
// head, only the remaining ids are stored and the slot's window starts k ids before the old end.
//
// One wave per slot: the ids to store (list length minus overlap).  Candidate overlaps are the
// positions of the new list's first id in the previous list, tried from the largest overlap down;
// each is verified by the whole wave.
__global__ __launch_bounds__(256) void k_partial_overlap(const int64_t *__restrict__ values,
                                                         const int64_t *__restrict__ offsets, int64_t B,
                                                         const int32_t *__restrict__ src_of,
                                                         const int32_t *__restrict__ inverse,
                                                         const int64_t *__restrict__ feat_uoff,
                                                         const int64_t *__restrict__ counts,
                                                         int64_t *__restrict__ win_len,
                                                         int32_t *__restrict__ piece)
{
    const int lane = threadIdx.x & 63;
    const int64_t U = counts[0];
    const int64_t stride = (int64_t)gridDim.x * 4;
    for (int64_t u = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6); u < U; u += stride) {
        const int64_t l = src_of[u];
        const int64_t f = l / B, b = l - f * B;
        const int64_t sb = offsets[l], len = offsets[l + 1] - sb;
        int64_t k = 0;
        const int64_t first_slot = feat_uoff[f];
        if (b > 0 && u > first_slot && (int64_t)inverse[l - 1] == u - 1 - first_slot && len > 0) {
            const int64_t lt = src_of[u - 1];
            const int64_t st = offsets[lt], len_t = offsets[lt + 1] - st;
            const int64_t kmax = len_t < len ? len_t : len;
            const int64_t head = values[sb];
            for (int64_t p0 = len_t - kmax; p0 < len_t && k == 0; p0 += 64) {
                const int64_t p = p0 + lane;
                uint64_t cand = __ballot(p < len_t && values[st + p] == head);
                while (cand != 0 && k == 0) {
                    const int64_t pc = p0 + __builtin_ctzll(cand);
                    cand &= cand - 1;
                    const int64_t kk = len_t - pc;  // overlap if the previous list's tail matches
                    bool ok = true;
                    for (int64_t i = lane; i < kk && ok; i += 64)
                        ok = values[st + pc + i] == values[sb + i];
                    if (__ballot(!ok) == 0)
                        k = kk;
                }
            }
        }
        if (lane == 0) {
            win_len[u] = len;
            piece[u] = (int32_t)(len - k);
        }
    }
}

// Positions of the stored pieces: exclusive scan of piece[] over the slots (pass 1: block sums;
// pass 2, after k_scan_blocks: window starts, per-feature prefix, total).
template <bool APPLY>
__global__ __launch_bounds__(kScanBlock) void k_partial_scan(const int32_t *__restrict__ piece,
                                                             const int64_t *__restrict__ win_len,
                                                             const int32_t *__restrict__ src_of, int64_t B,
                                                             int F, const int64_t *__restrict__ feat_uoff,
                                                             int64_t *__restrict__ counts,
                                                             int64_t *__restrict__ bs_cnt,
                                                             int64_t *__restrict__ bs_len,
                                                             int64_t *__restrict__ bs_head,
                                                             int64_t *__restrict__ piece_pos,
                                                             int64_t *__restrict__ win_start,
                                                             int64_t *__restrict__ feat_poff)
{
    const int64_t U = counts[0];
    const int64_t u = (int64_t)blockIdx.x * kScanBlock + threadIdx.x;
    const int64_t pc = u < U ? piece[u] : 0;
    int64_t ea, eb, ic, ta, tb, tc;
    block_scan3(pc, 0, -1, ea, eb, ic, ta, tb, tc);
    if (!APPLY) {
        if (threadIdx.x == 0) {
            bs_cnt[blockIdx.x] = ta;
            bs_len[blockIdx.x] = 0;
            bs_head[blockIdx.x] = -1;
        }
        return;
    }
    if (u < U) {
        const int64_t pos = bs_cnt[blockIdx.x] + ea;  // where this slot's piece is stored
        piece_pos[u] = pos;
        win_start[u] = pos + pc - win_len[u];
        const int64_t f = (int64_t)src_of[u] / B;
        if (u == feat_uoff[f])
            feat_poff[f] = pos;
        if (u == U - 1) {
            feat_poff[F] = pos + pc;
            counts[2] = pos + pc;
        }
    }
}

// Copies every slot's piece (the tail of its first row's list) and writes the per-row windows.
template <int SG>
__global__ __launch_bounds__(256) void k_partial_emit(const int64_t *__restrict__ values,
                                                      const int64_t *__restrict__ offsets, int64_t B,
                                                      int64_t n_lists, const int32_t *__restrict__ src_of,
                                                      const int32_t *__restrict__ piece,
                                                      const int64_t *__restrict__ piece_pos,
                                                      const int64_t *__restrict__ win_start,
                                                      const int64_t *__restrict__ win_len,
                                                      const int32_t *__restrict__ inverse,
                                                      const int64_t *__restrict__ feat_uoff,
                                                      const int64_t *__restrict__ counts,
                                                      int64_t *__restrict__ p_values,
                                                      int64_t *__restrict__ row_window, unsigned row_blocks)
{
    if (blockIdx.x < row_blocks) {
        const int64_t l = (int64_t)blockIdx.x * 256 + threadIdx.x;
        if (l < n_lists) {
            const int64_t u = feat_uoff[l / B] + inverse[l];
            row_window[2 * l] = win_start[u];
            row_window[2 * l + 1] = win_len[u];
        }
        return;
    }
    const int s = threadIdx.x % SG;
    const int64_t U = counts[0];
    const int64_t stride = (int64_t)(gridDim.x - row_blocks) * (256 / SG);
    for (int64_t u = (int64_t)(blockIdx.x - row_blocks) * (256 / SG) + threadIdx.x / SG; u < U;
         u += stride) {
        const int64_t l = src_of[u];
        const int64_t n = piece[u];
        const int64_t src = offsets[l + 1] - n;  // the last n ids of the list
        const int64_t dst = piece_pos[u];
        for (int64_t t = s; t < n; t += SG)
            p_values[dst + t] = values[src + t];
    }
}

__global__ void k_empty_partial(int F, int64_t *feat_uoff, int64_t *feat_poff, int64_t *counts)
{
    for (int f = threadIdx.x; f <= F; f += blockDim.x) {
        feat_uoff[f] = 0;
        feat_poff[f] = 0;
    }
    if (threadIdx.x == 0)
        counts[0] = counts[1] = counts[2] = 0;
}

// ---- run index of an IKJT from its arrays alone ------------------------------------------------
// A run is a maximal block of adjacent rows of a feature that name the same slot; its head is row 0
// of the feature or a row whose predecessor names another slot.  The first row of a slot is the
// smallest of its run heads.
__global__ __launch_bounds__(256) void k_fill_i32(int32_t *p, int64_t n, int32_t v)
{
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256)
        p[i] = v;
}

__global__ __launch_bounds__(256) void k_run_first(const int32_t *__restrict__ inverse,
                                                   const int64_t *__restrict__ feat_uoff, int64_t B,
                                                   int64_t n_rows, int32_t *__restrict__ first_row)
{
    const int64_t l = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (l >= n_rows)
        return;
    const int64_t f = l / B;
    const int32_t inv = inverse[l];
    if (l - f * B != 0 && inverse[l - 1] == inv)
        return;
    atomicMin(&first_row[feat_uoff[f] + inv], (int32_t)l);
}

// EMIT = false: per-block counts of run heads.  EMIT = true, after the scan of the block counts:
// the entries {row | (unique list, first-occurrence flag) << 32, ids at, ids}, the header
// {runs, U, M} and the closing entry.
template <bool EMIT>
__global__ __launch_bounds__(kScanBlock) void k_run_entries(const int32_t *__restrict__ inverse,
                                                            const int64_t *__restrict__ feat_uoff,
                                                            const int64_t *__restrict__ u_offsets, int64_t B,
                                                            int64_t n_rows, int F,
                                                            const int32_t *__restrict__ first_row,
                                                            int64_t *__restrict__ bs_cnt,
                                                            int64_t *__restrict__ bs_len,
                                                            int64_t *__restrict__ bs_head,
                                                            int64_t *__restrict__ run_index)
{
    const int64_t l = (int64_t)blockIdx.x * kScanBlock + threadIdx.x;
    int64_t head = 0, f = 0;
    int32_t inv = 0;
    if (l < n_rows) {
        f = l / B;
        inv = inverse[l];
        head = (l - f * B == 0 || inverse[l - 1] != inv) ? 1 : 0;
    }
    int64_t ea, eb, ic, ta, tb, tc;
    block_scan3(head, 0, -1, ea, eb, ic, ta, tb, tc);
    if (!EMIT) {
        if (threadIdx.x == 0) {
            bs_cnt[blockIdx.x] = ta;
            bs_len[blockIdx.x] = 0;
            bs_head[blockIdx.x] = -1;
        }
        return;
    }
    if (l < n_rows) {
        const int64_t r = bs_cnt[blockIdx.x] + ea;
        if (head) {
            const int64_t u = feat_uoff[f] + inv;
            int64_t *e = run_index + 3 * (1 + r);
            const uint32_t uf = (uint32_t)u | (first_row[u] == (int32_t)l ? 0x80000000u : 0u);
            e[0] = (int64_t)(((uint64_t)uf << 32) | (uint32_t)l);
            e[1] = u_offsets[u];
            e[2] = u_offsets[u + 1] - u_offsets[u];
        }
        if (l == n_rows - 1) {
            const int64_t n_runs = r + head, U = feat_uoff[F], M = u_offsets[U];
            run_index[0] = n_runs;
            run_index[1] = U;
            run_index[2] = M;
            run_index[3 * (1 + n_runs)] = n_rows;
            run_index[3 * (1 + n_runs) + 1] = M;
            run_index[3 * (1 + n_runs) + 2] = 0;
        }
    }
}

uint64_t table_cap(int64_t B)
{
    uint64_t cap = 64;
    while (cap < 2 * (uint64_t)B)
        cap <<= 1;
    return cap;
}

} // namespace

size_t recd_build_workspace(int F, int64_t B)
{
    // Covers the three builders (plain, grouped with up to F groups, partial): the hash table, seven
    // int32 and three int64 arrays of one entry per list, the block sums and the small maps, each
    // rounded up to the carver's 256-byte pieces.
    const int64_t n_lists = (int64_t)F * B;
    const int64_t nblk = (n_lists + kScanBlock - 1) / kScanBlock;
    size_t bytes = 0;
    bytes += (size_t)F * table_cap(B) * sizeof(uint64_t);
    bytes += 7 * ((size_t)n_lists * sizeof(int32_t) + 256);
    bytes += 3 * ((size_t)(n_lists + 1) * sizeof(int64_t) + 256);
    bytes += 3 * ((size_t)(nblk + 1) * sizeof(int64_t) + 256);
    bytes += 2 * ((size_t)(F + 2) * sizeof(int64_t) + 256);
    bytes += 16 * 256;
    return bytes;
}

namespace {

// Workspace of the slot search: hash table, per-item slot / representative / number / first row of
// every slot, block sums of the scans.  `items` = lists (features x B) or group rows (groups x B).
struct SlotWs {
    int64_t *counts;
    uint64_t *table;
    uint64_t cap;
    int32_t *slot_of, *rep, *number, *src_of, *hrank;
    int64_t *bs_cnt, *bs_len, *bs_head;
};

SlotWs carve_slots(WsCarver &c, int tables, int64_t B, int64_t items, int64_t scan_items)
{
    SlotWs w;
    const int64_t nblk = (scan_items + kScanBlock - 1) / kScanBlock;
    w.cap = table_cap(B);
    w.counts = c.take<int64_t>(4);
    w.table = c.take<uint64_t>((size_t)tables * w.cap);
    w.slot_of = c.take<int32_t>(items);
    w.rep = c.take<int32_t>(items);
    w.number = c.take<int32_t>(items);
    w.src_of = c.take<int32_t>(items);
    w.hrank = c.take<int32_t>(items);
    w.bs_cnt = c.take<int64_t>(nblk + 1);
    w.bs_len = c.take<int64_t>(nblk + 1);
    w.bs_head = c.take<int64_t>(nblk + 1);
    return w;
}

void clear_table(hipStream_t st, const SlotWs &w, int tables)
{
    const int64_t tab_n = (int64_t)tables * (int64_t)w.cap;
    const int fill_blocks = (int)((tab_n + 1023) / 1024 < 4096 ? (tab_n + 1023) / 1024 : 4096);
    hipLaunchKernelGGL(k_fill_u64, dim3(fill_blocks), dim3(256), 0, st, w.table, tab_n, kEmpty);
}

// Lists of a KJT into the per-feature tables: slot_of[l] (or -1 for a follower).
void insert_lists(recd_ctx *ctx, hipStream_t st, const SlotWs &w, int F, int64_t B,
                  const int64_t *values, const int64_t *offsets, const uint32_t *wbits = nullptr,
                  bool table_is_empty = false)
{
    constexpr int SG = 8;
    const int64_t n_lists = (int64_t)F * B;
    if (!table_is_empty)
        clear_table(st, w, F);
    int64_t hblocks = (n_lists + (kHashBlock / SG) * kLPG - 1) / ((kHashBlock / SG) * kLPG);
    hblocks = (hblocks + 7) / 8 * 8;  // the kernel deals its blocks to 8 XCDs
    recd_time_begin(ctx, RECD_T_HASH, st);
    if (wbits)
        hipLaunchKernelGGL((k_hash_insert<SG, true>), dim3((unsigned)hblocks), dim3(kHashBlock), 0, st, values, wbits,
                           offsets, B, n_lists, w.table, (uint32_t)(w.cap - 1), w.slot_of, ctx->weak_hash);
    else
        hipLaunchKernelGGL((k_hash_insert<SG, false>), dim3((unsigned)hblocks), dim3(kHashBlock), 0, st, values, wbits,
                           offsets, B, n_lists, w.table, (uint32_t)(w.cap - 1), w.slot_of, ctx->weak_hash);
    recd_time_end(ctx, RECD_T_HASH, st);
}

// After the insertion: representative and first-occurrence number of every item, first row of
// every slot, prefix of the slot counts per table (uoff) and, from the lengths that `offsets`
// gives, the position of every slot's ids (u_off); counts = {slots, ids}.
void number_slots(hipStream_t st, const SlotWs &w, int tables, int64_t B, const int64_t *offsets,
                  int64_t *u_off, int64_t *uoff, int64_t *mailbox = nullptr, int64_t seq = 0,
                  int64_t *run_index = nullptr)
{
    const int64_t n = (int64_t)tables * B;
    const unsigned nblk = (unsigned)((n + kScanBlock - 1) / kScanBlock);
    const uint32_t mask = (uint32_t)(w.cap - 1);
    hipLaunchKernelGGL(k_flags, dim3(nblk), dim3(kScanBlock), 0, st, offsets, B, n, w.table, mask, w.slot_of,
                       w.bs_cnt, w.bs_len, w.bs_head);
    hipLaunchKernelGGL(k_number, dim3(nblk), dim3(kScanBlock), 0, st, offsets, B, n, tables, w.table, mask,
                       w.slot_of, w.bs_cnt, w.bs_len, w.bs_head, w.rep, w.number, w.src_of, u_off, uoff,
                       w.counts, mailbox, seq, run_index ? w.hrank : nullptr, run_index);
}

unsigned copy_blocks_for(const recd_ctx *ctx, int64_t n_lists)
{
    int64_t b = (n_lists + (256 / 16) - 1) / (256 / 16);
    if (b > (int64_t)ctx->num_cu * 8)
        b = (int64_t)ctx->num_cu * 8;
    return (unsigned)b;
}

} // namespace


// weights / u_weights: null for a plain KJT
static recd_status build_plain(recd_ctx *ctx, int F, int64_t B, int64_t N, const int64_t *values,
                               const uint32_t *weights, const int64_t *offsets, int64_t *u_values,
                               uint32_t *u_weights, int64_t *u_offsets, int32_t *inverse,
                               int64_t *feat_uoff, int64_t *host_U_M, int64_t *run_index = nullptr)
{
    if (!ctx)
        return RECD_EINVAL;
    if (F < 0 || F > RECD_MAX_FEATURES || B < 0 || N < 0)
        return recd_fail(ctx, RECD_EINVAL, "bad sizes F=%d B=%lld N=%lld", F, (long long)B, (long long)N);
    const int64_t n_lists = (int64_t)F * B;
    if (n_lists >= (int64_t)1 << 31 || B >= (int64_t)1 << 30)
        return recd_fail(ctx, RECD_EINVAL, "F*B must stay below 2^31");
    if (!u_offsets || !feat_uoff || (n_lists > 0 && (!offsets || !inverse)) ||
        (N > 0 && (!values || !u_values)))
        return recd_fail(ctx, RECD_EINVAL, "null pointer argument");
    RECD_HIP(ctx, hipSetDevice(ctx->device));
    if (ctx->validate && n_lists > 0)
        RECD_TRY(recd_validate_kjt_offsets(ctx, F, B, N, offsets));

    if (ctx->small_path && !weights && n_lists > 0 && B <= kSmallB && F <= RECD_SMALL_MAX_FEATURES &&
        N <= kSmallIds && ctx->small_agg) {
        // one launch: a block per feature, tables in LDS
        hipStream_t st = ctx->stream;
        int64_t *mailbox = nullptr;
        int64_t seq = 0;
        if (!host_U_M && ctx->mailbox) {
            mailbox = ctx->mailbox_dev + 8;
            seq = ++ctx->build_seq;
        }
        uint32_t cap = 64;
        while (cap < 2 * (uint32_t)B)
            cap <<= 1;
        const int spin = ctx->small_path == 2 ? -1 : kSmallSpinLimit;
        const int sg = B * 8 <= kSmallThreads ? 8 : (B * 4 <= kSmallThreads ? 4 : (B * 2 <= kSmallThreads ? 2 : 1));
#define RECD_SMALL(SG)                                                                                              \
    hipLaunchKernelGGL((k_build_small<SG>), dim3((unsigned)F), dim3(kSmallThreads), 0, st, values, offsets, (int)B, F, \
                       cap - 1, ctx->weak_hash, spin, ctx->small_agg, u_values, u_offsets, inverse, feat_uoff,      \
                       ctx->build_counts_dev, mailbox, seq, run_index)
        if (sg == 8)
            RECD_SMALL(8);
        else if (sg == 4)
            RECD_SMALL(4);
        else if (sg == 2)
            RECD_SMALL(2);
        else
            RECD_SMALL(1);
#undef RECD_SMALL
        RECD_HIP(ctx, hipGetLastError());
        ctx->ws_used_since_build = false;
        ctx->build_valid = true;
        ctx->plan.valid = false;
        RECD_HIP(ctx, hipEventRecord(ctx->ev_built, st));
        ctx->built_inverse = inverse;
        ctx->built_u_values = u_values;
        if (host_U_M) {
            ctx->build_published = false;
            RECD_TRY(recd_fetch_scalars(ctx, ctx->build_counts_dev, 2, host_U_M));
            if (host_U_M[0] < 0)
                return recd_fail(ctx, RECD_EHIP, "the builder's blocks did not receive each other's counts in time");
        } else if (mailbox) {
            ctx->build_published = true;
            ctx->build_tagged = true;
        } else {
            RECD_TRY(recd_publish_build_counts(ctx));
        }
        return RECD_OK;
    }

    RECD_TRY(recd_reserve(ctx, recd_build_workspace(F, B)));
    ctx->ws_used_since_build = false;  // from here on: set again by the next workspace user
    WsCarver c(ctx->ws);
    SlotWs w = carve_slots(c, F, B, n_lists, n_lists);
    w.counts = ctx->build_counts_dev;  // {U, M}: outlives the workspace's reuse by later calls
    int64_t *counts = w.counts;
    hipStream_t st = ctx->stream;
    bool published = false;

    if (n_lists == 0) {
        hipLaunchKernelGGL(k_empty_ikjt, dim3(1), dim3(256), 0, st, F, u_offsets, feat_uoff, counts);
        if (run_index)  // no runs: the header and the closing entry, all zero
            hipLaunchKernelGGL(k_fill_u64, dim3(1), dim3(64), 0, st, reinterpret_cast<uint64_t *>(run_index),
                               (int64_t)6, 0ull);
    } else {
        // the context's own tables (kept empty between builds) instead of the workspace's
        const size_t slots = (size_t)F * w.cap;
        if (slots > ctx->build_table_slots) {
            RECD_HIP(ctx, hipStreamSynchronize(st));
            if (ctx->build_table)
                RECD_HIP(ctx, hipFree(ctx->build_table));
            ctx->build_table = nullptr;
            ctx->build_table_slots = 0;
            const size_t want = slots + slots / 4;
            void *tp = nullptr;
            if (hipMalloc(&tp, want * sizeof(uint64_t)) != hipSuccess) {
                (void)hipGetLastError();
                return recd_fail(ctx, RECD_ENOMEM, "hash tables of %zu bytes: allocation failed", want * sizeof(uint64_t));
            }
            ctx->build_table = static_cast<uint64_t *>(tp);
            ctx->build_table_slots = want;
            ctx->table_clean = false;
        }
        if (!ctx->table_clean) {
            const int64_t all = (int64_t)ctx->build_table_slots;
            hipLaunchKernelGGL(k_fill_u64, dim3(4096), dim3(256), 0, st, ctx->build_table, all, kEmpty);
        }
        w.table = ctx->build_table;
        ctx->table_clean = false;  // until this build's last kernel is enqueued
        insert_lists(ctx, st, w, F, B, values, offsets, weights, true);
        // without a host destination the counts go to the mailbox from the kernel that computes
        // them (no kernel of its own between the build and what the caller enqueues next)
        int64_t *mailbox = nullptr;
        int64_t seq = 0;
        if (!host_U_M && ctx->mailbox) {
            mailbox = ctx->mailbox_dev + 8;
            seq = ++ctx->build_seq;
            published = true;
        }
        number_slots(st, w, F, B, offsets, u_offsets, feat_uoff, mailbox, seq, run_index);
        const unsigned inv_blocks = (unsigned)((n_lists + 255) / 256);
        const unsigned fill_blocks = (unsigned)((slots + 4095) / 4096 < 2048 ? (slots + 4095) / 4096 : 2048);
        recd_time_begin(ctx, RECD_T_EMIT, st);
        hipLaunchKernelGGL((k_emit<16>), dim3(fill_blocks + inv_blocks + copy_blocks_for(ctx, n_lists)), dim3(256), 0,
                           st, values, offsets, B, n_lists, w.rep, w.number, w.src_of, u_offsets, counts,
                           u_values, inverse, inv_blocks, weights, u_weights, fill_blocks, ctx->build_table,
                           (int64_t)slots, w.hrank, run_index);
        recd_time_end(ctx, RECD_T_EMIT, st);
        RECD_HIP(ctx, hipGetLastError());
        ctx->table_clean = true;
    }
    RECD_HIP(ctx, hipGetLastError());
    ctx->build_valid = true;
    ctx->plan.valid = false;  // the builder reused the workspace a plan would live in
    RECD_HIP(ctx, hipEventRecord(ctx->ev_built, st));
    ctx->built_inverse = inverse;
    ctx->built_u_values = u_values;
    if (host_U_M) {
        ctx->build_published = false;  // fetched here; recd_last_ikjt_counts reads the device array
        RECD_TRY(recd_fetch_scalars(ctx, counts, 2, host_U_M));
    } else if (published) {
        ctx->build_published = true;
        ctx->build_tagged = false;
    } else {
        RECD_TRY(recd_publish_build_counts(ctx));  // the empty batch, or no mailbox
    }
    return RECD_OK;
}

extern "C" recd_status recd_build_ikjt(recd_ctx *ctx, int F, int64_t B, int64_t N,
                                       const int64_t *values, const int64_t *offsets,
                                       int64_t *u_values, int64_t *u_offsets, int32_t *inverse,
                                       int64_t *feat_uoff, int64_t *host_U_M)
{
    return build_plain(ctx, F, B, N, values, nullptr, offsets, u_values, nullptr, u_offsets, inverse, feat_uoff,
                       host_U_M);
}

// ---- allocation-free builder -------------------------------------------------------------------
// Scratch of recd_build_ikjt_noalloc: hash tables, per-list slot / representative / number / first
// row, block sums and counts for at most RECD_NOALLOC_MAX_LISTS lists.  One copy per GPU the library
// runs on, held until the process ends; every call on a GPU uses it (overlapping calls race).
namespace {
constexpr size_t kStaticTableSlots = 4 * (size_t)RECD_NOALLOC_MAX_LISTS;  // F * cap(B) <= max(64 F, 4 F B)
constexpr size_t kStaticScratchBytes =
    kStaticTableSlots * sizeof(uint64_t) + 5 * ((size_t)RECD_NOALLOC_MAX_LISTS * sizeof(int32_t) + 256) +
    3 * ((RECD_NOALLOC_MAX_LISTS / kScanBlock + 2) * sizeof(int64_t) + 256) + 2 * 256;
constexpr int kMaxDevices = 64;
char *g_scratch_ptr[kMaxDevices];  // device address of this GPU's copy of `scratch`
}
static __device__ __align__(256) char scratch[kStaticScratchBytes];

// The device address of the current device's copy of `scratch` (looked up once per device; the
// array's name itself is only a host-side stand-in).  Called with `device` current.
recd_status recd_static_scratch(recd_ctx *ctx, int device)
{
    if (device < 0 || device >= kMaxDevices)
        return recd_fail(ctx, RECD_EINVAL, "device %d: at most %d devices", device, kMaxDevices);
    char *p = __atomic_load_n(&g_scratch_ptr[device], __ATOMIC_ACQUIRE);
    if (!p) {
        void *sym = nullptr;
        RECD_HIP(ctx, hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch)));
        if (!sym)
            return recd_fail(ctx, RECD_EHIP, "hipGetSymbolAddress returned a null address");
        p = static_cast<char *>(sym);
        __atomic_store_n(&g_scratch_ptr[device], p, __ATOMIC_RELEASE);  // every thread finds the same address
    }
    ctx->static_scratch = p;
    return RECD_OK;
}

extern "C" recd_status recd_build_ikjt_noalloc(recd_ctx *ctx, int F, int64_t B, int64_t N,
                                               const int64_t *values, const int64_t *offsets,
                                               int64_t *u_values, int64_t *u_offsets, int32_t *inverse,
                                               int64_t *feat_uoff)
{
    if (!ctx)
        return RECD_EINVAL;
    if (F < 0 || F > RECD_MAX_FEATURES || B < 0 || N < 0)
        return recd_fail(ctx, RECD_EINVAL, "bad sizes F=%d B=%lld N=%lld", F, (long long)B, (long long)N);
    const int64_t n_lists = (int64_t)F * B;
    if (B > RECD_NOALLOC_MAX_LISTS || n_lists > RECD_NOALLOC_MAX_LISTS)
        return recd_fail(ctx, RECD_ECAPACITY, "F*B=%lld exceeds RECD_NOALLOC_MAX_LISTS=%d", (long long)n_lists,
                         RECD_NOALLOC_MAX_LISTS);
    if (!u_offsets || !feat_uoff || (n_lists > 0 && (!offsets || !inverse)) || (N > 0 && (!values || !u_values)))
        return recd_fail(ctx, RECD_EINVAL, "null pointer argument");
    if (!ctx->static_scratch)
        return recd_fail(ctx, RECD_EHIP, "the static scratch array was not found when the context was created");
    RECD_HIP(ctx, hipSetDevice(ctx->device));
    WsCarver c(ctx->static_scratch);
    const SlotWs w = carve_slots(c, F, B, n_lists, n_lists);
    if ((size_t)F * w.cap > kStaticTableSlots || c.off > kStaticScratchBytes)
        return recd_fail(ctx, RECD_ECAPACITY, "sizes exceed the static scratch array");
    hipStream_t st = ctx->stream;
    if (n_lists == 0) {
        hipLaunchKernelGGL(k_empty_ikjt, dim3(1), dim3(256), 0, st, F, u_offsets, feat_uoff, w.counts);
    } else {
        // the array keeps the last call's contents: the tables are cleared by a fill kernel first (no
        // memset, so that the call can be captured into a graph); every other piece is written
        // before it is read
        insert_lists(ctx, st, w, F, B, values, offsets, nullptr, false);
        number_slots(st, w, F, B, offsets, u_offsets, feat_uoff);
        const unsigned inv_blocks = (unsigned)((n_lists + 255) / 256);
        hipLaunchKernelGGL((k_emit<16>), dim3(inv_blocks + copy_blocks_for(ctx, n_lists)), dim3(256), 0, st, values,
                           offsets, B, n_lists, w.rep, w.number, w.src_of, u_offsets, w.counts, u_values, inverse,
                           inv_blocks);
    }
    RECD_HIP(ctx, hipGetLastError());
    return RECD_OK;
}

extern "C" recd_status recd_build_ikjt_runs(recd_ctx *ctx, int F, int64_t B, int64_t N,
                                            const int64_t *values, const int64_t *offsets,
                                            int64_t *u_values, int64_t *u_offsets, int32_t *inverse,
                                            int64_t *feat_uoff, int64_t *run_index, int64_t *host_U_M)
{
    if (ctx && !run_index)
        return recd_fail(ctx, RECD_EINVAL, "null run_index");
    return build_plain(ctx, F, B, N, values, nullptr, offsets, u_values, nullptr, u_offsets, inverse, feat_uoff,
                       host_U_M, run_index);
}

extern "C" recd_status recd_ikjt_run_index(recd_ctx *ctx, int F, int64_t B, const int32_t *inverse,
                                           const int64_t *feat_uoff, const int64_t *u_offsets,
                                           int64_t *run_index)
{
    if (!ctx)
        return RECD_EINVAL;
    if (F < 0 || F > RECD_MAX_FEATURES || B < 0)
        return recd_fail(ctx, RECD_EINVAL, "bad sizes F=%d B=%lld", F, (long long)B);
    const int64_t n_rows = (int64_t)F * B;
    if (n_rows >= (int64_t)1 << 31)
        return recd_fail(ctx, RECD_EINVAL, "F*B must stay below 2^31");
    if (!run_index || (n_rows > 0 && (!inverse || !feat_uoff || !u_offsets)))
        return recd_fail(ctx, RECD_EINVAL, "null pointer argument");
    RECD_HIP(ctx, hipSetDevice(ctx->device));
    hipStream_t st = ctx->stream;
    if (n_rows == 0) {
        hipLaunchKernelGGL(k_fill_u64, dim3(1), dim3(64), 0, st, reinterpret_cast<uint64_t *>(run_index), (int64_t)6,
                           0ull);
        RECD_HIP(ctx, hipGetLastError());
        return RECD_OK;
    }
    if (ctx->validate)
        RECD_TRY(recd_validate_inverse(ctx, F, B, feat_uoff, inverse));
    const int64_t nblk = (n_rows + kScanBlock - 1) / kScanBlock;
    ctx->plan.valid = false;  // this call reuses the workspace a backward plan would live in
    RECD_TRY(recd_reserve(ctx, 1024 + (size_t)n_rows * sizeof(int32_t) + 3 * ((size_t)(nblk + 1) * sizeof(int64_t) + 256) + 1024));
    WsCarver c(ctx->ws);
    (void)c.take<char>(1024);  // the head of the workspace stays with the validation passes' flags
    int32_t *first_row = c.take<int32_t>(n_rows);
    int64_t *bs_cnt = c.take<int64_t>(nblk + 1), *bs_len = c.take<int64_t>(nblk + 1), *bs_head = c.take<int64_t>(nblk + 1);
    const unsigned rb = (unsigned)((n_rows + 255) / 256);
    hipLaunchKernelGGL(k_fill_i32, dim3(rb < 4096 ? rb : 4096), dim3(256), 0, st, first_row, n_rows, 0x7fffffff);
    hipLaunchKernelGGL(k_run_first, dim3(rb), dim3(256), 0, st, inverse, feat_uoff, B, n_rows, first_row);
    hipLaunchKernelGGL((k_run_entries<false>), dim3((unsigned)nblk), dim3(kScanBlock), 0, st, inverse, feat_uoff,
                       u_offsets, B, n_rows, F, first_row, bs_cnt, bs_len, bs_head, run_index);
    hipLaunchKernelGGL(k_scan_blocks, dim3(1), dim3(kScanBlock), 0, st, bs_cnt, bs_len, bs_head, nblk);
    hipLaunchKernelGGL((k_run_entries<true>), dim3((unsigned)nblk), dim3(kScanBlock), 0, st, inverse, feat_uoff,
                       u_offsets, B, n_rows, F, first_row, bs_cnt, bs_len, bs_head, run_index);
    RECD_HIP(ctx, hipGetLastError());
    return RECD_OK;
}

extern "C" recd_status recd_build_ikjt_weighted(recd_ctx *ctx, int F, int64_t B, int64_t N,
                                                const int64_t *values, const float *weights,
                                                const int64_t *offsets, int64_t *u_values,
                                                float *u_weights, int64_t *u_offsets, int32_t *inverse,
                                                int64_t *feat_uoff, int64_t *host_U_M)
{
    if (!ctx)
        return RECD_EINVAL;
    if (N > 0 && (!weights || !u_weights))
        return recd_fail(ctx, RECD_EINVAL, "null weights");
    // with no id there is no weight either: the plain builder
    return build_plain(ctx, F, B, N, values, N > 0 ? reinterpret_cast<const uint32_t *>(weights) : nullptr,
                       offsets, u_values, reinterpret_cast<uint32_t *>(u_weights), u_offsets, inverse,
                       feat_uoff, host_U_M);
}


extern "C" recd_status recd_build_ikjt_grouped(recd_ctx *ctx, int F, int64_t B, int64_t N, int G,
                                               const int32_t *group_off, const int64_t *values,
                                               const int64_t *offsets, int64_t *u_values,
                                               int64_t *u_offsets, int32_t *inverse_g,
                                               int64_t *group_uoff, int64_t *feat_uoff,
                                               int32_t *inverse_per_feature, int64_t *host_counts)
{
    if (!ctx)
        return RECD_EINVAL;
    if (F < 0 || F > RECD_MAX_FEATURES || B < 0 || N < 0 || G < 0 || G > F)
        return recd_fail(ctx, RECD_EINVAL, "bad sizes F=%d B=%lld N=%lld G=%d", F, (long long)B,
                         (long long)N, G);
    if (!group_off || group_off[0] != 0 || group_off[G] != F)
        return recd_fail(ctx, RECD_EINVAL, "group_off must run from 0 to F");
    for (int g = 0; g < G; g++)
        if (group_off[g + 1] <= group_off[g])
            return recd_fail(ctx, RECD_EINVAL, "group %d is empty or group_off decreases", g);
    const int64_t n_lists = (int64_t)F * B, n_items = (int64_t)G * B;
    if (n_lists >= (int64_t)1 << 31 || B >= (int64_t)1 << 30)
        return recd_fail(ctx, RECD_EINVAL, "F*B must stay below 2^31");
    if (!u_offsets || !feat_uoff || !group_uoff || (n_lists > 0 && (!offsets || !inverse_g)) ||
        (N > 0 && (!values || !u_values)))
        return recd_fail(ctx, RECD_EINVAL, "null pointer argument");
    RECD_HIP(ctx, hipSetDevice(ctx->device));
    if (ctx->validate && n_lists > 0)
        RECD_TRY(recd_validate_kjt_offsets(ctx, F, B, N, offsets));

    ctx->plan.valid = false;  // this call reuses the workspace a backward plan would live in
    RECD_TRY(recd_reserve(ctx, recd_build_workspace(F, B)));
    WsCarver c(ctx->ws);
    const SlotWs w = carve_slots(c, G, B, n_items, n_lists);  // slots of the group rows
    int64_t *counts = c.take<int64_t>(4);                      // stored lists, stored ids
    int32_t *src_of = c.take<int32_t>(n_lists);
    int64_t *zero_off = c.take<int64_t>(n_items + 1);
    int64_t *u_tmp = c.take<int64_t>(n_items + 1);
    hipStream_t st = ctx->stream;
    if (n_lists == 0) {
        hipLaunchKernelGGL(k_empty_grouped, dim3(1), dim3(256), 0, st, F, G, u_offsets, feat_uoff,
                           group_uoff, counts, w.counts);
    } else {
        const int32_t *dev_group_off = nullptr, *dev_feat_group = nullptr;
        RECD_TRY(recd_group_map(ctx, F, G, group_off, &dev_group_off, &dev_feat_group));
        constexpr int SG = 8;
        clear_table(st, w, G);
        const int zero_blocks = (int)((n_items + 1 + 1023) / 1024 < 4096 ? (n_items + 1 + 1023) / 1024 : 4096);
        hipLaunchKernelGGL(k_fill_u64, dim3(zero_blocks), dim3(256), 0, st,
                           reinterpret_cast<uint64_t *>(zero_off), n_items + 1, 0ull);
        const int64_t hblocks = (n_items + (256 / SG) - 1) / (256 / SG);
        hipLaunchKernelGGL((k_group_hash_insert<SG>), dim3((unsigned)hblocks), dim3(256), 0, st, values,
                           offsets, B, n_items, dev_group_off, w.table, (uint32_t)(w.cap - 1), w.slot_of,
                           ctx->weak_hash);
        // numbering of the slots per group: the list-level kernels with the groups in the role of
        // features and lists of length zero
        number_slots(st, w, G, B, zero_off, u_tmp, group_uoff);
        const unsigned inv_blocks = (unsigned)((n_items + 255) / 256);
        hipLaunchKernelGGL((k_emit<16>), dim3(inv_blocks), dim3(256), 0, st, values, zero_off, B, n_items,
                           w.rep, w.number, w.src_of, u_tmp, w.counts, u_values, inverse_g, inv_blocks);
        // per feature: which lists are stored, where
        const int64_t nblk = (n_lists + kScanBlock - 1) / kScanBlock;
        hipLaunchKernelGGL((k_group_compact<false>), dim3((unsigned)nblk), dim3(kScanBlock), 0, st, offsets,
                           B, n_lists, F, dev_feat_group, w.rep, inverse_g, w.bs_cnt, w.bs_len, w.bs_head,
                           src_of, u_offsets, feat_uoff, inverse_per_feature, counts);
        hipLaunchKernelGGL(k_scan_blocks, dim3(1), dim3(kScanBlock), 0, st, w.bs_cnt, w.bs_len, w.bs_head,
                           nblk);
        hipLaunchKernelGGL((k_group_compact<true>), dim3((unsigned)nblk), dim3(kScanBlock), 0, st, offsets,
                           B, n_lists, F, dev_feat_group, w.rep, inverse_g, w.bs_cnt, w.bs_len, w.bs_head,
                           src_of, u_offsets, feat_uoff, inverse_per_feature, counts);
        hipLaunchKernelGGL((k_emit<16>), dim3(copy_blocks_for(ctx, n_lists)), dim3(256), 0, st, values,
                           offsets, B, n_lists, w.rep, w.number, src_of, u_offsets, counts, u_values,
                           inverse_g, 0u);
    }
    RECD_HIP(ctx, hipGetLastError());
    if (host_counts) {
        // counts = {stored lists, stored ids}, w.counts[0] = sum of the groups' slot counts; the
        // two live next to each other in the workspace only by way of this copy
        hipLaunchKernelGGL(k_copy_i64, dim3(1), dim3(1), 0, st, w.counts, counts + 2);
        RECD_TRY(recd_fetch_scalars(ctx, counts, 3, host_counts));
    }
    return RECD_OK;
}


extern "C" recd_status recd_build_partial_ikjt(recd_ctx *ctx, int F, int64_t B, int64_t N,
                                               const int64_t *values, const int64_t *offsets,
                                               int64_t *p_values, int64_t *win_start, int64_t *win_len,
                                               int32_t *inverse, int64_t *feat_uoff, int64_t *feat_poff,
                                               int64_t *row_window, int64_t *host_counts)
{
    if (!ctx)
        return RECD_EINVAL;
    if (F < 0 || F > RECD_MAX_FEATURES || B < 0 || N < 0)
        return recd_fail(ctx, RECD_EINVAL, "bad sizes F=%d B=%lld N=%lld", F, (long long)B, (long long)N);
    const int64_t n_lists = (int64_t)F * B;
    if (n_lists >= (int64_t)1 << 31 || B >= (int64_t)1 << 30 || N >= (int64_t)1 << 31)
        return recd_fail(ctx, RECD_EINVAL, "F*B and N must stay below 2^31");
    if (!feat_uoff || !feat_poff || (n_lists > 0 && (!offsets || !inverse || !win_start || !win_len)) ||
        (N > 0 && (!values || !p_values)))
        return recd_fail(ctx, RECD_EINVAL, "null pointer argument");
    RECD_HIP(ctx, hipSetDevice(ctx->device));
    if (ctx->validate && n_lists > 0)
        RECD_TRY(recd_validate_kjt_offsets(ctx, F, B, N, offsets));

    const int64_t nblk = (n_lists + kScanBlock - 1) / kScanBlock;
    ctx->plan.valid = false;  // this call reuses the workspace a backward plan would live in
    RECD_TRY(recd_reserve(ctx, recd_build_workspace(F, B)));
    WsCarver c(ctx->ws);
    const SlotWs w = carve_slots(c, F, B, n_lists, n_lists);
    int64_t *counts = w.counts;  // [0] slots, [1] ids of an IKJT, [2] ids stored
    int32_t *piece = c.take<int32_t>(n_lists);
    int64_t *u_off = c.take<int64_t>(n_lists + 1);
    int64_t *piece_pos = c.take<int64_t>(n_lists);
    int32_t *src_of = w.src_of;
    int64_t *bs_cnt = w.bs_cnt, *bs_len = w.bs_len, *bs_head = w.bs_head;
    hipStream_t st = ctx->stream;
    if (n_lists == 0) {
        hipLaunchKernelGGL(k_empty_partial, dim3(1), dim3(256), 0, st, F, feat_uoff, feat_poff, counts);
    } else {
        insert_lists(ctx, st, w, F, B, values, offsets);
        number_slots(st, w, F, B, offsets, u_off, feat_uoff);
        const unsigned inv_blocks = (unsigned)((n_lists + 255) / 256);
        hipLaunchKernelGGL((k_emit<16>), dim3(inv_blocks), dim3(256), 0, st, values, offsets, B, n_lists,
                           w.rep, w.number, src_of, u_off, counts, p_values, inverse, inv_blocks);
        int64_t ov_blocks = (n_lists + 3) / 4;
        if (ov_blocks > (int64_t)ctx->num_cu * 16)
            ov_blocks = (int64_t)ctx->num_cu * 16;
        hipLaunchKernelGGL(k_partial_overlap, dim3((unsigned)ov_blocks), dim3(256), 0, st, values, offsets,
                           B, src_of, inverse, feat_uoff, counts, win_len, piece);
        hipLaunchKernelGGL((k_partial_scan<false>), dim3((unsigned)nblk), dim3(kScanBlock), 0, st, piece,
                           win_len, src_of, B, F, feat_uoff, counts, bs_cnt, bs_len, bs_head, piece_pos,
                           win_start, feat_poff);
        hipLaunchKernelGGL(k_scan_blocks, dim3(1), dim3(kScanBlock), 0, st, bs_cnt, bs_len, bs_head,
                           nblk);
        hipLaunchKernelGGL((k_partial_scan<true>), dim3((unsigned)nblk), dim3(kScanBlock), 0, st, piece,
                           win_len, src_of, B, F, feat_uoff, counts, bs_cnt, bs_len, bs_head, piece_pos,
                           win_start, feat_poff);
        const unsigned row_blocks = row_window ? inv_blocks : 0u;
        hipLaunchKernelGGL((k_partial_emit<16>), dim3(row_blocks + copy_blocks_for(ctx, n_lists)), dim3(256), 0,
                           st, values, offsets, B, n_lists, src_of, piece, piece_pos, win_start, win_len,
                           inverse, feat_uoff, counts, p_values, row_window, row_blocks);
    }
    RECD_HIP(ctx, hipGetLastError());
    if (host_counts) {
        int64_t h[3];
        RECD_TRY(recd_fetch_scalars(ctx, counts, 3, h));
        host_counts[0] = h[0];  // U
        host_counts[1] = h[2];  // P: ids stored
        host_counts[2] = h[1];  // M: ids an IKJT would store
    }
    return RECD_OK;
}
