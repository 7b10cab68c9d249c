// Stage 2: centroid interaction with centroid pruning (Eq. 3-5) over every candidate passage.
//
// A passage's pruned score is sum_i max_j S_cq[code_j][i] over its tokens whose centroid passes
// Eq. 5, so it depends only on WHICH surviving centroids occur in the passage.  Few centroids
// survive t_cs (a small tail of high scores, Section 3.4), so the work splits in two:
//
//   streaming part   the candidates' token codes are read once, coalesced, straight from HBM
//                    (128-byte lines that no candidate touches are skipped); each code is looked
//                    up in a small LDS table of the K surviving centroids and turned into a slot
//                    number; one lane per passage then folds its slots into a K-bit set;
//   scoring part     the lane takes the column maxima of the <= K surviving rows named by the
//                    set (rows staged in LDS) and sums the 32 maxima in double, in index order.
//
// No matrix D~ is ever stacked (Section 4.5's padding-free idea), nothing is padded, and the
// order-independent max plus the fixed-order sum make a score a pure function of the passage.
// Queries with more than S2_MAX_KEPT surviving centroids (very low thresholds) take the gather
// form instead: one wave per passage fetching surviving rows from the L2-resident S_cq.
//
// Output of either form, per query: slot p of the key array holds the ranking key of candidate p
// when its bag is non-empty and the invalid key otherwise (slots of non-candidates are neither
// written nor read), a histogram of the valid keys' bins for the selection that follows, and a
// bitmap of the candidates whose bag is empty (score -infinity; they rank last, in passage-id
// order).  A query without any surviving centroid skips all of this: its candidates are exactly
// its empty-bag set.  No counters and no atomics with a return value on this path; a workgroup counts bins
// in LDS and adds its non-zero bins to the query's histogram once, at its end, so that queries
// whose passages all share one score (a single surviving centroid) do not queue up on one address.
#include "plaid_internal.h"

#include <math.h>

#define S2_THREADS 256
#define S2W_PASS 64      // passages per wave tile = 2 words of the candidate bitmap
#define S2_ITEMS 9       // 16-byte loads per lane and round, all in flight at once
#define S2W_CAP (64 * 4 * S2_ITEMS - 32)  // tokens a wave stages per round (one byte each), whatever their alignment
#define S2_LBWORDS ((S2_ITEMS + 3) / 4)   // words of the round's line bitmap (8 lines per item)
#define S2_TSTRIDE 36    // floats per staged S_cq row (16-byte aligned, rows spread over the banks)
// Inverted form: a workgroup owns 2^SHIFT consecutive passages, SHIFT = 11 (256 threads) for indexes whose range table
// stays small at that granularity, 13 (1024 threads) for large ones; both are instances of one kernel template.
#define IVR_THREADS(SHIFT) (256 << ((SHIFT) - 11))
static_assert(S2_LBWORDS <= 64, "one lane clears one word of the line bitmap");

// ------------------------------------------------------------------ gather form (K > S2_MAX_KEPT)
// Pruned score of the passage with tokens [t0, t1): uniform across the wave; `any` tells whether a token survived.
__device__ __forceinline__ float s2_gather_passage(const float *__restrict__ Sq, const uint32_t *__restrict__ kb,
                                                   int64_t t0, int64_t t1, const int32_t *__restrict__ codes, int lane,
                                                   bool &any)
{
    const int i = lane & 31, h = lane >> 5;
    float m = -INFINITY;
    any = false;
    for (int64_t base = t0; base < t1; base += 64) {
        const int cnt = t1 - base < 64 ? (int)(t1 - base) : 64;
        const int32_t code = lane < cnt ? codes[base + lane] : 0;
        bool hit = lane < cnt;
        if (hit) hit = (kb[code >> 5] >> (code & 31)) & 1u;
        unsigned long long mask = __ballot(hit);
        any = any || mask != 0;
        while (mask) {
            const int j0 = __ffsll((long long)mask) - 1;
            mask &= mask - 1;
            int j1 = j0;
            if (mask) {
                j1 = __ffsll((long long)mask) - 1;
                mask &= mask - 1;
            }
            const int c = __shfl(code, h ? j1 : j0);
            m = fmaxf(m, Sq[(int64_t)c * QLEN + i]);
        }
    }
    m = fmaxf(m, __shfl_xor(m, 32));
    return plaid_sum32_in_order(m);
}

// Body for one query over the bitmap words w_first + k * w_step < w_end (32 passages each), one wave per word at a
// time; cb[w - cb_first] is the candidate word w (global memory or LDS).
__device__ __forceinline__ void s2_gather_body(int q, const float *__restrict__ S, int64_t C,
                                               const uint32_t *__restrict__ keepbits, int64_t keep_words, const uint32_t *cb,
                                               int64_t cb_first, int64_t w_first, int64_t w_step, int64_t w_end,
                                               int64_t cand_words, int64_t P, const int64_t *__restrict__ doc_offsets,
                                               const int32_t *__restrict__ codes, float bin_hi, float bin_scale,
                                               uint32_t *__restrict__ keys_out, int32_t *lhist,
                                               uint32_t *__restrict__ emptybits)
{
    const int lane = threadIdx.x & 63;
    const float *Sq = S + (int64_t)q * C * QLEN;
    const uint32_t *kb = keepbits + (int64_t)q * keep_words;
    uint32_t *eb = emptybits + (int64_t)q * cand_words;
    for (int64_t w = w_first; w < w_end; w += w_step) {
        const uint32_t word = cb[w - cb_first];
        if (!word) {
            if (lane == 0) eb[w] = 0u;
            continue;
        }
        const int64_t p0 = w * 32;
        int64_t off = 0;
        if (lane <= 32 && p0 + lane <= P) off = doc_offsets[p0 + lane];
        float my = -INFINITY;
        bool my_empty = false;
        uint32_t rest = word;
        while (rest) {
            const int b = __ffs(rest) - 1;
            rest &= rest - 1;
            const int64_t t0 = __shfl(off, b), t1 = __shfl(off, b + 1);
            bool any;
            const float sc = s2_gather_passage(Sq, kb, t0, t1, codes, lane, any);
            if (lane == b) {
                my = sc;
                my_empty = !any;
            }
        }
        const bool cand = lane < 32 && ((word >> lane) & 1u);
        const bool live = cand && !my_empty;
        if (cand) keys_out[p0 + lane] = live ? plaid_score_to_ord(my) : PLAID_S2_NO_SCORE;
        if (live) atomicAdd(&lhist[plaid_s2_bin(my, bin_hi, bin_scale)], 1);
        const unsigned long long e64 = __ballot(cand && my_empty);
        if (lane == 0) eb[w] = (uint32_t)e64;
    }
}

// ------------------------------------------------------------------ streaming form (K <= S2_MAX_KEPT)
// Survivor table entry: (centroid id << 6) | slot, 0xFFFFFFFF = free.  The hash is collision-free on the survivors,
// so one probe decides: returns the slot (1..63) of a surviving centroid, 0 otherwise.
__device__ __forceinline__ uint32_t s2_lookup(const uint32_t *htab, uint32_t code, int hash_shift)
{
    const uint32_t e = htab[(code ^ (code >> hash_shift)) & (S2_HASH - 1)] ^ (code << 6);
    return e < 64u ? e : 0u;
}

// LDS traffic between the lanes of one wave needs no workgroup barrier: a wave's LDS operations complete in
// program order.  This only stops the compiler from moving accesses across the hand-over point.
__device__ __forceinline__ void s2_wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Every value that steers control flow below is wave-uniform and is forced into scalar registers with
// readfirstlane, so that all cross-lane operations (__shfl, __ballot) run with the full wave active.
__device__ __forceinline__ int s2_uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }

// First set bit of m at position >= from, 64 when there is none (all operands uniform).
__device__ __forceinline__ int s2_next_bit(unsigned long long m, int from)
{
    const unsigned long long rest = from < 64 ? (m >> from) << from : 0ull;
    return rest ? __ffsll((long long)rest) - 1 : 64;
}

// End of a workgroup: its LDS bin counts go to the query's histogram (all threads of the workgroup call this).
__device__ __forceinline__ void s2_flush_hist(const int32_t *lhist, int32_t *__restrict__ hist_q)
{
    __syncthreads();
    for (int e = threadIdx.x; e < SEL_BINS; e += blockDim.x) {
        const int32_t n = lhist[e];
        if (n) atomicAdd(&hist_q[e], n);
    }
}

// Pruned score of a bag whose surviving centroids are the slots in `members` (non-empty, bit 0 clear): column maxima
// of those rows of the staged table, summed over the query tokens in index order; eight query tokens at a time, so
// that few registers are live.  A bag with one survivor takes that row's precomputed sum (same additions, same order).
__device__ __forceinline__ float s2_score_members(uint64_t members, const float *Tl, const float *rowsum)
{
    if ((members & (members - 1)) == 0) return rowsum[__ffsll((long long)members) - 1];
    double d = 0.0;
#pragma unroll 1
    for (int g = 0; g < QLEN / 8; ++g) {
        float acc[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = -INFINITY;
        uint64_t rest = members;
        while (rest) {
            const int s = __ffsll((long long)rest) - 1;
            rest &= rest - 1;
            const float4 *row = reinterpret_cast<const float4 *>(Tl + s * S2_TSTRIDE + 8 * g);
            const float4 r0 = row[0], r1 = row[1];
            acc[0] = fmaxf(acc[0], r0.x);
            acc[1] = fmaxf(acc[1], r0.y);
            acc[2] = fmaxf(acc[2], r0.z);
            acc[3] = fmaxf(acc[3], r0.w);
            acc[4] = fmaxf(acc[4], r1.x);
            acc[5] = fmaxf(acc[5], r1.y);
            acc[6] = fmaxf(acc[6], r1.z);
            acc[7] = fmaxf(acc[7], r1.w);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) d += (double)acc[i];
    }
    return (float)d;
}

// The same score with all 32 running maxima in registers and two rows folded per step: one pass over the members.
// For kernels with registers to spare; the additions are the same and in the same order as in s2_score_members.
__device__ __forceinline__ float s2_score_members_wide(uint64_t members, const float *Tl, const float *rowsum)
{
    if ((members & (members - 1)) == 0) return rowsum[__ffsll((long long)members) - 1];
    float acc[QLEN];
#pragma unroll
    for (int i = 0; i < QLEN; ++i) acc[i] = -INFINITY;
    uint64_t rest = members;
    while (rest) {
        const int s0 = __ffsll((long long)rest) - 1;
        rest &= rest - 1;
        int s1 = 0;  // row 0 holds -infinity: a neutral second operand when the member count is odd
        if (rest) {
            s1 = __ffsll((long long)rest) - 1;
            rest &= rest - 1;
        }
        const float4 *ra = reinterpret_cast<const float4 *>(Tl + s0 * S2_TSTRIDE);
        const float4 *rb = reinterpret_cast<const float4 *>(Tl + s1 * S2_TSTRIDE);
#pragma unroll
        for (int g = 0; g < QLEN / 4; ++g) {
            const float4 a = ra[g], b = rb[g];
            acc[4 * g] = fmaxf(acc[4 * g], fmaxf(a.x, b.x));
            acc[4 * g + 1] = fmaxf(acc[4 * g + 1], fmaxf(a.y, b.y));
            acc[4 * g + 2] = fmaxf(acc[4 * g + 2], fmaxf(a.z, b.z));
            acc[4 * g + 3] = fmaxf(acc[4 * g + 3], fmaxf(a.w, b.w));
        }
    }
    double d = 0.0;
#pragma unroll
    for (int i = 0; i < QLEN; ++i) d += (double)acc[i];
    return (float)d;
}

// The query's survivor table in LDS: hash table, rows (slot 0 = -infinity) and single-survivor sums.  All threads of
// the workgroup call this; K <= S2_MAX_KEPT.
__device__ __forceinline__ void s2_stage_tables(int q, int K, int hsh, const int32_t *__restrict__ kept_ids,
                                                const float *__restrict__ T, uint32_t *htab, float *Tl, float *rowsum)
{
    const int tid = threadIdx.x;
    for (int e = tid; e < S2_HASH; e += blockDim.x) htab[e] = 0xFFFFFFFFu;
    const float *Tq = T + (int64_t)q * (S2_MAX_KEPT + 1) * QLEN;
    for (int e = tid; e < (K + 1) * QLEN; e += blockDim.x)
        Tl[(e >> 5) * S2_TSTRIDE + (e & 31)] = (e >> 5) ? Tq[e] : -INFINITY;
    __syncthreads();
    if (tid < K) {
        const uint32_t code = (uint32_t)kept_ids[(int64_t)q * S2_MAX_KEPT + tid];
        htab[(code ^ (code >> hsh)) & (S2_HASH - 1)] = (code << 6) | (uint32_t)(tid + 1);
        // one survivor in the bag: the maxima are its row, summed in the same order as in s2_score_members
        double d = 0.0;
        for (int i = 0; i < QLEN; ++i) d += (double)Tl[(tid + 1) * S2_TSTRIDE + i];
        rowsum[tid + 1] = (float)d;
    }
    __syncthreads();
}

// Persistent workgroups; wave w of the grid scores the 64-passage tiles w, w + W, w + 2W, ... (lane = passage).
__global__ __launch_bounds__(S2_THREADS) void s2_stream_kernel(
    const float *__restrict__ S, int64_t C, const uint32_t *__restrict__ keepbits, int64_t keep_words,
    const int32_t *__restrict__ codes, int64_t N, const int64_t *__restrict__ doc_offsets, int64_t P,
    const uint32_t *__restrict__ candbits, int64_t cand_words, const S2Meta *__restrict__ meta,
    const int32_t *__restrict__ kept_ids, const float *__restrict__ T, uint64_t *__restrict__ keys2, int64_t key_stride,
    int32_t *__restrict__ hist, uint32_t *__restrict__ emptybits)
{
    __shared__ __align__(16) uint8_t stage_all[S2_THREADS / 64][S2W_CAP + 64];
    __shared__ uint32_t linebits_all[S2_THREADS / 64][S2_LBWORDS];
    __shared__ uint32_t htab[S2_HASH];
    __shared__ __align__(16) float Tl[(S2_MAX_KEPT + 1) * S2_TSTRIDE];
    __shared__ int32_t lhist[SEL_BINS];
    __shared__ float rowsum[S2_MAX_KEPT + 1];  // score of a bag holding only slot s
    const int q = blockIdx.y;
    const int K = s2_uniform(meta[q].K);
    const float bin_hi = meta[q].bin_hi, bin_scale = meta[q].bin_scale;
    uint32_t *keys_out = reinterpret_cast<uint32_t *>(keys2 + (int64_t)q * key_stride);  // slot p: passage p's score word
    int32_t *hist_q = hist + (int64_t)q * SEL_BINS;
    const int tid = threadIdx.x, lane = tid & 63;
    if (K == 0) {
        // no centroid passes Eq. 5: every bag is empty whatever the codes are, so they are not read.  There is no valid
        // key and the histogram stays zero; the candidates themselves are the empty-bag set.
        const uint32_t *cb0 = candbits + (int64_t)q * cand_words;
        uint32_t *eb0 = emptybits + (int64_t)q * cand_words;
        for (int64_t w = (int64_t)blockIdx.x * S2_THREADS + tid; w < cand_words; w += (int64_t)gridDim.x * S2_THREADS)
            eb0[w] = cb0[w];
        return;
    }
    for (int e = tid; e < SEL_BINS; e += S2_THREADS) lhist[e] = 0;
    if (K > S2_MAX_KEPT) {  // too many survivors for slot sets (uniform for the whole workgroup): gather form
        __syncthreads();
        s2_gather_body(q, S, C, keepbits, keep_words, candbits + (int64_t)q * cand_words, 0,
                       (int64_t)blockIdx.x * 4 + (tid >> 6), (int64_t)gridDim.x * 4, cand_words, cand_words, P, doc_offsets, codes,
                       bin_hi, bin_scale, keys_out, lhist, emptybits);
        s2_flush_hist(lhist, hist_q);
        return;
    }
    const int hsh = s2_uniform(meta[q].hash_shift);
    const int wave = s2_uniform(tid >> 6);
    s2_stage_tables(q, K, hsh, kept_ids, T, htab, Tl, rowsum);

    uint8_t *stage = stage_all[wave];
    uint32_t *linebits = linebits_all[wave];
    const uint32_t *cb = candbits + (int64_t)q * cand_words;
    uint32_t *eb = emptybits + (int64_t)q * cand_words;
    const int ntiles = (int)((P + S2W_PASS - 1) / S2W_PASS);
    const int nwaves = (int)gridDim.x * (S2_THREADS / 64);

    // A tile's metadata (candidate words, passage offsets) is requested one tile ahead of its use.
    int tile = (int)blockIdx.x * (S2_THREADS / 64) + wave;
    uint32_t cword_n = 0u;
    int64_t olane_n = 0, oend_n = 0;
    auto request_meta = [&](int t) {
        if (t < ntiles) {  // uniform
            const int64_t p0n = (int64_t)t * S2W_PASS;
            const int tpn = (int)(P - p0n < S2W_PASS ? P - p0n : S2W_PASS);
            const int64_t win = (p0n >> 5) + (lane >> 5);
            cword_n = (lane < tpn && win < cand_words) ? cb[win] : 0u;
            olane_n = doc_offsets[p0n + (lane <= tpn ? lane : tpn)];
            oend_n = doc_offsets[p0n + tpn];
        }
    };
    request_meta(tile);
    for (; tile < ntiles; tile += nwaves) {
        const int64_t p0 = (int64_t)tile * S2W_PASS;
        const int tp = (int)(P - p0 < S2W_PASS ? P - p0 : S2W_PASS);
        const uint32_t cword = cword_n;
        const int64_t o_lane = olane_n, o_end = oend_n;
        request_meta(tile + nwaves);
        const bool cand = lane < tp && ((cword >> (lane & 31)) & 1u);
        const unsigned long long candm = __ballot(cand);
        if (candm == 0ull) {  // (uniform) no candidate here: only the empty-bag words are cleared
            const int64_t wi = (p0 >> 5) + (lane >> 5);
            if ((lane & 31) == 0 && wi < cand_words) eb[wi] = 0u;
            continue;
        }
        uint64_t set = 0;  // bit s = slot s occurs in my passage; bit 0 collects the pruned tokens

        // token range of my passage relative to the tile's first token
        const int64_t o0 = __shfl(o_lane, 0);
        int64_t r = o_lane - o0;
        const int my_lo = r > 0x7FFFFFFFll ? 0x7FFFFFFF : (int)r;
        int my_hi = __shfl_down(my_lo, 1);
        if (lane == 63) {  // lane 63 has no right neighbour: its end is the tile's end
            r = o_end - o0;
            my_hi = r > 0x7FFFFFFFll ? 0x7FFFFFFF : (int)r;
        }
        if (lane >= tp) my_hi = my_lo;

        // Rounds of consecutive whole passages that fit the staging buffer, each starting at a candidate; the passages
        // after the tile's last candidate are never staged.
        int ps = s2_uniform(__ffsll((long long)candm) - 1);
        const int plast = s2_uniform(63 - __clzll((long long)candm));
        while (ps <= plast) {  // ps, fit, pe are uniform; each round advances ps by at least one
            const int base = s2_uniform(__shfl(my_lo, ps));
            const int fit = s2_uniform(__popcll(__ballot(lane >= ps && lane <= plast && my_hi - base <= S2W_CAP)));
            if (fit == 0) {
                // a single passage longer than the staging buffer: its lane folds it straight from global memory
                if (lane == ps)
                    for (int64_t j = o0 + my_lo; j < o0 + my_hi; ++j) set |= 1ull << s2_lookup(htab, (uint32_t)codes[j], hsh);
                ps = s2_uniform(s2_next_bit(candm, ps + 1));
            } else {
                const int pe = ps + fit;
                const int end = s2_uniform(__shfl(my_hi, pe - 1));
                const int64_t g0 = o0 + base;   // first token of the round
                const int64_t a0 = g0 & ~31ll;  // start of its 128-byte line
                const int shift = (int)(g0 - a0);
                const int nchunk = (shift + (end - base) + 31) >> 5;  // 128-byte lines of the round, <= 8 * S2_ITEMS
                const bool mine = lane >= ps && lane < pe && cand;
                // lines of the round that hold a candidate's tokens; when every passage of the round is a candidate
                // that is all of them
                const unsigned long long round_mask = (pe < 64 ? (1ull << pe) : 0ull) - (1ull << ps);
                const bool dense = (candm & round_mask) == round_mask;  // uniform
                if (lane < S2_LBWORDS) linebits[lane] = dense ? 0xFFFFFFFFu : 0u;
                s2_wave_sync();
                if (!dense) {
                    if (mine && my_hi > my_lo) {
                        const int c0 = (my_lo - base + shift) >> 5, c1 = (my_hi - 1 - base + shift) >> 5;
                        for (int c = c0; c <= c1; ++c) atomicOr(&linebits[c >> 5], 1u << (c & 31));
                    }
                    s2_wave_sync();
                }
                // Stage one byte per token: the slot of its centroid (0 = pruned).  Item u of a lane is the 16 bytes at token
                // 4 * (64 u + lane), so item u of the wave covers lines 8u .. 8u+7, which is byte u of the line bitmap: a
                // uniform test skips the item when no candidate touches those lines.  All loads of the round are issued
                // before the first is used, so a round costs one memory latency.
                const int nitem = nchunk * 8;
                const int32_t *__restrict__ src = codes + a0;  // uniform base, 32-bit lane offsets
                uint32_t need[S2_LBWORDS];
    #pragma unroll
                for (int k = 0; k < S2_LBWORDS; ++k) need[k] = (uint32_t)s2_uniform((int)linebits[k]);
                int4 v[S2_ITEMS];
                uint32_t okm = 0u;
    #pragma unroll
                for (int u = 0; u < S2_ITEMS; ++u) {
                    v[u] = make_int4(-1, -1, -1, -1);
                    const uint32_t lines8 = (need[u >> 2] >> (8 * (u & 3))) & 0xFFu;  // uniform
                    if (lines8 != 0u) {
                        const int it = 64 * u + lane;
                        const bool ok = it < nitem && ((lines8 >> (lane >> 3)) & 1u) && a0 + 4ll * it + 3 < N;
                        if (ok) v[u] = *reinterpret_cast<const int4 *>(src + 4 * it);
                        okm |= ok ? 1u << u : 0u;
                    }
                }
                uint32_t hit = 0u;
    #pragma unroll
                for (int u = 0; u < S2_ITEMS; ++u) {
                    const uint32_t lines8 = (need[u >> 2] >> (8 * (u & 3))) & 0xFFu;  // uniform
                    if (lines8 != 0u) {
                        if ((okm >> u) & 1u) {
                            const uint32_t packed = s2_lookup(htab, (uint32_t)v[u].x, hsh) |
                                                    (s2_lookup(htab, (uint32_t)v[u].y, hsh) << 8) |
                                                    (s2_lookup(htab, (uint32_t)v[u].z, hsh) << 16) |
                                                    (s2_lookup(htab, (uint32_t)v[u].w, hsh) << 24);
                            *reinterpret_cast<uint32_t *>(stage + 4 * (64 * u + lane)) = packed;
                            hit |= packed;
                        }
                    }
                }
                // the one item that straddles the end of the code array (tokens past N belong to no passage)
                if (a0 + 4ll * nitem > N) {
                    const int64_t it = (N - a0) >> 2;
                    if (lane < 4 && it < nitem && a0 + 4 * it + lane < N) {
                        const uint32_t sl = s2_lookup(htab, (uint32_t)codes[a0 + 4 * it + lane], hsh);
                        stage[4 * it + lane] = (uint8_t)sl;
                        hit |= sl;
                    }
                }
                s2_wave_sync();
                const bool any_hit = __ballot(hit != 0u) != 0ull;  // uniform
                if (any_hit && mine && my_hi > my_lo) {
                    // four staged bytes at a time; most are zero (pruned tokens) and are skipped as a word
                    const int v0 = my_lo - base + shift, v1 = my_hi - base + shift;
                    const uint32_t *stage32 = reinterpret_cast<const uint32_t *>(stage);
                    for (int wd = v0 >> 2; wd <= (v1 - 1) >> 2; ++wd) {
                        uint32_t x = stage32[wd];
                        if (4 * wd < v0) x &= 0xFFFFFFFFu << (8 * (v0 - 4 * wd));       // bytes before the passage
                        if (4 * wd + 4 > v1) x &= 0xFFFFFFFFu >> (8 * (4 * wd + 4 - v1));  // bytes after it
                        if (x) {
                            set |= 1ull << (x & 0xFFu);
                            set |= 1ull << ((x >> 8) & 0xFFu);
                            set |= 1ull << ((x >> 16) & 0xFFu);
                            set |= 1ull << (x >> 24);
                        }
                    }
                }
                s2_wave_sync();
                ps = s2_uniform(s2_next_bit(candm, pe));
            }
        }

        // score: column maxima of the rows in the set, summed over the query tokens in index order; eight query tokens
        // at a time, so that few registers are live
        const uint64_t members = set & ~1ull;
        const bool empty = members == 0;
        float score = -INFINITY;
        if (cand && !empty) score = s2_score_members(members, Tl, rowsum);
        // emit: slot p of the key array belongs to candidate p; no counters, no ordering between waves
        const bool live = cand && !empty;
        if (cand) keys_out[p0 + lane] = live ? plaid_score_to_ord(score) : PLAID_S2_NO_SCORE;
        if (live) atomicAdd(&lhist[plaid_s2_bin(score, bin_hi, bin_scale)], 1);
        const unsigned long long eb64 = __ballot(cand && empty);
        if (lane == 0) {
            const int64_t w0 = p0 >> 5;
            if (w0 < cand_words) eb[w0] = (uint32_t)eb64;
            if (w0 + 1 < cand_words) eb[w0 + 1] = (uint32_t)(eb64 >> 32);
        }
    }
    s2_flush_hist(lhist, hist_q);
}


// ------------------------------------------------------------------ inverted form: candidates and bags from the inverted lists
// A passage contains centroid c exactly when it is in c's inverted list (Section 4.1 stores unique passage ids per
// centroid).  So the candidate set is the union of the probed centroids' lists, and the pruned bag of a passage
// (Eq. 5) is the set of surviving centroids whose lists contain it: both follow from the inverted lists of at most
// 32 nprobe + S2_MAX_KEPT centroids, far fewer bytes than the candidates' token codes whenever few centroids
// survive.  A workgroup owns a range of 2^SHIFT consecutive passages: it ORs the lists' entries that fall into
// its range into 64-bit words in LDS (bit 0 = candidate, bit s = surviving slot s), then scores, emits keys, the bin
// histogram, the candidate words and the empty-bag words of the range exactly as the streaming form does.  Where a
// list enters a range comes from a table built once per index: table[c][r] = position in list c of its first entry
// with passage id >= r * 2^SHIFT.
#define IVR_EMPTY 0xFFFFFFFFu
#define IVR_LISTS 256  // lists handled per LDS round (brought by the first IVR_LISTS threads of the workgroup)
#define IVR_SHORT 64   // a list with at most this many entries in the range joins the pooled pass
#define IVR_DENSE_DIV 16  // a list with at least P / 16 entries also gets a bitmap over the passages

// table[c][r] for every non-empty (list, range) pair; the others keep IVR_EMPTY until ivr_fill_kernel.
__global__ __launch_bounds__(256) void ivr_mark_kernel(const int64_t *__restrict__ ivf_offsets,
                                                       const int32_t *__restrict__ ivf_pids, int64_t C, int64_t nr,
                                                       int shift, uint32_t *__restrict__ table)
{
    for (int64_t c = blockIdx.x; c < C; c += gridDim.x) {
        const int64_t s = ivf_offsets[c], t = ivf_offsets[c + 1];
        for (int64_t e = s + threadIdx.x; e < t; e += blockDim.x) {
            const int64_t r = (int64_t)(uint32_t)ivf_pids[e] >> shift;
            const bool first = e == s || ((int64_t)(uint32_t)ivf_pids[e - 1] >> shift) != r;
            if (first && r < nr) table[c * (nr + 1) + r] = (uint32_t)(e - s);
        }
    }
}
// A range a list has no entry in starts where the next one does; the last column is the list's length.
__global__ __launch_bounds__(256) void ivr_fill_kernel(const int64_t *__restrict__ ivf_offsets, int64_t C, int64_t nr,
                                                       uint32_t *__restrict__ table)
{
    const int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= C) return;
    uint32_t next = (uint32_t)(ivf_offsets[c + 1] - ivf_offsets[c]);
    uint32_t *row = table + c * (nr + 1);
    row[nr] = next;
    for (int64_t r = nr - 1; r >= 0; --r) {
        const uint32_t v = row[r];
        if (v == IVR_EMPTY || v > next) row[r] = next;  // (v > next only if a list is not ascending: keep the row monotone)
        else next = v;
    }
}

size_t plaid_ivf_range_table_bytes(int64_t C, int64_t P, int shift)
{
    const int64_t nr = (P + (1ll << shift) - 1) >> shift;
    return (size_t)C * (size_t)(nr + 1) * sizeof(uint32_t);
}
void plaid_launch_ivf_range_table(hipStream_t st, const int64_t *ivf_offsets, const int32_t *ivf_pids, int64_t C, int64_t P,
                                  int shift, uint32_t *table)
{
    const int64_t nr = (P + (1ll << shift) - 1) >> shift;
    plaid_launch_fill_u32(st, table, C * (nr + 1), IVR_EMPTY);
    hipLaunchKernelGGL(ivr_mark_kernel, dim3((unsigned)(C < 8192 ? C : 8192)), dim3(256), 0, st, ivf_offsets, ivf_pids, C, nr, shift, table);
    hipLaunchKernelGGL(ivr_fill_kernel, dim3((unsigned)((C + 255) / 256)), dim3(256), 0, st, ivf_offsets, C, nr, table);
}

// Dense lists.  The centroid of a frequent token occurs in a large share of the passages: its list is then longer than
// a bitmap over the passages (P / 8 bytes), and a query that probes it would read megabytes of passage ids to set
// nearly every candidate bit.  Lists with at least P / IVR_DENSE_DIV entries therefore also get such a bitmap at index
// creation: dense_id[c] = row of the bitmap, or -1.
__global__ __launch_bounds__(256) void ivr_dense_mark_kernel(const int64_t *__restrict__ ivf_offsets, int64_t C, int64_t P,
                                                             int32_t *__restrict__ dense_id, int32_t *__restrict__ counter)
{
    const int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= C) return;
    const int64_t len = ivf_offsets[c + 1] - ivf_offsets[c];
    dense_id[c] = (len > 0 && len * IVR_DENSE_DIV >= P) ? atomicAdd(counter, 1) : -1;
}
__global__ __launch_bounds__(256) void ivr_dense_fill_kernel(const int64_t *__restrict__ ivf_offsets,
                                                             const int32_t *__restrict__ ivf_pids, int64_t C, int64_t P,
                                                             const int32_t *__restrict__ dense_id, uint32_t *__restrict__ bits,
                                                             int64_t words)
{
    for (int64_t c = blockIdx.x; c < C; c += gridDim.x) {
        const int32_t d = dense_id[c];
        if (d < 0) continue;  // uniform
        uint32_t *row = bits + (int64_t)d * words;
        const int64_t s = ivf_offsets[c], t = ivf_offsets[c + 1];
        for (int64_t e = s + threadIdx.x; e < t; e += blockDim.x) {
            const uint32_t pid = (uint32_t)ivf_pids[e];
            if ((int64_t)pid < P) atomicOr(&row[pid >> 5], 1u << (pid & 31));
        }
    }
}
void plaid_launch_ivf_dense_mark(hipStream_t st, const int64_t *ivf_offsets, int64_t C, int64_t P, int32_t *dense_id,
                                 int32_t *counter)
{
    hipLaunchKernelGGL(ivr_dense_mark_kernel, dim3((unsigned)((C + 255) / 256)), dim3(256), 0, st, ivf_offsets, C, P, dense_id,
                       counter);
}
void plaid_launch_ivf_dense_fill(hipStream_t st, const int64_t *ivf_offsets, const int32_t *ivf_pids, int64_t C, int64_t P,
                                 const int32_t *dense_id, uint32_t *bits, int64_t words)
{
    hipLaunchKernelGGL(ivr_dense_fill_kernel, dim3((unsigned)(C < 8192 ? C : 8192)), dim3(256), 0, st, ivf_offsets, ivf_pids, C,
                       P, dense_id, bits, words);
}

// Exclusive prefix sum of one value per thread over the first IVR_LISTS threads of the workgroup, into
// out[0 .. IVR_LISTS]; scratch: one int per wave of those threads.  All threads of the workgroup call this.
__device__ __forceinline__ void ivr_block_scan(int v, int32_t *out, int32_t *wave_tot)
{
    const int tid = threadIdx.x, lane = tid & 63;
    if (tid >= IVR_LISTS) {  // (whole waves) the other threads only keep the barriers company
        __syncthreads();
        __syncthreads();
        return;
    }
    int incl = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int t = __shfl_up(incl, d);
        if (lane >= d) incl += t;
    }
    if (lane == 63) wave_tot[tid >> 6] = incl;
    __syncthreads();
    int base = 0;
    for (int wv = 0; wv < (tid >> 6); ++wv) base += wave_tot[wv];
    out[tid + 1] = base + incl;
    if (tid == 0) out[0] = 0;
    __syncthreads();
}

// LDS work arrays of ivr_apply_round.
struct IvrLists {
    int64_t long_start[IVR_LISTS];              // compacted lists with more than IVR_SHORT entries in the range
    int32_t long_cnt[IVR_LISTS];
    unsigned long long long_val[IVR_LISTS];
    int64_t short_start[IVR_LISTS];             // per thread: its list when it has 1 .. IVR_SHORT entries in the range
    unsigned long long short_val[IVR_LISTS];
    int32_t pref[IVR_LISTS + 1];                // packed prefix sums: long-list count << 20 | short entries
    int32_t wave_tot[IVR_LISTS / 64];
    int32_t next;
};

// One round of list application: thread t < IVR_LISTS brings one list (cnt entries of ivf_pids from `first` on fall into
// the range of `range` passages, cnt = 0: none; the other threads bring none) and the bits `val` to OR into the set words of those passages.  Lists with few entries are pooled into
// one flat index range that all threads share (a lane finds its entry by binary search in the prefix sums), so that
// fifty lists of two entries cost one memory round trip instead of fifty; a long list is walked by one wave, 512
// entries per step with eight loads in flight, waves taking lists from a shared counter.  All threads call this.
template <typename SetT>
__device__ __forceinline__ void ivr_apply_round(int cnt, int64_t first, unsigned long long val,
                                                const int32_t *__restrict__ ivf_pids, uint32_t r0, uint32_t range,
                                                SetT *lsets, IvrLists &L)
{
    const int tid = threadIdx.x, lane = tid & 63;
    const bool is_long = cnt > IVR_SHORT;
    const int packed = is_long ? (1 << 20) : cnt;
    if (tid == 0) L.next = 0;
    ivr_block_scan(packed, L.pref, L.wave_tot);
    if (is_long) {
        const int at = L.pref[tid] >> 20;
        L.long_start[at] = first;
        L.long_cnt[at] = cnt;
        L.long_val[at] = val;
    } else if (cnt > 0) {
        L.short_start[tid] = first;
        L.short_val[tid] = val;
    }
    __syncthreads();
    const int n_long = L.pref[IVR_LISTS] >> 20, n_short = L.pref[IVR_LISTS] & 0xFFFFF;
    for (int w = tid; w < n_short; w += (int)blockDim.x) {
        int lo = 0, hi = IVR_LISTS;  // largest lo whose short-entry prefix is <= w: the list that holds entry w
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if ((L.pref[mid] & 0xFFFFF) <= w) lo = mid;
            else hi = mid;
        }
        const uint32_t loc = (uint32_t)ivf_pids[L.short_start[lo] + (w - (L.pref[lo] & 0xFFFFF))] - r0;
        if (loc < range) atomicOr(&lsets[loc], (SetT)L.short_val[lo]);  // (false only if a list is not ascending)
    }
    for (;;) {
        int l = 0;
        if (lane == 0) l = atomicAdd(&L.next, 1);
        l = s2_uniform(__shfl(l, 0));
        if (l >= n_long) break;
        const int n = s2_uniform(L.long_cnt[l]);
        const int32_t *__restrict__ src = ivf_pids + L.long_start[l];
        const SetT v = (SetT)L.long_val[l];
        for (int e0 = 0; e0 < n; e0 += 512) {
            uint32_t pid[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int e = e0 + 64 * u + lane;
                pid[u] = e < n ? (uint32_t)src[e] : 0xFFFFFFFFu;
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const uint32_t loc = pid[u] - r0;
                if (pid[u] != 0xFFFFFFFFu && loc < range) atomicOr(&lsets[loc], v);
            }
        }
    }
    __syncthreads();
}

// Queries none of whose centroids passes Eq. 5: every bag is empty, so stage 2 only has to produce the candidate set,
// and a passage needs one bit instead of a set word.  A workgroup then covers 2^19 passages (64 KB of LDS bits): a wave
// walks one probed centroid's list at a time (512 entries per step, eight loads in flight), and the bits are written
// out once, as the candidate words and as the empty-bag words.  The fine-grained kernel below skips these queries.
#define UW_SHIFT 19
#define UW_WORDS (1 << (UW_SHIFT - 5))
#define UW_THREADS 1024
#define UW_LONG 4096  // entries from which on a list is walked by all waves together
#define IVR_WIDE_MIN_QUERIES 32
static_assert(UW_SHIFT >= 13, "a wide range is a whole number of table ranges");
__global__ __launch_bounds__(UW_THREADS) void s2_union_wide_kernel(
    const int32_t *__restrict__ uniq, const int32_t *__restrict__ n_uniq, int uniq_stride,
    const int64_t *__restrict__ ivf_offsets, const int32_t *__restrict__ ivf_pids, const uint32_t *__restrict__ table,
    int64_t nr, int shift, int64_t P, const S2Meta *__restrict__ meta, const int32_t *__restrict__ dense_id,
    const uint32_t *__restrict__ dense_bits, uint32_t *__restrict__ candbits, int64_t cand_words,
    uint32_t *__restrict__ emptybits)
{
    __shared__ uint32_t bits[UW_WORDS];
    __shared__ int64_t first[IVR_LISTS];
    __shared__ int32_t count[IVR_LISTS];
    __shared__ int32_t dense[IVR_LISTS];  // rows of the dense-list bitmaps probed in this round
    __shared__ int32_t n_dense;
    const int q = blockIdx.y;
    if (s2_uniform(meta[q].K) != 0) return;  // uniform
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = s2_uniform(tid >> 6);
    const int64_t fr0 = (int64_t)blockIdx.x << (UW_SHIFT - shift);  // table ranges [fr0, fr1)
    const int64_t fr1 = fr0 + (1ll << (UW_SHIFT - shift)) < nr ? fr0 + (1ll << (UW_SHIFT - shift)) : nr;
    const uint32_t p0 = (uint32_t)blockIdx.x << UW_SHIFT;
    for (int e = tid; e < UW_WORDS; e += UW_THREADS) bits[e] = 0u;
    const int nu = n_uniq[q];
    for (int u0 = 0; u0 < nu; u0 += IVR_LISTS) {
        const int nb = nu - u0 < IVR_LISTS ? nu - u0 : IVR_LISTS;
        __syncthreads();  // the bits are zero / the previous round's lists are done
        if (tid == 0) n_dense = 0;
        __syncthreads();
        if (tid < nb) {
            const int32_t c = uniq[(int64_t)q * uniq_stride + u0 + tid];
            const int32_t d = dense_id[c];
            if (d >= 0) {  // its bitmap is OR-ed in below
                dense[atomicAdd(&n_dense, 1)] = d;
                count[tid] = 0;
            } else {
                const uint32_t a = table[(int64_t)c * (nr + 1) + fr0], b = table[(int64_t)c * (nr + 1) + fr1];
                first[tid] = ivf_offsets[c] + a;
                count[tid] = b > a ? (int)(b - a) : 0;
            }
        }
        __syncthreads();
        // steps s0, s0 + stride, ... of list l (a step = 512 entries).  A lane takes eight consecutive entries and merges
        // the bits that fall into one word before it touches LDS: in the list of a centroid that occurs in nearly every
        // passage consecutive entries are consecutive passages, and one entry per lane would send 32 lanes to each word.
        auto walk = [&](int l, int s0, int stride) {
            const int n = s2_uniform(count[l]);
            const int32_t *__restrict__ src = ivf_pids + first[l];
            for (int e0 = s0 * 512; e0 < n; e0 += stride * 512) {
                uint32_t pid[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int e = e0 + 8 * lane + u;
                    pid[u] = e < n ? (uint32_t)src[e] : 0xFFFFFFFFu;
                }
                uint32_t cw = 0xFFFFFFFFu, acc = 0u;
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const uint32_t loc = pid[u] - p0;
                    if (pid[u] != 0xFFFFFFFFu && loc < (1u << UW_SHIFT)) {
                        const uint32_t w = loc >> 5, bit = 1u << (loc & 31);
                        if (w != cw) {
                            if (acc) atomicOr(&bits[cw], acc);
                            cw = w;
                            acc = bit;
                        } else {
                            acc |= bit;
                        }
                    }
                }
                if (acc) atomicOr(&bits[cw], acc);
            }
        };
        // a wave takes whole lists of ordinary length; the lists of centroids that occur in most passages (hundreds
        // of thousands of entries) are shared by all waves
        for (int l = wave; l < nb; l += UW_THREADS / 64)
            if (count[l] <= UW_LONG) walk(l, 0, 1);
        for (int l = 0; l < nb; ++l)
            if (count[l] > UW_LONG) walk(l, wave, UW_THREADS / 64);
        const int nd = n_dense;
        if (nd > 0) {  // uniform
            __syncthreads();  // the walks' atomics are done: each word now has one owner thread
            const int64_t wf = (int64_t)p0 >> 5;
            const int64_t nwr = cand_words - wf < UW_WORDS ? cand_words - wf : UW_WORDS;
            for (int64_t w = tid; w < nwr; w += UW_THREADS) {
                uint32_t v = bits[w];
                for (int d = 0; d < nd; ++d) v |= dense_bits[(int64_t)dense[d] * cand_words + wf + w];
                bits[w] = v;
            }
        }
    }
    __syncthreads();
    const int64_t w_first = (int64_t)p0 >> 5;
    uint32_t *cbq = candbits + (int64_t)q * cand_words + w_first;
    uint32_t *ebq = emptybits + (int64_t)q * cand_words + w_first;
    const int64_t nw = cand_words - w_first < UW_WORDS ? cand_words - w_first : UW_WORDS;
    for (int64_t w = tid; w < nw; w += UW_THREADS) {
        uint32_t v = bits[w];
        const int64_t pbase = (int64_t)p0 + 32 * w;  // passages past the end never enter the lists; the mask is a guard
        if (pbase + 32 > P) v &= pbase < P ? (1u << (uint32_t)(P - pbase)) - 1u : 0u;
        cbq[w] = v;
        ebq[w] = v;
    }
}

// Counting sort of a round's bags by size (LDS).
#define S2_ORDER_ROUND 2048  // passages per round
struct S2Order {
    int32_t count[64];                // bags of each size (2..63 members)
    int32_t start[64];                // running positions, largest size first
    int32_t total;
    uint16_t list[S2_ORDER_ROUND];    // round-local passages in that order
};
// The list-application arrays and the sort are never live together.
union S2InvertScratch {
    IvrLists lists;
    S2Order order;
};

// SetT: the per-passage set word.  Queries with at most 31 surviving centroids fit 32-bit words (bit 0 = candidate,
// bits 1..31 = slots), which halves the kernel's largest LDS array and lets two of the 1024-thread workgroups share a
// compute unit; the 64-bit instance serves the other queries.  Both are launched; each leaves the other's queries alone.
template <int SHIFT, typename SetT>
__global__ __launch_bounds__(IVR_THREADS(SHIFT)) void s2_invert_kernel(
    const int32_t *__restrict__ uniq, const int32_t *__restrict__ n_uniq, int uniq_stride,
    const int64_t *__restrict__ ivf_offsets, const int32_t *__restrict__ ivf_pids, const uint32_t *__restrict__ table,
    int64_t nr, const float *__restrict__ S, int64_t C, const uint32_t *__restrict__ keepbits, int64_t keep_words,
    const int32_t *__restrict__ codes, const int64_t *__restrict__ doc_offsets, int64_t P, const S2Meta *__restrict__ meta,
    const int32_t *__restrict__ kept_ids, const float *__restrict__ T, uint32_t *__restrict__ candbits, int64_t cand_words,
    uint64_t *__restrict__ keys2, int64_t key_stride, int32_t *__restrict__ hist, uint32_t *__restrict__ emptybits,
    int skip_k0, const int32_t *__restrict__ qcount, const int32_t *__restrict__ qlist, int qlist_stride)
{
    constexpr int RANGE = 1 << SHIFT, THREADS = IVR_THREADS(SHIFT);
    __shared__ SetT lsets[RANGE];
    __shared__ uint32_t lcand[RANGE / 32], lempty[RANGE / 32];
    __shared__ uint32_t htab[S2_HASH];
    __shared__ __align__(16) float Tl[(S2_MAX_KEPT + 1) * S2_TSTRIDE];
    __shared__ float rowsum[S2_MAX_KEPT + 1];
    __shared__ int32_t lhist[SEL_BINS];
    __shared__ S2InvertScratch scratch;
    __shared__ uint32_t slot_probed[2];  // bit s: surviving slot s is also a probed centroid
    const int64_t r = blockIdx.x;
    const uint32_t r0 = (uint32_t)(r << SHIFT);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = s2_uniform(tid >> 6);
    // This instance's queries: those with 1..31 (32-bit sets) or more (64-bit sets) surviving centroids, and with the
    // 32-bit instance those without any unless s2_union_wide_kernel has produced their candidate and empty-bag words.
    // Row y of the grid takes entries y, y + gridDim.y, ... of the lists the probe kernel made.
    // skip_k0 bit 1 (64-bit instance only): this instance is the only one launched and takes every query (a launch of a
    // few queries: one kernel less on the way of each).
    const int cls = sizeof(SetT) == 4 ? 1 : 2;
    const bool take_all = sizeof(SetT) == 8 && (skip_k0 & 2);
    const bool skip_none = skip_k0 & 1;
    const int n_first = take_all ? qcount[1] : qcount[cls];                      // entries of list 1 (or of this class)
    const int n_second = take_all ? qcount[2] : 0;                               // then of list 2
    const int n_none = ((cls == 1 || take_all) && !skip_none) ? qcount[0] : 0;   // then of list 0
    const int n_all = n_first + n_second + n_none;
    // Only the 2048-passage instance with 64-bit sets loops: its class is usually empty or nearly so, and a launch of
    // nq rows of workgroups that all find nothing to do costs tens of microseconds.  The other instances are launched
    // with one row per query and take one entry (a class that holds most of the chunk's queries runs faster that way).
    constexpr bool LOOP = SHIFT == 11 && sizeof(SetT) == 8;
    int qi = blockIdx.y;
    if (qi >= n_all) return;  // uniform
    do {
    const int q = qi < n_first ? qlist[(int64_t)(take_all ? 1 : cls) * qlist_stride + qi]
                               : (qi < n_first + n_second ? qlist[2ll * qlist_stride + qi - n_first]
                                                          : qlist[qi - n_first - n_second]);
    const int K = s2_uniform(meta[q].K);
    if (!take_all && (K <= 31) != (sizeof(SetT) == 4)) continue;  // (never: the lists are made from the same K)
    const bool slots = K > 0 && K <= S2_MAX_KEPT;  // bags are kept as slot sets
    const int hsh = s2_uniform(meta[q].hash_shift);
    for (int e = tid; e < RANGE; e += THREADS) lsets[e] = (SetT)0;
    for (int e = tid; e < SEL_BINS; e += THREADS) lhist[e] = 0;
    if (tid < 2) slot_probed[tid] = 0u;
    if (slots) s2_stage_tables(q, K, hsh, kept_ids, T, htab, Tl, rowsum);
    else __syncthreads();

    // The lists to apply, in one index space: the probed centroids' (candidate bit, plus the slot bit when the centroid
    // also survives), then the surviving centroids' that were not probed (slot bit only).  A round takes IVR_LISTS of
    // them: the centroid ids are fetched first, the slots of the probed ones marked in LDS, and only then -- one
    // barrier later, which by then costs no memory round trip -- do all lists of the round look up their stretch of
    // the range together.  (A surviving centroid's round comes after every probed centroid's mark.)
    const int nu = n_uniq[q], ntot = nu + (slots ? K : 0);
    for (int u0 = 0; u0 < ntot; u0 += IVR_LISTS) {
        const int e = u0 + tid;
        const bool mine = tid < IVR_LISTS && e < ntot, survivor = mine && e >= nu;
        int32_t c = -1;
        if (mine) c = survivor ? kept_ids[(int64_t)q * S2_MAX_KEPT + e - nu] : uniq[(int64_t)q * uniq_stride + e];
        unsigned long long val = 0;
        if (mine && !survivor) {
            const uint32_t sl = slots ? s2_lookup(htab, (uint32_t)c, hsh) : 0u;
            val = 1ull | (sl ? 1ull << sl : 0ull);
            if (sl) atomicOr(&slot_probed[sl >> 5], 1u << (sl & 31));
        }
        __syncthreads();
        if (survivor) {
            const int sl = e - nu + 1;
            val = 1ull << sl;
            if ((slot_probed[sl >> 5] >> (sl & 31)) & 1u) c = -1;  // already applied with its probed list
        }
        int cnt = 0;
        int64_t first = 0;
        if (c >= 0) {
            const uint32_t a = table[(int64_t)c * (nr + 1) + r], b = table[(int64_t)c * (nr + 1) + r + 1];
            first = ivf_offsets[c] + a;
            cnt = b > a ? (int)(b - a) : 0;
        }
        ivr_apply_round(cnt, first, val, ivf_pids, r0, (uint32_t)RANGE, lsets, scratch.lists);
    }

    const int64_t w_first = (int64_t)r0 >> 5;  // first bitmap word of the range
    // emit the range: lane = passage, 64 passages per step
    const float bin_hi = meta[q].bin_hi, bin_scale = meta[q].bin_scale;
    uint32_t *keys_out = reinterpret_cast<uint32_t *>(keys2 + (int64_t)q * key_stride);  // slot p: passage p's score word
    uint32_t *cbq = candbits + (int64_t)q * cand_words;
    uint32_t *ebq = emptybits + (int64_t)q * cand_words;
    // Pass 1, lane = passage in passage order: candidate and empty-bag words, the keys of empty bags and of bags with one
    // member (a table look-up), and how many bags there are of each larger size.
    // Pass 2, lane = bag with two members or more, in the order of their sizes (a counting sort of the passages of a
    // round in LDS): the lanes of a wave then run about the same number of steps over their members, where in passage
    // order each wave would run as long as its largest bag takes.
    S2Order &ord = scratch.order;
    for (int b0 = 0; b0 < RANGE; b0 += S2_ORDER_ROUND) {  // (the last list application ended with a barrier)
        if (slots) {
            for (int e = tid; e < 64; e += THREADS) ord.count[e] = 0;
            __syncthreads();
        }
        for (int g = b0 / 64 + wave; g < (b0 + S2_ORDER_ROUND) / 64; g += THREADS / 64) {
            const SetT vs = lsets[64 * g + lane];
            const int64_t pid = (int64_t)r0 + 64 * g + lane;
            const bool cand = (vs & (SetT)1) && pid < P;
            const SetT members = vs & ~(SetT)1;
            const unsigned long long cm = __ballot(cand);
            bool empty = true;
            if (slots) {
                empty = members == 0;
                const int size = sizeof(SetT) == 4 ? __popc((uint32_t)members) : __popcll((unsigned long long)members);
                float score = -INFINITY;
                if (cand && size == 1) score = rowsum[__ffsll((long long)(unsigned long long)members) - 1];
                if (cand && size <= 1) keys_out[pid] = empty ? PLAID_S2_NO_SCORE : plaid_score_to_ord(score);
                if (cand && size > 1) atomicAdd(&ord.count[size], 1);
                if (cand && size == 1) atomicAdd(&lhist[plaid_s2_bin(score, bin_hi, bin_scale)], 1);
            }
            const unsigned long long em = __ballot(cand && empty);
            if (lane == 0) {
                lcand[2 * g] = (uint32_t)cm;
                lcand[2 * g + 1] = (uint32_t)(cm >> 32);
                lempty[2 * g] = (uint32_t)em;
                lempty[2 * g + 1] = (uint32_t)(em >> 32);
            }
        }
        if (slots) {  // uniform
            __syncthreads();
            if (tid < 64) {  // exclusive prefix over the sizes, largest first: the long bags start the pass
                const int c = ord.count[63 - lane];
                int incl = c;
#pragma unroll
                for (int d = 1; d < 64; d <<= 1) {
                    const int t = __shfl_up(incl, d);
                    if (lane >= d) incl += t;
                }
                ord.start[63 - lane] = incl - c;
                if (lane == 63) ord.total = incl;
            }
            __syncthreads();
            for (int p = b0 + tid; p < b0 + S2_ORDER_ROUND; p += THREADS) {
                const SetT vs = lsets[p];
                const SetT members = vs & ~(SetT)1;
                if ((vs & (SetT)1) && (int64_t)r0 + p < P && (members & (members - 1)) != 0) {
                    const int size = sizeof(SetT) == 4 ? __popc((uint32_t)members) : __popcll((unsigned long long)members);
                    ord.list[atomicAdd(&ord.start[size], 1)] = (uint16_t)(p - b0);
                }
            }
            __syncthreads();
            const int total = ord.total;
            for (int e = tid; e < total; e += THREADS) {
                const int p = b0 + ord.list[e];
                const unsigned long long members = (unsigned long long)(lsets[p] & ~(SetT)1);
                const float score = s2_score_members_wide(members, Tl, rowsum);
                keys_out[(int64_t)r0 + p] = plaid_score_to_ord(score);
                atomicAdd(&lhist[plaid_s2_bin(score, bin_hi, bin_scale)], 1);
            }
            if (b0 + S2_ORDER_ROUND < RANGE) __syncthreads();  // the arrays are set up again for the next round
        }
    }
    __syncthreads();
    // the range's candidate and empty-bag words, one contiguous store each
    int64_t w_end = w_first + RANGE / 32;
    if (w_end > cand_words) w_end = cand_words;
    static_assert(2 * (RANGE / 32) <= THREADS, "one thread per word of the two bitmaps");
    if (tid < RANGE / 32 && w_first + tid < w_end) cbq[w_first + tid] = lcand[tid];
    if (K <= S2_MAX_KEPT && tid >= RANGE / 32 && tid < 2 * (RANGE / 32) && w_first + (tid - RANGE / 32) < w_end)
        ebq[w_first + tid - RANGE / 32] = lempty[tid - RANGE / 32];
    if (K > S2_MAX_KEPT) {
        // too many survivors for slot sets: the range's candidates are scored from their token codes
        s2_gather_body(q, S, C, keepbits, keep_words, lcand, w_first, w_first + wave, THREADS / 64, w_end, cand_words, P,
                       doc_offsets, codes, bin_hi, bin_scale, keys_out, lhist, emptybits);
    }
    if (K > 0) s2_flush_hist(lhist, hist + (int64_t)q * SEL_BINS);
    if (LOOP) __syncthreads();  // the LDS arrays are set up again for the next query
    } while (LOOP && (qi += (int)gridDim.y) < n_all);
}

void plaid_launch_stage2_inverted(hipStream_t st, const int32_t *uniq, const int32_t *n_uniq, int uniq_stride,
                                  const int64_t *ivf_offsets, const int32_t *ivf_pids, const uint32_t *table, const float *S,
                                  int64_t C, const uint32_t *keepbits, int64_t keep_words, const int32_t *codes,
                                  const int64_t *doc_offsets, int64_t P, int nq, const Stage2Buffers &b, uint32_t *candbits,
                                  int64_t cand_words, uint64_t *keys2, int64_t key_stride, const int32_t *dense_id,
                                  const uint32_t *dense_bits, int shift)
{
    const int64_t nr = (P + (1ll << shift) - 1) >> shift;
    const int64_t nwide = (P + (1ll << UW_SHIFT) - 1) >> UW_SHIFT;
    // One workgroup per query and 2^19 passages pays off once the launch holds enough queries to fill the chip with such
    // workgroups; below that the fine-grained kernel (one workgroup per 2^shift passages) also takes the queries
    // without a surviving centroid.
    const int wide = nq >= IVR_WIDE_MIN_QUERIES ? 1 : 0;
    if (wide)
        hipLaunchKernelGGL(s2_union_wide_kernel, dim3((unsigned)nwide, nq), dim3(UW_THREADS), 0, st, uniq, n_uniq, uniq_stride,
                           ivf_offsets, ivf_pids, table, nr, shift, P, b.meta, dense_id, dense_bits, candbits, cand_words,
                           b.emptybits);
    // the looping instance (2048 passages, 64-bit sets): 128 rows of workgroups share its queries
#define S2_INVERT(SH_, T_)                                                                                                  \
    hipLaunchKernelGGL((s2_invert_kernel<SH_, T_>), dim3((unsigned)nr, (SH_ == 11 && sizeof(T_) == 8 && nq > 128) ? 128 : nq), \
                       dim3(IVR_THREADS(SH_)), 0, st, uniq, n_uniq,                                                          \
                       uniq_stride, ivf_offsets, ivf_pids, table, nr, S, C, keepbits, keep_words, codes, doc_offsets, P,     \
                       b.meta, b.kept_ids, b.T, candbits, cand_words, keys2, key_stride, b.hist, b.emptybits, wide,         \
                       b.qcount, b.qlist, b.qlist_stride)
    if (shift == 11 && nq < 8) {
        // a few queries: the 64-bit instance alone, taking every query (same sets, same scores, one launch less)
        hipLaunchKernelGGL((s2_invert_kernel<11, unsigned long long>), dim3((unsigned)nr, nq), dim3(IVR_THREADS(11)), 0, st, uniq,
                           n_uniq, uniq_stride, ivf_offsets, ivf_pids, table, nr, S, C, keepbits, keep_words, codes, doc_offsets,
                           P, b.meta, b.kept_ids, b.T, candbits, cand_words, keys2, key_stride, b.hist, b.emptybits, wide | 2,
                           b.qcount, b.qlist, b.qlist_stride);
    } else if (shift == 11) {
        S2_INVERT(11, uint32_t);
        S2_INVERT(11, unsigned long long);
    } else {
        S2_INVERT(13, uint32_t);
        S2_INVERT(13, unsigned long long);
    }
#undef S2_INVERT
}

// ------------------------------------------------------------------ host side
void plaid_launch_stage2(hipStream_t st, const float *S, int64_t C, const uint32_t *keepbits, int64_t keep_words,
                         const int32_t *probed, int nprobe, const uint32_t *candbits, int64_t cand_words, int64_t P,
                         int64_t N, const int64_t *doc_offsets, const int32_t *codes, int nq, const Stage2Buffers &b,
                         uint64_t *keys2, int64_t key_stride)
{
    (void)probed;
    (void)nprobe;
    // persistent workgroups; enough of them to fill the chip for one query, fewer per query in a large chunk
    const int64_t ntiles = (P + S2W_PASS - 1) / S2W_PASS;
    int64_t gs = (ntiles + 3) / 4;
    const int64_t gcap = nq >= 16 ? 96 : (nq >= 4 ? 320 : 1280);
    if (gs > gcap) gs = gcap;
    hipLaunchKernelGGL(s2_stream_kernel, dim3((unsigned)gs, nq), dim3(S2_THREADS), 0, st, S, C, keepbits, keep_words, codes, N,
                       doc_offsets, P, candbits, cand_words, b.meta, b.kept_ids, b.T, keys2, key_stride, b.hist,
                       b.emptybits);
}
