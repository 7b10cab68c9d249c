// Batched top-m selection on unique 64-bit ranking keys (ascending key = better rank).
//
// Every cut of the pipeline (nprobe centroids per token, ndocs after stage 2, ndocs/4 after
// stage 3, k at the end) is "the m smallest keys of a list".  Lists of up to SEL_SORT_CAP keys are
// sorted by one workgroup in LDS.  Longer lists go through a two-level most-significant-digit
// radix selection that starts below the keys' common prefix (the producer accumulates the AND/OR
// of its keys): level 0 histograms an 11-bit digit over the whole list, level 1 over the keys that
// fell into the boundary bin; keys in lower bins are selected for sure, the remaining boundary
// (normally a handful of exact score ties) is resolved by the finishing workgroup, which falls
// back to an in-block radix selection over global memory if that boundary is still long.
// Nothing is read back to the host; all counts live in device memory.
#include "plaid_internal.h"

#include <math.h>

#define SEL_THREADS 256
#define FIN_THREADS 1024

__device__ __forceinline__ SelState *state_of(SelState *base, int seg) { return base + seg; }

// ------------------------------------------------------------------ AND/OR of a list (when the producer has not)
__global__ __launch_bounds__(SEL_THREADS) void sel_andor_kernel(const uint64_t *__restrict__ keys, int64_t key_stride,
                                                                const int32_t *__restrict__ counts, SelState *state)
{
    const int seg = blockIdx.y;
    const int n = counts[seg];
    const uint64_t *k = keys + (int64_t)seg * key_stride;
    unsigned long long o = 0, no = 0;
    for (int64_t i = (int64_t)blockIdx.x * SEL_THREADS + threadIdx.x; i < n; i += (int64_t)gridDim.x * SEL_THREADS) {
        const unsigned long long v = k[i];
        o |= v;
        no |= ~v;
    }
    for (int d = 1; d < 64; d <<= 1) {
        o |= __shfl_xor(o, d);
        no |= __shfl_xor(no, d);
    }
    if ((threadIdx.x & 63) == 0 && (o | no)) {
        SelState *s = state_of(state, seg);
        atomicOr(&s->key_or, o);
        atomicOr(&s->key_nor, no);
    }
}

__device__ __forceinline__ void digit_plan(const SelState *s, int &shift0, int &width0, int &shift1, int &width1)
{
    const unsigned long long diff = s->key_or & s->key_nor;  // bits in which the keys differ
    const int hi = diff ? 63 - __clzll((long long)diff) : -1;
    width0 = hi + 1 < SEL_RADIX_BITS ? hi + 1 : SEL_RADIX_BITS;
    shift0 = hi + 1 - width0;
    width1 = shift0 < SEL_RADIX_BITS ? shift0 : SEL_RADIX_BITS;
    shift1 = shift0 - width1;
}
__device__ __forceinline__ int digit_of(uint64_t key, int shift, int width)
{
    return (int)((key >> shift) & ((1u << width) - 1u));
}

// ------------------------------------------------------------------ level-0 histogram over the whole list
__global__ __launch_bounds__(SEL_THREADS) void sel_hist0_kernel(const uint64_t *__restrict__ keys, int64_t key_stride,
                                                                const int32_t *__restrict__ counts, int32_t m,
                                                                SelState *state, int32_t *__restrict__ hist)
{
    __shared__ int32_t lh[SEL_BINS];
    const int seg = blockIdx.y;
    SelState *s = state_of(state, seg);
    const int n = counts[seg];
    int shift0, width0, shift1, width1;
    digit_plan(s, shift0, width0, shift1, width1);
    for (int b = threadIdx.x; b < SEL_BINS; b += SEL_THREADS) lh[b] = 0;
    __syncthreads();
    const uint64_t *k = keys + (int64_t)seg * key_stride;
    for (int64_t i = (int64_t)blockIdx.x * SEL_THREADS + threadIdx.x; i < n; i += (int64_t)gridDim.x * SEL_THREADS)
        atomicAdd(&lh[digit_of(k[i], shift0, width0)], 1);
    __syncthreads();
    int32_t *gh = hist + (int64_t)seg * 2 * SEL_BINS;
    for (int b = threadIdx.x; b < SEL_BINS; b += SEL_THREADS)
        if (lh[b]) atomicAdd(&gh[b], lh[b]);
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        s->n_in = n;
        s->m_rem[0] = m < n ? m : n;
        s->shift[0] = shift0;
        s->width[0] = width0;
        s->shift[1] = shift1;
        s->width[1] = width1;
    }
}

// Finds the boundary bin of a histogram: the smallest b with count(bins <= b) >= m_rem.  Every thread of
// the block returns the same (bstar, before).  bstar = SEL_BINS when the whole list is taken.
__device__ void find_boundary(const int32_t *__restrict__ gh, int32_t m_rem, int32_t *scan /* [SEL_THREADS] */,
                              int32_t *res /* [2] */, int &bstar, int &before, int32_t m_cap = 0x7FFFFFFF)
{
    constexpr int PER = SEL_BINS / SEL_THREADS;
    int32_t loc[PER];
    int32_t sum = 0;
    for (int j = 0; j < PER; ++j) {
        loc[j] = gh[threadIdx.x * PER + j];
        sum += loc[j];
    }
    scan[threadIdx.x] = sum;
    if (threadIdx.x == 0) {
        res[0] = SEL_BINS;
        res[1] = 0;
    }
    __syncthreads();
    for (int d = 1; d < SEL_THREADS; d <<= 1) {
        int32_t v = threadIdx.x >= d ? scan[threadIdx.x - d] : 0;
        __syncthreads();
        scan[threadIdx.x] += v;
        __syncthreads();
    }
    const int32_t incl = scan[threadIdx.x], excl = incl - sum;
    if (m_cap != 0x7FFFFFFF) m_rem = m_cap < scan[SEL_THREADS - 1] ? m_cap : scan[SEL_THREADS - 1];  // min(m, #keys)
    if (m_rem > 0 && excl < m_rem && m_rem <= incl) {
        int32_t run = excl;
        for (int j = 0; j < PER; ++j) {
            if (run + loc[j] >= m_rem) {
                res[0] = threadIdx.x * PER + j;
                res[1] = run;
                break;
            }
            run += loc[j];
        }
    }
    if (m_rem <= 0 && threadIdx.x == 0) {
        res[0] = -1;  // take nothing, keep nothing
        res[1] = 0;
    }
    __syncthreads();
    bstar = res[0];
    before = res[1];
    if (bstar == SEL_BINS) before = scan[SEL_THREADS - 1];
}

// ------------------------------------------------------------------ level kernel: split a list by its digit
template <int LEVEL>
__global__ __launch_bounds__(SEL_THREADS) void sel_level_kernel(const uint64_t *__restrict__ keys, int64_t key_stride,
                                                                SelState *state, int32_t *__restrict__ hist,
                                                                uint64_t *__restrict__ sure, int64_t sure_stride,
                                                                uint64_t *__restrict__ list_out, int64_t list_stride)
{
    __shared__ int32_t scan[SEL_THREADS];
    __shared__ int32_t res[2];
    __shared__ int32_t lh[LEVEL == 0 ? SEL_BINS : 1];
    const int seg = blockIdx.y;
    SelState *s = state_of(state, seg);
    const int n = LEVEL == 0 ? s->n_in : s->n_list[0];
    const int32_t m_rem = s->m_rem[LEVEL];
    const int shift = s->shift[LEVEL], width = s->width[LEVEL];
    const int shift_n = s->shift[1], width_n = s->width[1];
    int bstar, before;
    find_boundary(hist + ((int64_t)seg * 2 + LEVEL) * SEL_BINS, m_rem, scan, res, bstar, before);
    if (blockIdx.x == 0 && threadIdx.x == 0) s->m_rem[LEVEL + 1] = m_rem - before;
    if (LEVEL == 0) {
        for (int b = threadIdx.x; b < SEL_BINS; b += SEL_THREADS) lh[b] = 0;
        __syncthreads();
    }
    const uint64_t *k = keys + (int64_t)seg * key_stride;
    uint64_t *my_sure = sure + (int64_t)seg * sure_stride;
    uint64_t *my_out = list_out + (int64_t)seg * list_stride;
    const int lane = threadIdx.x & 63;
    const int64_t n_round = ((int64_t)n + 63) & ~63ll;  // whole waves iterate together (ballots below)
    for (int64_t i = (int64_t)blockIdx.x * SEL_THREADS + threadIdx.x; i < n_round; i += (int64_t)gridDim.x * SEL_THREADS) {
        uint64_t key = 0;
        int cls = 2;  // 0 = surely selected, 1 = boundary, 2 = dropped
        if (i < n) {
            key = k[i];
            const int d = digit_of(key, shift, width);
            cls = d < bstar ? 0 : (d == bstar ? 1 : 2);
        }
        const unsigned long long b0 = __ballot(cls == 0), b1 = __ballot(cls == 1);
        const unsigned long long below = (1ull << lane) - 1ull;
        int base0 = 0, base1 = 0;
        if (lane == 0) {
            if (b0) base0 = atomicAdd(&s->n_sure, __popcll(b0));
            if (b1) base1 = atomicAdd(&s->n_list[LEVEL], __popcll(b1));
        }
        base0 = __shfl(base0, 0);
        base1 = __shfl(base1, 0);
        if (cls == 0) my_sure[base0 + __popcll(b0 & below)] = key;
        if (cls == 1) {
            my_out[base1 + __popcll(b1 & below)] = key;
            if (LEVEL == 0) atomicAdd(&lh[digit_of(key, shift_n, width_n)], 1);
        }
    }
    if (LEVEL == 0) {
        __syncthreads();
        int32_t *gh = hist + ((int64_t)seg * 2 + 1) * SEL_BINS;
        for (int b = threadIdx.x; b < SEL_BINS; b += SEL_THREADS)
            if (lh[b]) atomicAdd(&gh[b], lh[b]);
    }
}

// ------------------------------------------------------------------ finishing workgroup
__device__ void lds_bitonic_sort(uint64_t *s, int n2)
{
    for (int k = 2; k <= n2; k <<= 1)
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int i = threadIdx.x; i < n2; i += FIN_THREADS) {
                const int p = i ^ j;
                if (p > i) {
                    const uint64_t a = s[i], b = s[p];
                    const bool up = (i & k) == 0;
                    if ((a > b) == up) {
                        s[i] = b;
                        s[p] = a;
                    }
                }
            }
            __syncthreads();
        }
}
__device__ __forceinline__ int next_pow2(int n)
{
    int p = 1;
    while (p < n) p <<= 1;
    return p;
}

// DIRECT: the list is the input itself (no levels ran).  Otherwise: sure keys + boundary list1.
template <bool DIRECT>
__global__ __launch_bounds__(FIN_THREADS) void sel_finish_kernel(const uint64_t *__restrict__ keys, int64_t key_stride,
                                                                 const int32_t *__restrict__ counts, int32_t m,
                                                                 SelState *state, const uint64_t *__restrict__ sure,
                                                                 int64_t sure_stride, const uint64_t *__restrict__ list1,
                                                                 int64_t list_stride, uint64_t *__restrict__ out,
                                                                 int64_t out_stride, int32_t *__restrict__ out_counts,
                                                                 int sorted)
{
    __shared__ uint64_t sk[SEL_SORT_CAP];
    __shared__ int32_t h256[256];
    __shared__ int32_t sh[4];
    const int seg = blockIdx.x;
    const uint64_t *bl;
    const uint64_t *sr = nullptr;
    int nb, n_sure, m_rem, top_bit;
    if (DIRECT) {
        bl = keys + (int64_t)seg * key_stride;
        nb = counts[seg];
        n_sure = 0;
        m_rem = m < nb ? m : nb;
        top_bit = 64;
    } else {
        SelState *s = state_of(state, seg);
        bl = list1 + (int64_t)seg * list_stride;
        sr = sure + (int64_t)seg * sure_stride;
        nb = s->n_list[1];
        n_sure = s->n_sure;
        m_rem = s->m_rem[2];
        top_bit = s->shift[1];  // boundary keys agree on every bit at or above this position
    }
    uint64_t *o = out + (int64_t)seg * out_stride;
    const int total_out = n_sure + m_rem;
    if (threadIdx.x == 0) out_counts[seg] = total_out;

    if (n_sure + nb <= SEL_SORT_CAP) {
        // common case: sort the union; the first total_out keys are the answer, in rank order
        const int tot = n_sure + nb, n2 = next_pow2(tot > 1 ? tot : 1);
        for (int i = threadIdx.x; i < n2; i += FIN_THREADS)
            sk[i] = i < n_sure ? sr[i] : (i < tot ? bl[i - n_sure] : PLAID_KEY_MAX);
        __syncthreads();
        lds_bitonic_sort(sk, n2);
        for (int i = threadIdx.x; i < total_out; i += FIN_THREADS) o[i] = sk[i];
        return;
    }

    // long boundary: find the m_rem-th smallest boundary key by 8-bit radix passes over global memory
    uint64_t prefix = 0, pmask = 0;  // bits decided so far
    int r = m_rem;
    int pos = top_bit;
    while (pos > 0 && r > 0) {
        const int w = pos < 8 ? pos : 8;
        pos -= w;
        for (int b = threadIdx.x; b < 256; b += FIN_THREADS) h256[b] = 0;
        __syncthreads();
        for (int i = threadIdx.x; i < nb; i += FIN_THREADS) {
            const uint64_t key = bl[i];
            if ((key & pmask) == prefix) atomicAdd(&h256[(int)((key >> pos) & ((1u << w) - 1u))], 1);
        }
        __syncthreads();
        if (threadIdx.x == 0) {
            int run = 0, b = 0;
            for (; b < (1 << w); ++b) {
                if (run + h256[b] >= r) break;
                run += h256[b];
            }
            sh[0] = b;
            sh[1] = run;
        }
        __syncthreads();
        prefix |= (uint64_t)sh[0] << pos;
        pmask |= (uint64_t)((1u << w) - 1u) << pos;
        r -= sh[1];
        __syncthreads();
    }
    // keys are unique, so after all bits are decided `prefix` (restricted to pmask) is the threshold key itself
    if (threadIdx.x == 0) sh[2] = 0;
    __syncthreads();
    for (int i = threadIdx.x; i < n_sure; i += FIN_THREADS) o[i] = sr[i];
    if (m_rem > 0)
        for (int i = threadIdx.x; i < nb; i += FIN_THREADS) {
            const uint64_t key = bl[i];
            if ((key & pmask) <= prefix) o[n_sure + atomicAdd(&sh[2], 1)] = key;
        }
    __syncthreads();
    if (sorted && total_out <= SEL_SORT_CAP) {
        __threadfence_block();
        const int n2 = next_pow2(total_out > 1 ? total_out : 1);
        for (int i = threadIdx.x; i < n2; i += FIN_THREADS) sk[i] = i < total_out ? o[i] : PLAID_KEY_MAX;
        __syncthreads();
        lds_bitonic_sort(sk, n2);
        for (int i = threadIdx.x; i < total_out; i += FIN_THREADS) o[i] = sk[i];
    }
}

// ------------------------------------------------------------------ global bitonic sort (only for m > SEL_SORT_CAP, sorted)
__global__ void sel_pad_copy_kernel(const uint64_t *__restrict__ src, int64_t src_stride, const int32_t *__restrict__ counts,
                                    uint64_t *__restrict__ dst, int64_t n2)
{
    const int seg = blockIdx.y;
    const int n = counts[seg];
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n2; i += (int64_t)gridDim.x * blockDim.x)
        dst[(int64_t)seg * n2 + i] = i < n ? src[(int64_t)seg * src_stride + i] : PLAID_KEY_MAX;
}
__global__ void sel_bitonic_step_kernel(uint64_t *__restrict__ a, int64_t n2, int64_t k, int64_t j)
{
    uint64_t *s = a + (int64_t)blockIdx.y * n2;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n2; i += (int64_t)gridDim.x * blockDim.x) {
        const int64_t p = i ^ j;
        if (p > i) {
            const uint64_t x = s[i], y = s[p];
            const bool up = (i & k) == 0;
            if ((x > y) == up) {
                s[i] = y;
                s[p] = x;
            }
        }
    }
}
__global__ void sel_copy_back_kernel(const uint64_t *__restrict__ src, int64_t n2, const int32_t *__restrict__ counts,
                                     uint64_t *__restrict__ dst, int64_t dst_stride)
{
    const int seg = blockIdx.y;
    const int n = counts[seg];
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
        dst[(int64_t)seg * dst_stride + i] = src[(int64_t)seg * n2 + i];
}

// ------------------------------------------------------------------ short lists: one workgroup sorts the list in LDS
// Lists of up to SEL_SORT_CAP keys: a workgroup loads the list into LDS padded with PLAID_KEY_MAX to the next power of
// two of its actual length, runs a bitonic network over it (one compare-exchange per thread and pass: thread t owns
// the pair (lo, lo | j) with lo = t with a zero inserted at bit log2(j)), and the first min(m, n) keys are the result
// in rank order.  n log^2 n compare-exchanges instead of the n^2 comparisons of rank counting, and only as much LDS as
// the longest list of the launch needs (the launcher passes it as dynamic shared memory).
// The 64 pairs a wave owns in one pass lie inside one aligned block of 128 keys whenever j <= 64, and a wave owns the
// same blocks in every pass, so those passes (most of the network) need no workgroup barrier: a wave's LDS
// operations complete in program order.  Only the passes with j >= 128 exchange keys between waves.
template <int THREADS>
__device__ __forceinline__ int lds_sort_list(uint64_t *sk, const uint64_t *__restrict__ k, int n)
{
    int n2 = 2;
    while (n2 < n) n2 <<= 1;
    for (int i = threadIdx.x; i < n2; i += THREADS) sk[i] = i < n ? k[i] : PLAID_KEY_MAX;
    __syncthreads();
    const int half = n2 >> 1;
    for (int kk = 2; kk <= n2; kk <<= 1)
        for (int j = kk >> 1; j > 0; j >>= 1) {
            const bool wide = j >= 128;  // uniform over the workgroup
            if (wide)
                __syncthreads();
            else
                __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            for (int t = threadIdx.x; t < half; t += THREADS) {
                const int lo = ((t & ~(j - 1)) << 1) | (t & (j - 1)), hi = lo | j;
                const uint64_t a = sk[lo], b = sk[hi];
                const bool up = (lo & kk) == 0;
                if ((a > b) == up) {
                    sk[lo] = b;
                    sk[hi] = a;
                }
            }
            if (wide) __syncthreads();
        }
    __syncthreads();
    return n2;
}

template <int THREADS>
__global__ __launch_bounds__(THREADS) void sel_sort_kernel(const uint64_t *__restrict__ keys, int64_t key_stride,
                                                           const int32_t *__restrict__ counts, int32_t n_cap, int32_t m,
                                                           uint64_t *__restrict__ out, int64_t out_stride,
                                                           int32_t *__restrict__ out_counts)
{
    extern __shared__ uint64_t sel_sort_lds[];
    const int seg = blockIdx.x;
    int n = counts[seg];
    if (n > n_cap) n = n_cap;
    const int n_out = m < n ? m : n;
    if (threadIdx.x == 0) out_counts[seg] = n_out;
    if (n_out == 0) return;
    lds_sort_list<THREADS>(sel_sort_lds, keys + (int64_t)seg * key_stride, n);
    uint64_t *o = out + (int64_t)seg * out_stride;
    for (int i = threadIdx.x; i < n_out; i += THREADS) o[i] = sel_sort_lds[i];
}

// The same for the final ranking: ids and scores go straight to the caller's buffers, best first, and the
// slots beyond min(k, count) are filled with (-1, -infinity).
template <int THREADS>
__global__ __launch_bounds__(THREADS) void sel_sort_output_kernel(const uint64_t *__restrict__ keys, int64_t key_stride,
                                                                  const int32_t *__restrict__ counts, int32_t n_cap,
                                                                  int32_t k, int32_t *__restrict__ out_ids,
                                                                  float *__restrict__ out_scores)
{
    extern __shared__ uint64_t sel_sort_lds[];
    const int seg = blockIdx.x;
    int n = counts[seg];
    if (n > n_cap) n = n_cap;
    const int n_out = k < n ? k : n;
    int32_t *oi = out_ids + (int64_t)seg * k;
    float *os = out_scores + (int64_t)seg * k;
    for (int j = n_out + threadIdx.x; j < k; j += THREADS) {
        oi[j] = -1;
        os[j] = -INFINITY;
    }
    if (n_out == 0) return;
    lds_sort_list<THREADS>(sel_sort_lds, keys + (int64_t)seg * key_stride, n);
    for (int i = threadIdx.x; i < n_out; i += THREADS) {
        const uint64_t key = sel_sort_lds[i];
        oi[i] = (int32_t)(key & 0xFFFFFFFFu);
        os[i] = plaid_ord_to_score((uint32_t)(key >> 32));
    }
}

// ------------------------------------------------------------------ short lists, few of them: selection by rank counting
// With only a few lists in the launch (single-query latency) one workgroup per list leaves the chip idle and the
// network's passes are a chain of LDS round trips.  Then the n^2 form is quicker: the rank of a key is the number of
// smaller keys (keys are unique), so key j goes to out[rank] when rank < m.  Every workgroup holds the whole list in
// LDS and ranks 32 of its keys, eight lanes sharing the comparisons of one key.
#define RANK_MAX_LISTS 16
#define RANK_KEYS_PER_BLOCK 32
__global__ __launch_bounds__(256) void sel_rank_kernel(const uint64_t *__restrict__ keys, int64_t key_stride,
                                                       const int32_t *__restrict__ counts, int32_t n_cap, int32_t m,
                                                       uint64_t *__restrict__ out, int64_t out_stride,
                                                       int32_t *__restrict__ out_counts)
{
    extern __shared__ uint64_t sk[];
    const int seg = blockIdx.y;
    int n = counts[seg];
    if (n > n_cap) n = n_cap;
    if (blockIdx.x == 0 && threadIdx.x == 0) out_counts[seg] = m < n ? m : n;
    const int j0 = blockIdx.x * RANK_KEYS_PER_BLOCK;
    if (j0 >= n) return;
    const uint64_t *k = keys + (int64_t)seg * key_stride;
    for (int i = threadIdx.x; i < n; i += 256) sk[i] = k[i];
    __syncthreads();
    const int j = j0 + (threadIdx.x >> 3), part = threadIdx.x & 7;
    const uint64_t key = j < n ? sk[j] : PLAID_KEY_MAX;
    int rank = 0;
    for (int i = part; i < n; i += 8) rank += sk[i] < key ? 1 : 0;
    rank += __shfl_xor(rank, 1);
    rank += __shfl_xor(rank, 2);
    rank += __shfl_xor(rank, 4);
    if (part == 0 && j < n && rank < m) out[(int64_t)seg * out_stride + rank] = key;
}

// Rank counting for the final ranking.
__global__ __launch_bounds__(256) void sel_rank_output_kernel(const uint64_t *__restrict__ keys, int64_t key_stride,
                                                              const int32_t *__restrict__ counts, int32_t n_cap, int32_t k,
                                                              int32_t *__restrict__ out_ids, float *__restrict__ out_scores)
{
    extern __shared__ uint64_t sk[];
    const int seg = blockIdx.y;
    int n = counts[seg];
    if (n > n_cap) n = n_cap;
    int32_t *oi = out_ids + (int64_t)seg * k;
    float *os = out_scores + (int64_t)seg * k;
    if (blockIdx.x == 0)
        for (int j = (n < k ? n : k) + threadIdx.x; j < k; j += 256) {
            oi[j] = -1;
            os[j] = -INFINITY;
        }
    const int j0 = blockIdx.x * RANK_KEYS_PER_BLOCK;
    if (j0 >= n) return;
    const uint64_t *kk = keys + (int64_t)seg * key_stride;
    for (int i = threadIdx.x; i < n; i += 256) sk[i] = kk[i];
    __syncthreads();
    const int j = j0 + (threadIdx.x >> 3), part = threadIdx.x & 7;
    const uint64_t key = j < n ? sk[j] : PLAID_KEY_MAX;
    int rank = 0;
    for (int i = part; i < n; i += 8) rank += sk[i] < key ? 1 : 0;
    rank += __shfl_xor(rank, 1);
    rank += __shfl_xor(rank, 2);
    rank += __shfl_xor(rank, 4);
    if (part == 0 && j < n && rank < k) {
        oi[rank] = (int32_t)(key & 0xFFFFFFFFu);
        os[rank] = plaid_ord_to_score((uint32_t)(key >> 32));
    }
}

static inline int64_t sort_pow2(int64_t n)
{
    int64_t p = 2;
    while (p < n) p <<= 1;
    return p;
}

void plaid_launch_rank_output(hipStream_t st, const uint64_t *keys, int64_t key_stride, const int32_t *counts, int nseg,
                              int64_t n_upper, int32_t k, int32_t *out_ids, float *out_scores)
{
    const size_t lds = (size_t)sort_pow2(n_upper) * 8;  // one thread per pair of the padded list, 256 to 1024
    if (nseg <= RANK_MAX_LISTS) {
        const int gx = (int)((n_upper + RANK_KEYS_PER_BLOCK - 1) / RANK_KEYS_PER_BLOCK);
        hipLaunchKernelGGL(sel_rank_output_kernel, dim3(gx > 0 ? gx : 1, nseg), dim3(256), lds, st, keys, key_stride, counts,
                           (int32_t)n_upper, k, out_ids, out_scores);
    } else if (n_upper <= 512)
        hipLaunchKernelGGL(sel_sort_output_kernel<256>, dim3(nseg), dim3(256), lds, st, keys, key_stride, counts,
                           (int32_t)n_upper, k, out_ids, out_scores);
    else if (n_upper <= 1024)
        hipLaunchKernelGGL(sel_sort_output_kernel<512>, dim3(nseg), dim3(512), lds, st, keys, key_stride, counts,
                           (int32_t)n_upper, k, out_ids, out_scores);
    else
        hipLaunchKernelGGL(sel_sort_output_kernel<1024>, dim3(nseg), dim3(1024), lds, st, keys, key_stride, counts,
                           (int32_t)n_upper, k, out_ids, out_scores);
}

// ------------------------------------------------------------------ host side
static inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }
static inline int64_t pow2_at_least(int64_t n)
{
    int64_t p = 1;
    while (p < n) p <<= 1;
    return p;
}

// Scratch of one selection instance comes in two parts: a small head (state + histograms) that must be
// zero before the producer of the keys runs, and a body (sure / boundary lists, sort buffer) that needs no
// initialisation.  The body is only needed for lists longer than SEL_SORT_CAP or more than SEL_SORT_CAP
// sorted results.
size_t plaid_select_zero_bytes(int nseg)
{
    return align256((size_t)nseg * sizeof(SelState)) + align256((size_t)nseg * 2 * SEL_BINS * sizeof(int32_t));
}
size_t plaid_select_body_bytes(int nseg, int64_t n_upper, int32_t m)
{
    size_t b = 0;
    const int64_t mm = m < n_upper ? m : n_upper;
    if (n_upper > SEL_SORT_CAP) b += align256((size_t)nseg * mm * 8) + 2 * align256((size_t)nseg * n_upper * 8);
    if (mm > SEL_SORT_CAP) b += align256((size_t)nseg * pow2_at_least(mm) * 8);
    return b;
}
size_t plaid_select_scratch_bytes(int nseg, int64_t n_upper, int32_t m)
{
    return plaid_select_zero_bytes(nseg) + plaid_select_body_bytes(nseg, n_upper, m);
}

SelScratch plaid_select_scratch_carve2(void *zero_base, void *body_base, int nseg, int64_t n_upper, int32_t m)
{
    SelScratch sc{};
    char *z = (char *)zero_base;
    sc.state = (SelState *)z;
    sc.hist = (int32_t *)(z + align256((size_t)nseg * sizeof(SelState)));
    char *p = (char *)body_base;
    const int64_t mm = m < n_upper ? m : n_upper;
    if (n_upper > SEL_SORT_CAP) {
        sc.sure = (uint64_t *)p;
        sc.sure_stride = mm;
        p += align256((size_t)nseg * mm * 8);
        sc.list0 = (uint64_t *)p;
        p += align256((size_t)nseg * n_upper * 8);
        sc.list1 = (uint64_t *)p;
        p += align256((size_t)nseg * n_upper * 8);
        sc.list_stride = n_upper;
    }
    sc.sortbuf = (mm > SEL_SORT_CAP) ? (uint64_t *)p : nullptr;
    return sc;
}
SelScratch plaid_select_scratch_carve(void *base, int nseg, int64_t n_upper, int32_t m)
{
    return plaid_select_scratch_carve2(base, (char *)base + plaid_select_zero_bytes(nseg), nseg, n_upper, m);
}

static int blocks_for(int64_t n, int nseg)
{
    int64_t b = (n + SEL_THREADS * 8 - 1) / (SEL_THREADS * 8);
    const int64_t cap = nseg >= 16 ? 64 : (nseg >= 4 ? 256 : 1024);
    if (b > cap) b = cap;
    if (b < 1) b = 1;
    return (int)b;
}

void plaid_launch_select(hipStream_t st, const uint64_t *keys, int64_t key_stride, const int32_t *counts, int nseg,
                         int64_t n_upper, int32_t m, uint64_t *out, int64_t out_stride, int32_t *out_counts, int sorted,
                         const SelScratch &sc, int state_ready)
{
    // the caller zeroes state + hist (plaid_launch_fill_u32 over the head of the scratch) before the
    // producer runs; see search.hip
    if (n_upper <= SEL_SORT_CAP) {
        const size_t lds = (size_t)sort_pow2(n_upper) * 8;
        if (nseg <= RANK_MAX_LISTS) {
            const int gx = (int)((n_upper + RANK_KEYS_PER_BLOCK - 1) / RANK_KEYS_PER_BLOCK);
            hipLaunchKernelGGL(sel_rank_kernel, dim3(gx > 0 ? gx : 1, nseg), dim3(256), lds, st, keys, key_stride, counts,
                               (int32_t)n_upper, m, out, out_stride, out_counts);
        } else if (n_upper <= 512)
            hipLaunchKernelGGL(sel_sort_kernel<256>, dim3(nseg), dim3(256), lds, st, keys, key_stride, counts,
                               (int32_t)n_upper, m, out, out_stride, out_counts);
        else if (n_upper <= 1024)
            hipLaunchKernelGGL(sel_sort_kernel<512>, dim3(nseg), dim3(512), lds, st, keys, key_stride, counts,
                               (int32_t)n_upper, m, out, out_stride, out_counts);
        else
            hipLaunchKernelGGL(sel_sort_kernel<1024>, dim3(nseg), dim3(1024), lds, st, keys, key_stride, counts,
                               (int32_t)n_upper, m, out, out_stride, out_counts);
        return;
    } else {
        const int gx = blocks_for(n_upper, nseg);
        if (!state_ready)
            hipLaunchKernelGGL(sel_andor_kernel, dim3(gx, nseg), dim3(SEL_THREADS), 0, st, keys, key_stride, counts,
                               sc.state);
        hipLaunchKernelGGL(sel_hist0_kernel, dim3(gx, nseg), dim3(SEL_THREADS), 0, st, keys, key_stride, counts, m,
                           sc.state, sc.hist);
        hipLaunchKernelGGL(sel_level_kernel<0>, dim3(gx, nseg), dim3(SEL_THREADS), 0, st, keys, key_stride, sc.state,
                           sc.hist, sc.sure, sc.sure_stride, sc.list0, sc.list_stride);
        const int gx1 = gx > 16 ? 16 : gx;
        hipLaunchKernelGGL(sel_level_kernel<1>, dim3(gx1, nseg), dim3(SEL_THREADS), 0, st, sc.list0, sc.list_stride,
                           sc.state, sc.hist, sc.sure, sc.sure_stride, sc.list1, sc.list_stride);
        hipLaunchKernelGGL(sel_finish_kernel<false>, dim3(nseg), dim3(FIN_THREADS), 0, st, keys, key_stride, counts, m,
                           sc.state, sc.sure, sc.sure_stride, sc.list1, sc.list_stride, out, out_stride, out_counts,
                           sorted);
    }
    const int64_t mm = m < n_upper ? m : n_upper;
    if (sorted && mm > SEL_SORT_CAP) {
        // rare: more than SEL_SORT_CAP results in rank order -> bitonic network in global memory
        uint64_t *buf = sc.sortbuf;
        const int64_t n2 = pow2_at_least(mm);
        const int gx = (int)((n2 + 255) / 256 > 1024 ? 1024 : (n2 + 255) / 256);
        hipLaunchKernelGGL(sel_pad_copy_kernel, dim3(gx, nseg), dim3(256), 0, st, out, out_stride, out_counts, buf, n2);
        for (int64_t k = 2; k <= n2; k <<= 1)
            for (int64_t j = k >> 1; j > 0; j >>= 1)
                hipLaunchKernelGGL(sel_bitonic_step_kernel, dim3(gx, nseg), dim3(256), 0, st, buf, n2, k, j);
        hipLaunchKernelGGL(sel_copy_back_kernel, dim3(gx, nseg), dim3(256), 0, st, buf, n2, out_counts, out, out_stride);
    }
}

// =================================================================================================
// Stage-2 selection: the ndocs best candidates out of up to P keys plus the empty-bag candidates.
//
// The producer has already counted the keys into SEL_BINS score bins (bin 0 = best), so the cut is
// found without another pass: keys in bins before the boundary bin are selected for sure, the
// boundary bin (normally a few hundred keys) is sorted by the finishing workgroup.  Exact score
// ties are common (passages with the same surviving centroids score identically), so a boundary
// bin can be long: then one digit pass over its keys -- starting at the highest bit in which they
// differ, which skips the tied score bits and lands in the passage id -- cuts it down first.
// Candidates with an empty bag (-infinity) are appended last, in passage-id order, straight from
// their bitmap.
// =================================================================================================
__global__ __launch_bounds__(SEL_THREADS) void sel2_filter_kernel(const uint64_t *__restrict__ keys, int64_t key_stride,
                                                                  const uint32_t *__restrict__ candbits, int64_t cand_words,
                                                                  int64_t P, int32_t m, const S2Meta *__restrict__ meta,
                                                                  const int32_t *__restrict__ hist, Sel2State *state,
                                                                  uint64_t *__restrict__ out, int64_t out_stride,
                                                                  uint64_t *__restrict__ blist, int64_t blist_stride)
{
    __shared__ int32_t scan[SEL_THREADS];
    __shared__ int32_t res[2];
    const int seg = blockIdx.y;
    Sel2State *s = state + seg;
    const S2Meta mt = meta[seg];
    if (mt.K == 0) return;  // no surviving centroid: no valid key, the state stays zero and the fill takes over
    int bstar, before;
    find_boundary(hist + (int64_t)seg * SEL_BINS, 0, scan, res, bstar, before, m);  // takes min(m, number of keys)
    const int32_t n_keys = scan[SEL_THREADS - 1];
    if (blockIdx.x == 0 && threadIdx.x == 0) s->m_rem = (m < n_keys ? m : n_keys) - before;
    if (n_keys == 0) return;
    const uint32_t *k = reinterpret_cast<const uint32_t *>(keys + (int64_t)seg * key_stride);  // score word of passage i
    const uint32_t *cb = candbits + (int64_t)seg * cand_words;
    uint64_t *my_out = out + (int64_t)seg * out_stride;
    uint64_t *my_bl = blist + (int64_t)seg * blist_stride;
    const int lane = threadIdx.x & 63;
    // A wave takes SEL2_GROUPS x 64 consecutive slots per step and reserves its output positions with one pair of
    // counter updates per step (the updates return a value, so their round trip is the step's latency).
    constexpr int SEL2_GROUPS = 8;
    const int64_t wave_id = (int64_t)blockIdx.x * (SEL_THREADS / 64) + __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int64_t n_waves = (int64_t)gridDim.x * (SEL_THREADS / 64);
    unsigned long long o = 0, no = 0;
    for (int64_t i0 = wave_id * (64 * SEL2_GROUPS); i0 < P; i0 += n_waves * (64 * SEL2_GROUPS)) {  // uniform per wave
        uint64_t key[SEL2_GROUPS];
        int cls[SEL2_GROUPS];  // 0 = surely selected, 1 = boundary, 2 = dropped
        unsigned long long b0[SEL2_GROUPS], b1[SEL2_GROUPS];
        int n0 = 0, n1 = 0;
        // word i is meaningful only when passage i is a candidate; it then holds its score word or "no score".  The
        // candidate bits and the score words are requested together (a word that means nothing is read and dropped): one
        // round trip to memory per step.
        uint32_t cw[SEL2_GROUPS], sw[SEL2_GROUPS];
#pragma unroll
        for (int u = 0; u < SEL2_GROUPS; ++u) {
            const int64_t i = i0 + 64 * u + lane;
            cw[u] = i < P ? cb[i >> 5] : 0u;
            sw[u] = i < P ? k[i] : PLAID_S2_NO_SCORE;
        }
#pragma unroll
        for (int u = 0; u < SEL2_GROUPS; ++u) {
            const int64_t i = i0 + 64 * u + lane;
            key[u] = PLAID_KEY_MAX;
            if (((cw[u] >> (i & 31)) & 1u) && sw[u] != PLAID_S2_NO_SCORE) key[u] = ((uint64_t)sw[u] << 32) | (uint32_t)i;
        }
#pragma unroll
        for (int u = 0; u < SEL2_GROUPS; ++u) {
            cls[u] = 2;
            if (key[u] != PLAID_KEY_MAX) {
                const int d = plaid_s2_bin(plaid_ord_to_score((uint32_t)(key[u] >> 32)), mt.bin_hi, mt.bin_scale);
                cls[u] = d < bstar ? 0 : (d == bstar ? 1 : 2);
            }
            b0[u] = __ballot(cls[u] == 0);
            b1[u] = __ballot(cls[u] == 1);
            n0 += __popcll(b0[u]);
            n1 += __popcll(b1[u]);
        }
        const unsigned long long below = (1ull << lane) - 1ull;
        int base0 = 0, base1 = 0;
        if (lane == 0) {
            if (n0) base0 = atomicAdd(&s->n_sure, n0);
            if (n1) base1 = atomicAdd(&s->n_b, n1);
        }
        base0 = __shfl(base0, 0);
        base1 = __shfl(base1, 0);
#pragma unroll
        for (int u = 0; u < SEL2_GROUPS; ++u) {
            if (cls[u] == 0) my_out[base0 + __popcll(b0[u] & below)] = key[u];
            if (cls[u] == 1) {
                my_bl[base1 + __popcll(b1[u] & below)] = key[u];
                o |= key[u];
                no |= ~key[u];
            }
            base0 += __popcll(b0[u]);
            base1 += __popcll(b1[u]);
        }
    }
    for (int d = 1; d < 64; d <<= 1) {
        o |= __shfl_xor(o, d);
        no |= __shfl_xor(no, d);
    }
    if (lane == 0 && (o | no)) {
        atomicOr(&s->b_or, o);
        atomicOr(&s->b_nor, no);
    }
}

// A boundary list longer than this goes through a digit pass (all workgroups of the query) before the finishing
// workgroup sorts what is left: far below what that workgroup could sort (SEL_SORT_CAP), because its sort is the one
// serial step of the selection.  Two such passes can be chained (LEVEL 1 reads the bin filter's list, LEVEL 2 the list
// LEVEL 1 leaves): when a few distinct scores are shared by very many passages, the first digit falls into the score
// bits and leaves one whole tie group, the second falls into the passage-id bits and leaves 2^-11 of it.
#define SEL2_DIGIT_MIN 1024
#define SEL2_SECOND_MIN_PASSAGES (1 << 19)  // indexes with more passages than this get the second digit pass
template <int LEVEL>
__device__ __forceinline__ int sel2_level_input(const Sel2State *s, int &m_rem)
{
    m_rem = LEVEL == 1 ? s->m_rem : s->m_rem1;
    // (LEVEL 2 has work only when LEVEL 1 had: n_b1 is zero otherwise)
    return LEVEL == 1 ? s->n_b : s->n_b1;
}
template <int LEVEL>
__device__ __forceinline__ void sel2_digit_plan(const Sel2State *s, int &shift, int &width)
{
    const unsigned long long diff = LEVEL == 1 ? s->b_or & s->b_nor : s->b_or1 & s->b_nor1;
    const int hi = diff ? 63 - __clzll((long long)diff) : -1;
    width = hi + 1 < SEL_RADIX_BITS ? hi + 1 : SEL_RADIX_BITS;
    shift = hi + 1 - width;
}

// Digit histogram of an over-long boundary list (no-op otherwise).
template <int LEVEL>
__global__ __launch_bounds__(SEL_THREADS) void sel2_digit_hist_kernel(const uint64_t *__restrict__ blist,
                                                                      int64_t blist_stride, Sel2State *state,
                                                                      int32_t *__restrict__ hist1)
{
    __shared__ int32_t lh[SEL_BINS];
    const int seg = blockIdx.y;
    Sel2State *s = state + seg;
    int m_rem;
    const int n = sel2_level_input<LEVEL>(s, m_rem);
    if (n <= SEL2_DIGIT_MIN) return;
    int shift, width;
    sel2_digit_plan<LEVEL>(s, shift, width);
    for (int b = threadIdx.x; b < SEL_BINS; b += SEL_THREADS) lh[b] = 0;
    __syncthreads();
    const uint64_t *k = blist + (int64_t)seg * blist_stride;
    for (int64_t i = (int64_t)blockIdx.x * SEL_THREADS + threadIdx.x; i < n; i += (int64_t)gridDim.x * SEL_THREADS)
        atomicAdd(&lh[digit_of(k[i], shift, width)], 1);
    __syncthreads();
    int32_t *gh = hist1 + (int64_t)seg * SEL_BINS;
    for (int b = threadIdx.x; b < SEL_BINS; b += SEL_THREADS)
        if (lh[b]) atomicAdd(&gh[b], lh[b]);
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        if (LEVEL == 1) s->shift1 = shift, s->width1 = width;
        else s->shift2 = shift, s->width2 = width;
    }
}

// Digit filter of an over-long boundary list (no-op otherwise): smaller digits are selected, the boundary digit
// goes to blist1 (LEVEL 1 also records in which bits the keys it leaves differ, for LEVEL 2's plan).
template <int LEVEL>
__global__ __launch_bounds__(SEL_THREADS) void sel2_digit_filter_kernel(const uint64_t *__restrict__ blist,
                                                                        int64_t blist_stride, Sel2State *state,
                                                                        const int32_t *__restrict__ hist1,
                                                                        uint64_t *__restrict__ out, int64_t out_stride,
                                                                        uint64_t *__restrict__ blist1,
                                                                        int64_t blist1_stride)
{
    __shared__ int32_t scan[SEL_THREADS];
    __shared__ int32_t res[2];
    const int seg = blockIdx.y;
    Sel2State *s = state + seg;
    int32_t m_rem;
    const int n = sel2_level_input<LEVEL>(s, m_rem);
    if (n <= SEL2_DIGIT_MIN) return;
    int shift, width;
    sel2_digit_plan<LEVEL>(s, shift, width);
    int bstar, before;
    find_boundary(hist1 + (int64_t)seg * SEL_BINS, m_rem, scan, res, bstar, before);
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        if (LEVEL == 1) s->m_rem1 = m_rem - before;
        else s->m_rem2 = m_rem - before;
    }
    int32_t *n_left = LEVEL == 1 ? &s->n_b1 : &s->n_b2;
    const uint64_t *k = blist + (int64_t)seg * blist_stride;
    uint64_t *my_out = out + (int64_t)seg * out_stride;
    uint64_t *my_bl = blist1 + (int64_t)seg * blist1_stride;
    const int lane = threadIdx.x & 63;
    const int64_t n_round = ((int64_t)n + 63) & ~63ll;
    unsigned long long o = 0, no = 0;
    for (int64_t i = (int64_t)blockIdx.x * SEL_THREADS + threadIdx.x; i < n_round; i += (int64_t)gridDim.x * SEL_THREADS) {
        uint64_t key = 0;
        int cls = 2;
        if (i < n) {
            key = k[i];
            const int d = digit_of(key, shift, width);
            cls = d < bstar ? 0 : (d == bstar ? 1 : 2);
        }
        const unsigned long long b0 = __ballot(cls == 0), b1 = __ballot(cls == 1);
        const unsigned long long below = (1ull << lane) - 1ull;
        int base0 = 0, base1 = 0;
        if (lane == 0) {
            if (b0) base0 = atomicAdd(&s->n_sure, __popcll(b0));
            if (b1) base1 = atomicAdd(n_left, __popcll(b1));
        }
        base0 = __shfl(base0, 0);
        base1 = __shfl(base1, 0);
        if (cls == 0) my_out[base0 + __popcll(b0 & below)] = key;
        if (cls == 1) {
            my_bl[base1 + __popcll(b1 & below)] = key;
            o |= key;
            no |= ~key;
        }
    }
    if (LEVEL == 1) {
        for (int d = 1; d < 64; d <<= 1) {
            o |= __shfl_xor(o, d);
            no |= __shfl_xor(no, d);
        }
        if (lane == 0 && (o | no)) {
            atomicOr(&s->b_or1, o);
            atomicOr(&s->b_nor1, no);
        }
    }
}

// One workgroup per query: finish the boundary list, then append empty-bag candidates in pid order.
__global__ __launch_bounds__(FIN_THREADS) void sel2_finish_kernel(const uint64_t *__restrict__ blist, int64_t blist_stride,
                                                                  const uint64_t *__restrict__ blist1,
                                                                  int64_t blist1_stride, const Sel2State *state,
                                                                  const uint32_t *__restrict__ emptybits,
                                                                  int64_t cand_words, int64_t P, int32_t m, int levels,
                                                                  uint64_t *__restrict__ out, int64_t out_stride,
                                                                  int32_t *__restrict__ out_counts)
{
    __shared__ uint64_t sk[SEL_SORT_CAP];
    __shared__ int32_t h256[256];
    __shared__ int32_t sh[4];
    const int seg = blockIdx.x;
    const Sel2State *s = state + seg;
    // how many digit filters this query's boundary list went through (levels: how many were launched); the second one
    // writes where the first one read
    const int done = (levels >= 1 && s->n_b > SEL2_DIGIT_MIN) ? ((levels >= 2 && s->n_b1 > SEL2_DIGIT_MIN) ? 2 : 1) : 0;
    const uint64_t *bl = done == 1 ? blist1 + (int64_t)seg * blist1_stride : blist + (int64_t)seg * blist_stride;
    const int nb = done == 2 ? s->n_b2 : (done == 1 ? s->n_b1 : s->n_b);
    const int m_rem = done == 2 ? s->m_rem2 : (done == 1 ? s->m_rem1 : s->m_rem);
    const int n_sure = s->n_sure;
    // boundary keys agree on every bit at or above this position
    const int top_bit = done == 2 ? s->shift2 : (done == 1 ? s->shift1 : 64);
    uint64_t *o = out + (int64_t)seg * out_stride;
    int total = n_sure + m_rem;

    if (nb <= SEL_SORT_CAP) {
        const int n2 = next_pow2(nb > 1 ? nb : 1);
        for (int i = threadIdx.x; i < n2; i += FIN_THREADS) sk[i] = i < nb ? bl[i] : PLAID_KEY_MAX;
        __syncthreads();
        lds_bitonic_sort(sk, n2);
        for (int i = threadIdx.x; i < m_rem; i += FIN_THREADS) o[n_sure + i] = sk[i];
    } else {
        // still long (huge tie groups): radix selection over global memory by this one workgroup.  The keys of such a
        // list mostly share their digit (that is what made the list long), so a wave whose keys all have one digit
        // counts them with a single LDS update instead of 64 updates of one address.
        uint64_t prefix = 0, pmask = 0;
        int r = m_rem;
        int pos = top_bit;
        const int lane = threadIdx.x & 63;
        const int nb_round = (nb + FIN_THREADS - 1) / FIN_THREADS * FIN_THREADS;  // whole waves in every step
        while (pos > 0 && r > 0) {
            const int w = pos < 8 ? pos : 8;
            pos -= w;
            for (int b = threadIdx.x; b < 256; b += FIN_THREADS) h256[b] = 0;
            __syncthreads();
            for (int i0 = threadIdx.x; i0 < nb_round; i0 += 4 * FIN_THREADS) {
                uint64_t key[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int i = i0 + u * FIN_THREADS;
                    key[u] = i < nb ? bl[i] : ~prefix;  // a key past the end never matches the prefix
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int i = i0 + u * FIN_THREADS;
                    const int dgt = (i < nb && (key[u] & pmask) == prefix) ? (int)((key[u] >> pos) & ((1u << w) - 1u)) : -1;
                    const int first = __builtin_amdgcn_readfirstlane(dgt);
                    const unsigned long long same = __ballot(dgt == first);
                    if (same == __ballot(true)) {  // uniform digit (or no key in play) in this wave
                        if (lane == (int)__builtin_ctzll(same) && first >= 0) atomicAdd(&h256[first], __popcll(same));
                    } else if (dgt >= 0) {
                        atomicAdd(&h256[dgt], 1);
                    }
                }
            }
            __syncthreads();
            if (threadIdx.x == 0) {
                int run = 0, b = 0;
                for (; b < (1 << w); ++b) {
                    if (run + h256[b] >= r) break;
                    run += h256[b];
                }
                sh[0] = b;
                sh[1] = run;
            }
            __syncthreads();
            prefix |= (uint64_t)sh[0] << pos;
            pmask |= (uint64_t)((1u << w) - 1u) << pos;
            r -= sh[1];
            __syncthreads();
        }
        if (threadIdx.x == 0) sh[2] = 0;
        __syncthreads();
        if (m_rem > 0)
            for (int i0 = threadIdx.x; i0 < nb_round; i0 += FIN_THREADS) {
                const uint64_t key = i0 < nb ? bl[i0] : 0;
                const bool take = i0 < nb && (key & pmask) <= prefix;
                const unsigned long long tk = __ballot(take);
                if (tk) {  // one counter update per wave
                    int base = 0;
                    if (lane == (int)__builtin_ctzll(tk)) base = atomicAdd(&sh[2], __popcll(tk));
                    base = __shfl(base, (int)__builtin_ctzll(tk));
                    if (take) o[n_sure + base + __popcll(tk & ((1ull << lane) - 1ull))] = key;
                }
            }
    }
    __syncthreads();

    // empty-bag candidates: ascending pid, until m slots are filled.  One bitmap word per thread and round; positions
    // from a wave-level prefix sum of the popcounts plus the wave totals.
    if (total < m) {
        int32_t *wsum = h256;  // [FIN_THREADS / 64] wave totals
        const uint32_t *eb = emptybits + (int64_t)seg * cand_words;
        const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
        for (int64_t w0 = 0; w0 < cand_words && total < m; w0 += FIN_THREADS) {
            const int64_t w = w0 + threadIdx.x;
            uint32_t v = 0u;
            if (w < cand_words) {
                v = eb[w];
                if ((w + 1) * 32 > P) {
                    const int64_t keep = P - w * 32;
                    v = keep <= 0 ? 0u : (keep >= 32 ? v : (v & ((1u << keep) - 1u)));
                }
            }
            const int cnt = __popc(v);
            int incl = cnt;
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                const int t = __shfl_up(incl, d);
                if (lane >= d) incl += t;
            }
            __syncthreads();  // the previous round's readers of wsum are done
            if (lane == 63) wsum[wave] = incl;
            __syncthreads();
            int pos = total + incl - cnt, all = 0;
            for (int wv = 0; wv < FIN_THREADS / 64; ++wv) {
                const int t = wsum[wv];
                if (wv < wave) pos += t;
                all += t;
            }
            while (v && pos < m) {
                const int bit = __ffs(v) - 1;
                v &= v - 1;
                o[pos++] = plaid_make_key(-INFINITY, (uint32_t)(w * 32 + bit));
            }
            total = total + all < m ? total + all : m;  // uniform: every thread adds the same wave totals
        }
    }
    if (threadIdx.x == 0) out_counts[seg] = total;
}

void plaid_launch_select2(hipStream_t st, uint64_t *keys2, int64_t key_stride, const uint32_t *candbits, int nq, int64_t P,
                          int64_t cand_words, int32_t m, const Stage2Buffers &b, uint64_t *out, int64_t out_stride,
                          int32_t *out_counts)
{
    const int gx = blocks_for(P, nq);
    hipLaunchKernelGGL(sel2_filter_kernel, dim3(gx, nq), dim3(SEL_THREADS), 0, st, keys2, key_stride, candbits, cand_words, P,
                       m, b.meta, b.hist, b.state, out, out_stride, b.blist, P);
    // Digit filters: only a boundary list longer than SEL2_DIGIT_MIN makes them do anything.  The second pair is worth its
    // two launches for large indexes (a tie group can be as long as the index) in launches of several queries; otherwise
    // the query's finishing workgroup handles a long remainder alone (same result).  keys2 serves as the first
    // filter's output list, b.blist (its input) as the second one's.
    const int levels = P > SEL2_DIGIT_MIN ? ((nq >= 8 && P > SEL2_SECOND_MIN_PASSAGES) ? 2 : 1) : 0;
    if (levels >= 1) {
        hipLaunchKernelGGL(sel2_digit_hist_kernel<1>, dim3(gx, nq), dim3(SEL_THREADS), 0, st, b.blist, P, b.state, b.hist1);
        hipLaunchKernelGGL(sel2_digit_filter_kernel<1>, dim3(gx, nq), dim3(SEL_THREADS), 0, st, b.blist, P, b.state, b.hist1,
                           out, out_stride, keys2, key_stride);
    }
    if (levels >= 2) {
        hipLaunchKernelGGL(sel2_digit_hist_kernel<2>, dim3(gx, nq), dim3(SEL_THREADS), 0, st, keys2, key_stride, b.state, b.hist2);
        hipLaunchKernelGGL(sel2_digit_filter_kernel<2>, dim3(gx, nq), dim3(SEL_THREADS), 0, st, keys2, key_stride, b.state,
                           b.hist2, out, out_stride, b.blist, P);
    }
    hipLaunchKernelGGL(sel2_finish_kernel, dim3(nq), dim3(FIN_THREADS), 0, st, b.blist, P, keys2, key_stride, b.state,
                       b.emptybits, cand_words, P, m, levels, out, out_stride, out_counts);
}
