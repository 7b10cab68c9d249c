// Candidate generation, second half (Section 4.1): the candidate set of a query is the union of the
// inverted lists (unique passage ids per centroid) of its probed centroids.  It is kept as a bitmap
// over passage ids, which deduplicates for free and is already in ascending pid order for stage 2.
//
// The concatenation of the probed lists is treated as one flat work range: a prefix sum of the list
// lengths sits in LDS and each thread finds its (list, element) by binary search, so one long head
// list and a hundred short ones balance across the whole grid.
#include "plaid_internal.h"

#define IVF_THREADS 256
#define IVF_BATCH 1024  // lists handled per LDS round

__global__ __launch_bounds__(IVF_THREADS) void ivf_union_kernel(const int32_t *__restrict__ uniq,
                                                                const int32_t *__restrict__ n_uniq, int uniq_stride,
                                                                const int64_t *__restrict__ ivf_offsets,
                                                                const int32_t *__restrict__ ivf_pids,
                                                                uint32_t *__restrict__ candbits, int64_t cand_words)
{
    __shared__ int64_t start[IVF_BATCH];
    __shared__ int64_t pref[IVF_BATCH + 1];
    const int q = blockIdx.y;
    const int nu = n_uniq[q];
    uint32_t *bits = candbits + (int64_t)q * cand_words;
    for (int u0 = 0; u0 < nu; u0 += IVF_BATCH) {
        const int nb = nu - u0 < IVF_BATCH ? nu - u0 : IVF_BATCH;
        for (int t = threadIdx.x; t < nb; t += IVF_THREADS) {
            const int32_t c = uniq[(int64_t)q * uniq_stride + u0 + t];
            const int64_t s = ivf_offsets[c];
            start[t] = s;
            pref[t + 1] = ivf_offsets[c + 1] - s;
        }
        __syncthreads();
        if (threadIdx.x == 0) {
            pref[0] = 0;
            for (int t = 0; t < nb; ++t) pref[t + 1] += pref[t];
        }
        __syncthreads();
        const int64_t total = pref[nb];
        const int lane = threadIdx.x & 63;
        const int64_t total_round = (total + 63) & ~63ll;  // whole waves iterate together (shuffles below)
        for (int64_t w = (int64_t)blockIdx.x * IVF_THREADS + threadIdx.x; w < total_round; w += (int64_t)gridDim.x * IVF_THREADS) {
            uint32_t my_word = 0xFFFFFFFFu, my_bits = 0u;
            if (w < total) {
                int lo = 0, hi = nb;  // largest lo with pref[lo] <= w
                while (hi - lo > 1) {
                    const int mid = (lo + hi) >> 1;
                    if (pref[mid] <= w) lo = mid;
                    else hi = mid;
                }
                const uint32_t pid = (uint32_t)ivf_pids[start[lo] + (w - pref[lo])];
                my_word = pid >> 5;
                my_bits = 1u << (pid & 31);
            }
            // lists are ascending, so neighbouring lanes mostly hit the same bitmap word: a segmented OR over
            // runs of equal words leaves one atomic per run (a dense head list: 2 per wave instead of 64)
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                const uint32_t ow = __shfl_up(my_word, d), ob = __shfl_up(my_bits, d);
                if (lane >= d && ow == my_word) my_bits |= ob;
            }
            const uint32_t nw = __shfl_down(my_word, 1);
            const bool last = lane == 63 || nw != my_word;
            if (last && my_word != 0xFFFFFFFFu) {
                uint32_t *word = bits + my_word;
                if ((*word & my_bits) != my_bits) atomicOr(word, my_bits);  // a stale read only costs a redundant atomic
            }
        }
        __syncthreads();
    }
}

void plaid_launch_ivf_union(hipStream_t st, const int32_t *uniq, const int32_t *n_uniq, int uniq_stride,
                            const int64_t *ivf_offsets, const int32_t *ivf_pids, int nq, uint32_t *candbits,
                            int64_t cand_words)
{
    const int gx = nq >= 16 ? 32 : (nq >= 4 ? 128 : 512);
    hipLaunchKernelGGL(ivf_union_kernel, dim3(gx, nq), dim3(IVF_THREADS), 0, st, uniq, n_uniq, uniq_stride, ivf_offsets,
                       ivf_pids, candbits, cand_words);
}
