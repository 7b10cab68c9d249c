// Vanilla ColBERTv2 candidate generation (Section 4.1), the baseline PLAID is compared with: the inverted list of a
// centroid holds the ids of the EMBEDDINGS assigned to it, so the candidate passages of a query are found by walking
// the embedding lists of its probed centroids and looking up the passage of every embedding.
#include "plaid_internal.h"

// probebits[q] = bitmap over the centroids of the query's distinct probed centroids (zero on entry).
__global__ __launch_bounds__(256) void van_probe_mask_kernel(const int32_t *__restrict__ uniq, const int32_t *__restrict__ n_uniq,
                                                             int uniq_stride, uint32_t *__restrict__ probebits, int64_t keep_words)
{
    const int q = blockIdx.x;
    const int nu = n_uniq[q];
    for (int u = threadIdx.x; u < nu; u += blockDim.x) {
        const uint32_t c = (uint32_t)uniq[(int64_t)q * uniq_stride + u];
        atomicOr(&probebits[(int64_t)q * keep_words + (c >> 5)], 1u << (c & 31));
    }
}

// candbits[q] |= passages owning an embedding of the probed centroids' embedding lists.  The lists of a query form one
// flat range of work (prefix sums of the list lengths in LDS, a thread finds its list by binary search), spread over
// the grid's x dimension.  Consecutive embeddings mostly belong to one passage: a bit already seen set is not set again.
#define VAN_BATCH 256
__global__ __launch_bounds__(256) void van_union_kernel(const int32_t *__restrict__ uniq, const int32_t *__restrict__ n_uniq,
                                                        int uniq_stride, const int64_t *__restrict__ eoff,
                                                        const int32_t *__restrict__ eids, const int32_t *__restrict__ tok2pid,
                                                        uint32_t *__restrict__ candbits, int64_t cand_words)
{
    __shared__ int64_t start[VAN_BATCH];
    __shared__ int64_t pref[VAN_BATCH + 1];
    const int q = blockIdx.y;
    const int nu = n_uniq[q];
    uint32_t *bits = candbits + (int64_t)q * cand_words;
    for (int u0 = 0; u0 < nu; u0 += VAN_BATCH) {
        const int nb = nu - u0 < VAN_BATCH ? nu - u0 : VAN_BATCH;
        __syncthreads();
        if ((int)threadIdx.x < nb) {
            const int32_t c = uniq[(int64_t)q * uniq_stride + u0 + threadIdx.x];
            start[threadIdx.x] = eoff[c];
            pref[threadIdx.x + 1] = eoff[c + 1] - eoff[c];
        }
        __syncthreads();
        if (threadIdx.x == 0) {
            pref[0] = 0;
            for (int t = 0; t < nb; ++t) pref[t + 1] += pref[t];
        }
        __syncthreads();
        const int64_t total = pref[nb];
        for (int64_t w = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; w < total; w += (int64_t)gridDim.x * blockDim.x) {
            int lo = 0, hi = nb;  // largest lo with pref[lo] <= w
            while (hi - lo > 1) {
                const int mid = (lo + hi) >> 1;
                if (pref[mid] <= w) lo = mid;
                else hi = mid;
            }
            const uint32_t pid = (uint32_t)tok2pid[eids[start[lo] + (w - pref[lo])]];
            uint32_t *word = bits + (pid >> 5);
            const uint32_t bit = 1u << (pid & 31);
            if ((*word & bit) == 0u) atomicOr(word, bit);  // a stale read only costs a redundant atomic
        }
    }
}

void plaid_launch_vanilla_candidates(hipStream_t st, const int32_t *uniq, const int32_t *n_uniq, int uniq_stride,
                                     const int64_t *eoff, const int32_t *eids, const int32_t *tok2pid, int nq, int64_t keep_words,
                                     uint32_t *probebits, uint32_t *candbits, int64_t cand_words)
{
    hipLaunchKernelGGL(van_probe_mask_kernel, dim3(nq), dim3(256), 0, st, uniq, n_uniq, uniq_stride, probebits, keep_words);
    const int gx = nq >= 16 ? 64 : (nq >= 4 ? 256 : 1024);
    hipLaunchKernelGGL(van_union_kernel, dim3(gx, nq), dim3(256), 0, st, uniq, n_uniq, uniq_stride, eoff, eids, tok2pid, candbits,
                       cand_words);
}
