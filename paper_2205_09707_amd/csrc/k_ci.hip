// Centroid interaction (Eq. 3-4) and centroid pruning (Eq. 5): the score of a passage is
// sum_i max_j S_cq[code_j][i] over its tokens j (only tokens whose centroid is kept, when pruning).
// The rows S_cq[code_j] are never stacked into a matrix: a wave keeps one running maximum per query
// token (lane i and lane i+32 both serve token i, on alternate passage tokens) and sums the 32 maxima
// at the end -- in double, in index order, as the definition's sum over the query tokens reads.
//
// This file holds the gather formulation for a list of passages (one wave per passage, rows fetched
// from the L2-resident S): stage 3.
#include "plaid_internal.h"

#include <math.h>

#define CI_FLY 8

// Score of the passage with tokens [t0, t1).  Uniform across the wave; -inf when no token contributes.
template <bool PRUNE>
__device__ __forceinline__ float ci_passage(const float *__restrict__ Sq, const uint32_t *__restrict__ kb, int64_t t0,
                                            int64_t t1, const int32_t *__restrict__ codes, int lane)
{
    const int i = lane & 31, h = lane >> 5;
    float m = -INFINITY;
    for (int64_t base = t0; base < t1; base += 64) {
        const int cnt = t1 - base < 64 ? (int)(t1 - base) : 64;
        const int32_t code = lane < cnt ? codes[base + lane] : 0;
        if (!PRUNE) {
            // CI_FLY row pairs in flight, then 4, then one at a time (a row is 128 bytes somewhere in the query's S_cq:
            // the more requests a wave keeps in flight, the closer the gather gets to the memory system's rate)
            int j = 0;
            for (; j + 2 * CI_FLY <= cnt; j += 2 * CI_FLY) {
                float v[CI_FLY];
#pragma unroll
                for (int u = 0; u < CI_FLY; ++u) v[u] = Sq[(int64_t)__shfl(code, j + 2 * u + h) * QLEN + i];
#pragma unroll
                for (int u = 0; u < CI_FLY; ++u) m = fmaxf(m, v[u]);
            }
            for (; j + 8 <= cnt; j += 8) {
                const int c0 = __shfl(code, j + h), c1 = __shfl(code, j + 2 + h), c2 = __shfl(code, j + 4 + h),
                          c3 = __shfl(code, j + 6 + h);
                const float v0 = Sq[(int64_t)c0 * QLEN + i], v1 = Sq[(int64_t)c1 * QLEN + i],
                            v2 = Sq[(int64_t)c2 * QLEN + i], v3 = Sq[(int64_t)c3 * QLEN + i];
                m = fmaxf(fmaxf(m, v0), fmaxf(v1, fmaxf(v2, v3)));
            }
            for (; j < cnt; j += 2) {
                const int jj = j + h < cnt ? j + h : j;
                const int c = __shfl(code, jj);
                m = fmaxf(m, Sq[(int64_t)c * QLEN + i]);
            }
        } else {
            bool hit = lane < cnt;
            if (hit) hit = (kb[code >> 5] >> (code & 31)) & 1u;
            unsigned long long mask = __ballot(hit);
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
    }
    m = fmaxf(m, __shfl_xor(m, 32));
    return plaid_sum32_in_order(m);
}

// Stage 3: out_keys[q][j] = key(score of passage of in_keys[q][j]).
__global__ __launch_bounds__(256) void ci_list_kernel(const float *__restrict__ S, int64_t C,
                                                      const int64_t *__restrict__ doc_offsets,
                                                      const int32_t *__restrict__ codes,
                                                      const uint64_t *__restrict__ in_keys, int64_t in_stride,
                                                      const int32_t *__restrict__ in_counts,
                                                      uint64_t *__restrict__ out_keys, int64_t out_stride)
{
    const int q = blockIdx.y;
    const int lane = threadIdx.x & 63;
    const int j = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (j >= in_counts[q]) return;
    const uint32_t pid = (uint32_t)(in_keys[(int64_t)q * in_stride + j] & 0xFFFFFFFFu);
    const float sc = ci_passage<false>(S + (int64_t)q * C * QLEN, nullptr, doc_offsets[pid], doc_offsets[pid + 1], codes, lane);
    if (lane == 0) out_keys[(int64_t)q * out_stride + j] = plaid_make_key(sc, pid);
}

void plaid_launch_ci_list(hipStream_t st, const float *S, int64_t C, const int64_t *doc_offsets, const int32_t *codes,
                          int nq, const uint64_t *in_keys, int64_t in_stride, const int32_t *in_counts, int n_upper,
                          uint64_t *out_keys, int64_t out_stride)
{
    hipLaunchKernelGGL(ci_list_kernel, dim3((n_upper + 3) / 4, nq), dim3(256), 0, st, S, C, doc_offsets, codes, in_keys,
                       in_stride, in_counts, out_keys, out_stride);
}
