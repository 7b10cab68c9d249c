// Centroid interaction without pruning (Eq. 3-4): the score of a passage is sum_i max_j S_cq[code_j][i] over its
// tokens j.  The rows S_cq[code_j] are never stacked into a matrix: a wave keeps running maxima per query token and
// sums the 32 maxima at the end -- in double, in index order, as the definition's sum over the query tokens reads.
//
// This file holds the gather formulation for a list of passages: stage 3.  One wave per passage.  A row of S_cq is
// 128 bytes: eight lanes fetch it with one 16-byte load each, so one load instruction of the wave brings the rows of
// eight tokens; lane (r, part) = (lane / 8, lane % 8) keeps the maxima of query tokens 4 part .. 4 part + 3 over the
// tokens r, r + 8, ... of the passage, and the eight partial maxima of a query token meet once per passage.
#include "plaid_internal.h"

#include <math.h>

#define CI_PPW 2  // passages a wave takes at a time

__device__ __forceinline__ float4 ci_max4(float4 a, float4 b)
{
    return make_float4(fmaxf(a.x, b.x), fmaxf(a.y, b.y), fmaxf(a.z, b.z), fmaxf(a.w, b.w));
}

// The rows of the first min(cnt, 8 N) tokens of a chunk (cnt <= 8 N), N loads in flight: lane (r, part) takes 16 bytes
// of the rows of tokens r, r + 8, ...; a slot past the end fetches the last token's row again (same maxima).
template <bool WIDE, int N>
__device__ __forceinline__ float4 ci_rows(const char *__restrict__ base, uint32_t row, int cnt, int r, int part, float4 m)
{
    float4 v[N];
#pragma unroll
    for (int u = 0; u < N; ++u) {
        int t = 8 * u + r;
        t = t < cnt ? t : cnt - 1;
        const uint32_t rt = (uint32_t)__shfl((int)row, t);
        const uint64_t off = WIDE ? ((uint64_t)rt << 7) + 16u * (uint32_t)part : (uint64_t)(rt + 16u * (uint32_t)part);
        v[u] = *reinterpret_cast<const float4 *>(base + off);
    }
#pragma unroll
    for (int u = 0; u < N; ++u) m = ci_max4(m, v[u]);
    return m;
}

// The codes of the tokens tb + lane < t1 (0 past the end).
__device__ __forceinline__ int32_t ci_chunk_codes(const int32_t *__restrict__ codes, int64_t tb, int64_t t1, int lane)
{
    int32_t c = 0;
    if (tb + lane < t1) c = codes[tb + lane];
    return c;
}

__device__ __forceinline__ int64_t ci_uniform(int64_t v)
{
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)v);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)((uint64_t)v >> 32));
    return (int64_t)(((uint64_t)hi << 32) | lo);
}

// Running maxima of the passage with tokens [t0, t1): lane (r, part) returns the maxima of query tokens 4 part ..
// 4 part + 3 over the tokens r, r + 8, ... (-inf where it saw none).
// Sq: this query's S_cq; !WIDE: at most 2^32 bytes, so that row offsets fit 32 bits (C <= 2^25).
// c0 = ci_chunk_codes of the passage's first chunk (requested by the caller ahead of time).
template <bool WIDE>
__device__ __forceinline__ float4 ci_passage(const float *__restrict__ Sq, int64_t t0, int64_t t1,
                                             const int32_t *__restrict__ codes, int lane, int32_t c0)
{
    const int part = lane & 7, r = lane >> 3;
    const char *__restrict__ base = reinterpret_cast<const char *>(Sq);
    float4 m = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
    for (int64_t tb = t0; tb < t1; tb += 64) {  // uniform
        const int cnt = t1 - tb < 64 ? (int)(t1 - tb) : 64;
        // byte offset (WIDE: number) of this lane's token's row
        const uint32_t row = (uint32_t)(tb == t0 ? c0 : ci_chunk_codes(codes, tb, t1, lane)) << (WIDE ? 0 : 7);
        // 8 tokens per load instruction, all of a chunk's instructions in flight together
        switch ((cnt + 7) >> 3) {  // uniform
        case 1: m = ci_rows<WIDE, 1>(base, row, cnt, r, part, m); break;
        case 2: m = ci_rows<WIDE, 2>(base, row, cnt, r, part, m); break;
        case 3: m = ci_rows<WIDE, 3>(base, row, cnt, r, part, m); break;
        case 4: m = ci_rows<WIDE, 4>(base, row, cnt, r, part, m); break;
        case 5: m = ci_rows<WIDE, 5>(base, row, cnt, r, part, m); break;
        case 6: m = ci_rows<WIDE, 6>(base, row, cnt, r, part, m); break;
        case 7: m = ci_rows<WIDE, 7>(base, row, cnt, r, part, m); break;
        default: m = ci_rows<WIDE, 8>(base, row, cnt, r, part, m); break;
        }
    }
    return m;
}

// Stage 3: out_keys[q][j] = key(score of passage of in_keys[q][j]).
//
// The grid is one-dimensional and consecutive workgroups go to the chip's eight partitions in turn, each with a
// second-level cache of its own: workgroup L serves query 8 (L / 8 / gx) + L % 8, so that all workgroups of a query run
// on one partition and the rows its passages share (a query's passages name the same frequent centroids over and over)
// are fetched into that cache once.  With fewer than eight queries (spread) a query's workgroups go to all partitions.
//
// A wave takes CI_PPW consecutive passages at a time: their ids, then their token ranges, then their first 64 codes are
// requested together, so that the chain of dependent loads in front of the row gathers is paid once per group.  The
// lanes' partial maxima meet in LDS (wave-private areas, no workgroup barrier): lane t < 32 takes the maximum of query
// token t over the eight token classes, and when the group is done lane a adds up the 32 maxima of passage a -- one
// chain of additions for the whole group.
template <bool WIDE>
__global__ __launch_bounds__(256) void ci_list_kernel(const float *__restrict__ S, int64_t C,
                                                      const int64_t *__restrict__ doc_offsets,
                                                      const int32_t *__restrict__ codes,
                                                      const uint64_t *__restrict__ in_keys, int64_t in_stride,
                                                      const int32_t *__restrict__ in_counts, int nq, int gx, int spread,
                                                      uint64_t *__restrict__ out_keys, int64_t out_stride)
{
    constexpr int G = CI_PPW;
    __shared__ __align__(16) float part_max[4][8][QLEN];  // [wave][token class r][query token]
    __shared__ __align__(16) float col_max[4][G][QLEN];   // [wave][passage of the group][query token]
    int q, x;
    if (spread) {
        q = blockIdx.x / gx;
        x = blockIdx.x % gx;
    } else {
        const int k = blockIdx.x >> 3;
        q = 8 * (k / gx) + (blockIdx.x & 7);
        x = k % gx;
    }
    if (q >= nq) return;
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int n = in_counts[q];
    const float *__restrict__ Sq = S + (int64_t)q * C * QLEN;
    const uint64_t *__restrict__ ik = in_keys + (int64_t)q * in_stride;
    for (int64_t j0 = ((int64_t)x * 4 + wv) * G; j0 < n; j0 += 4ll * G * gx) {  // one round unless the list is huge
        uint32_t pid[G];
        int64_t t0[G], t1[G];
        int32_t c0[G];
        uint64_t key[G];
#pragma unroll
        for (int a = 0; a < G; ++a) key[a] = ik[j0 + a < n ? j0 + a : j0];
#pragma unroll
        for (int a = 0; a < G; ++a) pid[a] = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)key[a]);
#pragma unroll
        for (int a = 0; a < G; ++a) {
            t0[a] = doc_offsets[pid[a]];
            t1[a] = doc_offsets[pid[a] + 1];
        }
#pragma unroll
        for (int a = 0; a < G; ++a) {
            t0[a] = ci_uniform(t0[a]);
            t1[a] = ci_uniform(t1[a]);
        }
#pragma unroll
        for (int a = 0; a < G; ++a) c0[a] = ci_chunk_codes(codes, t0[a], t1[a], lane);
#pragma unroll
        for (int a = 0; a < G; ++a) {
            const float4 m = ci_passage<WIDE>(Sq, t0[a], t1[a], codes, lane, c0[a]);
            // lane (r, part) holds query tokens 4 part .. 4 part + 3 of class r
            *reinterpret_cast<float4 *>(&part_max[wv][lane >> 3][4 * (lane & 7)]) = m;
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            if (lane < QLEN) {
                float v = part_max[wv][0][lane];
#pragma unroll
                for (int r = 1; r < 8; ++r) v = fmaxf(v, part_max[wv][r][lane]);
                col_max[wv][a][lane] = v;
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
        // lane a: the sum over the query tokens of Eq. 4 for passage a, in double, in index order, rounded once
        if (lane < G && j0 + lane < n) {
            double d = 0.0;
#pragma unroll
            for (int i4 = 0; i4 < QLEN / 4; ++i4) {
                const float4 v = *reinterpret_cast<const float4 *>(&col_max[wv][lane][4 * i4]);
                d += (double)v.x;
                d += (double)v.y;
                d += (double)v.z;
                d += (double)v.w;
            }
            uint32_t my_pid = pid[0];
#pragma unroll
            for (int a = 1; a < G; ++a) my_pid = lane == a ? pid[a] : my_pid;
            out_keys[(int64_t)q * out_stride + j0 + lane] = plaid_make_key((float)d, my_pid);
        }
    }
}

void plaid_launch_ci_list(hipStream_t st, const float *S, int64_t C, const int64_t *doc_offsets, const int32_t *codes,
                          int nq, const uint64_t *in_keys, int64_t in_stride, const int32_t *in_counts, int n_upper,
                          uint64_t *out_keys, int64_t out_stride)
{
    const int spread = nq < 8 ? 1 : 0;
    const int64_t slots = spread ? nq : 8 * (((int64_t)nq + 7) / 8);  // query slots of the grid
    int64_t gx = ((int64_t)n_upper + 4 * CI_PPW - 1) / (4 * CI_PPW);
    const int64_t cap = (1ll << 23) / slots;  // at most 2^23 workgroups (2^31 threads) per launch
    if (gx > cap) gx = cap;
    if (gx < 1) gx = 1;
    if (C <= (1ll << 25))
        hipLaunchKernelGGL(ci_list_kernel<false>, dim3((unsigned)(slots * gx)), dim3(256), 0, st, S, C, doc_offsets, codes,
                           in_keys, in_stride, in_counts, nq, (int)gx, spread, out_keys, out_stride);
    else
        hipLaunchKernelGGL(ci_list_kernel<true>, dim3((unsigned)(slots * gx)), dim3(256), 0, st, S, C, doc_offsets, codes,
                           in_keys, in_stride, in_counts, nq, (int)gx, spread, out_keys, out_stride);
}
