// Query-centroid scores S_cq = C . Q^T (Eq. 2) with the centroid pruning map of Eq. 5 fused in.
//
// Every later decision of the pipeline (which centroids are probed, which survive t_cs, which
// passages make the ndocs and ndocs/4 cuts) is a comparison of these values or of sums of them,
// so they are computed the way the definition reads: each S[c][i] is the dot product accumulated
// in double over the dimensions in index order, rounded once to fp32.  A product of two fp32
// values is exact in double, so a chain of fused multiply-adds in that order gives the same bits
// as "multiply, then add" on any machine -- the scores carry no accumulation-order freedom.
//
// Mapping: one lane owns one centroid row and keeps TOK double accumulators (one per query
// token of its token group); the query, pre-converted to double and transposed to [dim][32], is
// uniform across the wave and is fetched through the scalar unit, so the inner loop is one
// v_fma_f64 per (dimension, token) with no per-lane operand traffic besides the centroid row.
// Output row c of S is the 128-byte record that a token's centroid id later gathers.
#include "plaid_internal.h"

// Qd[q][t][i] = (double) Q[q][i][t]
__global__ void scq_prepare_kernel(const float *__restrict__ Q, double *__restrict__ Qd)
{
    const int q = blockIdx.x;
    for (int e = threadIdx.x; e < QLEN * DIM; e += blockDim.x) {
        const int t = e >> 5, i = e & 31;
        Qd[(int64_t)q * QLEN * DIM + e] = (double)Q[(int64_t)q * QLEN * DIM + i * DIM + t];
    }
}

template <int TOK>  // query tokens per wave: 16 or 8 (smaller = more waves when C is small)
__global__ __launch_bounds__(256) void scq_kernel(const float *__restrict__ Cm, int64_t C, const double *__restrict__ Qd,
                                                  float *__restrict__ S)
{
    constexpr int GROUPS = QLEN / TOK;
    const int q = blockIdx.y;
    const int lane = threadIdx.x & 63;
    // wave-uniform, so that the query operands below are fetched by scalar loads
    const int64_t wave = (int64_t)blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t c = (wave / GROUPS) * 64 + lane;
    const int i0 = (int)(wave % GROUPS) * TOK;
    if ((wave / GROUPS) * 64 >= C) return;
    const double *__restrict__ qd = Qd + (int64_t)q * QLEN * DIM + i0;
    const float *__restrict__ row = Cm + (c < C ? c : C - 1) * DIM;
    double acc[TOK];
#pragma unroll
    for (int i = 0; i < TOK; ++i) acc[i] = 0.0;
    // the row is consumed in four 32-dimension chunks; chunk k+1 is in flight while chunk k is multiplied
    float4 cur[8], nxt[8];
#pragma unroll
    for (int v = 0; v < 8; ++v) cur[v] = *reinterpret_cast<const float4 *>(row + 4 * v);
#pragma unroll 1
    for (int tb = 0; tb < DIM; tb += 32) {
        const int tn = tb + 32 < DIM ? tb + 32 : tb;  // the last round reloads its own chunk (unused)
#pragma unroll
        for (int v = 0; v < 8; ++v) nxt[v] = *reinterpret_cast<const float4 *>(row + tn + 4 * v);
#pragma unroll
        for (int v = 0; v < 8; ++v) {
            const double a[4] = {(double)cur[v].x, (double)cur[v].y, (double)cur[v].z, (double)cur[v].w};
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int i = 0; i < TOK; ++i) acc[i] = fma(a[u], qd[(tb + 4 * v + u) * QLEN + i], acc[i]);
        }
#pragma unroll
        for (int v = 0; v < 8; ++v) cur[v] = nxt[v];
    }
    if (c < C) {
        float *o = S + ((int64_t)q * C + c) * QLEN + i0;
#pragma unroll
        for (int i = 0; i < TOK; i += 4)
            *reinterpret_cast<float4 *>(o + i) =
                make_float4((float)acc[i], (float)acc[i + 1], (float)acc[i + 2], (float)acc[i + 3]);
    }
}

// Eq. 5: bit c of keepbits[q] = (max_i S[q][c][i] >= t_cs), inclusive.  Eight lanes share a row.
__global__ __launch_bounds__(256) void keep_kernel(const float *__restrict__ S, int64_t C, float t_cs,
                                                   uint32_t *__restrict__ keepbits, int64_t keep_words)
{
    const int q = blockIdx.y;
    const float *Sq = S + (int64_t)q * C * QLEN;
    uint32_t *kb = keepbits + (int64_t)q * keep_words;
    const int sub = threadIdx.x & 7;
    __shared__ uint32_t part[4];
    // a block covers 32 rows per step, i.e. one bitmap word
    for (int64_t w = blockIdx.x; w < keep_words; w += gridDim.x) {
        const int64_t c = w * 32 + (threadIdx.x >> 3);
        float m = -INFINITY;
        if (c < C) {
            const float4 v = *reinterpret_cast<const float4 *>(Sq + c * QLEN + 4 * sub);
            m = fmaxf(fmaxf(v.x, v.y), fmaxf(v.z, v.w));
        }
        m = fmaxf(m, __shfl_xor(m, 1));
        m = fmaxf(m, __shfl_xor(m, 2));
        m = fmaxf(m, __shfl_xor(m, 4));
        const bool keep = c < C && m >= t_cs;
        const unsigned long long b = __ballot(keep && sub == 0);  // bit 8r of the wave's ballot = row r of this wave
        // compress bits 0, 8, ..., 56 into one byte
        unsigned long long x = b & 0x0101010101010101ull;
        x = (x * 0x0102040810204080ull) >> 56;
        if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = (uint32_t)x;
        __syncthreads();
        if (threadIdx.x == 0) kb[w] = part[0] | (part[1] << 8) | (part[2] << 16) | (part[3] << 24);
        __syncthreads();
    }
}

void plaid_launch_scq(hipStream_t st, const float *centroids, int64_t C, const float *Q, double *Qd, int nq, float t_cs,
                      float *S, uint32_t *keepbits, int64_t keep_words)
{
    hipLaunchKernelGGL(scq_prepare_kernel, dim3(nq), dim3(256), 0, st, Q, Qd);
    const int64_t rows64 = (C + 63) / 64;
    // enough waves to cover the 1024 SIMDs of the chip when C (times the queries of the chunk) is small
    if (rows64 * 2 * nq >= 2048)
        hipLaunchKernelGGL(scq_kernel<16>, dim3((unsigned)((rows64 * 2 + 3) / 4), nq), dim3(256), 0, st, centroids, C, Qd,
                           S);
    else
        hipLaunchKernelGGL(scq_kernel<8>, dim3((unsigned)((rows64 * 4 + 3) / 4), nq), dim3(256), 0, st, centroids, C, Qd, S);
    int64_t gx = keep_words;
    const int64_t cap = nq >= 8 ? 256 : 2048;
    if (gx > cap) gx = cap;
    hipLaunchKernelGGL(keep_kernel, dim3((unsigned)gx, nq), dim3(256), 0, st, S, C, t_cs, keepbits, keep_words);
}
