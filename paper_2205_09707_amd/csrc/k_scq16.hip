// S_cq = C . Q^T (Eq. 2) on the half-precision matrix instruction, with both operands split into two fp16 terms.
//
// An fp32 value a is written a = a1 + 2^-11 a2 + d, with a1 = fp16(a), a2 = fp16(2^11 (a - a1)) and |d| <= 2^-22 |a|
// (each rounding keeps 11 significant bits; a1 is taken as 0 below fp16's normal range, so no operand is subnormal but
// for values under 2^-25).  Then a b = a1 b1 + 2^-11 (a1 b2 + a2 b1) + r with |r| <= 3 * 2^-22 |a b|: three products
// of fp16 values, each exact in fp32, accumulated in fp32 by v_mfma_f32_32x32x16_f16 -- a1 b1 in one accumulator, the
// two cross terms in a second one that is scaled by 2^-11 when the two are added.  For vectors of norm at most one the
// result differs from the exact dot product by at most 3 * 2^-22 (dropped terms) plus the fp32 accumulation error of
// the 128 products, 128 * 2^-24 in the worst case: PLAID_SCQ16_EPS = 2^-16 covers both with room to spare.  Discrete
// decisions never rest on these values alone: the probe kernel re-evaluates in double, as the definition reads, every
// entry that lies within the bound of a decision (k_scq.hip).
//
// Work split: a workgroup of four waves owns 256 consecutive centroids; a wave keeps the operands of its 64 centroid
// rows (two 32-row tiles) in registers for the whole kernel and walks a group of queries, whose operands (16 KB per
// query, already split and laid out in operand order by scq16_split_kernel) pass through LDS, double-buffered, shared
// by the four waves.  Per query and tile: 24 matrix instructions, then the epilogue straight from the accumulators:
// S (a store instruction writes two whole 128-byte rows), the tile's column maxima, and the pruning bits of Eq. 5 in
// two flavours -- "passes even if every entry were PLAID_SCQ16_EPS lower" (kept for sure) and "would pass if some
// entry were PLAID_SCQ16_EPS higher" (ambiguous: decided later in double).
#include "plaid_internal.h"

#include <math.h>

typedef _Float16 scq16_half8 __attribute__((ext_vector_type(8)));
typedef float scq16_floatx16 __attribute__((ext_vector_type(16)));

#define H16_THREADS 256
#define H16_WAVES (H16_THREADS / 64)
#define H16_NT 2                                  // 32-row tiles per wave
#define H16_WG_TILES (H16_WAVES * H16_NT)         // tiles per workgroup (the operand table is padded to a multiple of it)
#define H16_STEPS (DIM / 16)                      // matrix instructions along the 128 dimensions
#define H16_TILE_VEC (2 * H16_STEPS * 64)         // 16-byte operand vectors per tile: [term][step][lane]
#define H16_SCALE 2048.0f                         // 2^11: keeps the second term in fp16's normal range

// Operand layout of v_mfma_f32_32x32x16_f16, lane = 32 h + m: the A operand holds row m of a 32-row tile, the B operand
// column m, both at dimensions 16 s + 8 h .. 16 s + 8 h + 7 of step s.  Centroid tiles and queries use the same layout:
// dst[tile][term][step][lane] = eight consecutive dimensions of row 32 tile + m, term 0 = a1, term 1 = a2.
// Rows at or past n_rows are zero.  zero / zero_words: workspace words this launch clears on the side (may be null).
__global__ __launch_bounds__(256) void scq16_split_kernel(const float *__restrict__ src, int64_t n_rows, int64_t n_tiles,
                                                          scq16_half8 *__restrict__ dst, uint32_t *__restrict__ zero,
                                                          int64_t zero_words)
{
    const int64_t t0 = (int64_t)blockIdx.x * blockDim.x + threadIdx.x, step = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = t0; i < zero_words; i += step) zero[i] = 0u;
    for (int64_t e = t0; e < n_tiles * (H16_STEPS * 64); e += step) {
        const int64_t tile = e / (H16_STEPS * 64);
        const int s = (int)(e >> 6) & (H16_STEPS - 1), lane = (int)(e & 63);
        const int64_t row = tile * 32 + (lane & 31);
        const int k0 = 16 * s + 8 * (lane >> 5);
        float x[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        if (row < n_rows) {
            const float4 *p = reinterpret_cast<const float4 *>(src + row * DIM + k0);
            const float4 u = p[0], v = p[1];
            x[0] = u.x, x[1] = u.y, x[2] = u.z, x[3] = u.w, x[4] = v.x, x[5] = v.y, x[6] = v.z, x[7] = v.w;
        }
        scq16_half8 h1, h2;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const _Float16 a1 = fabsf(x[j]) >= 6.103515625e-05f ? (_Float16)x[j] : (_Float16)0.0f;  // 2^-14
            h1[j] = a1;
            h2[j] = (_Float16)((x[j] - (float)a1) * H16_SCALE);
        }
        dst[(tile * 2 + 0) * (H16_STEPS * 64) + s * 64 + lane] = h1;
        dst[(tile * 2 + 1) * (H16_STEPS * 64) + s * 64 + lane] = h2;
    }
}

// Workgroup barrier that orders LDS accesses only.  __syncthreads() would also wait for every outstanding global
// store, and this kernel keeps a query's worth of score stores in flight per wave when it reaches the barrier.
__device__ __forceinline__ void scq16_lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Grid: x = block of 32 * H16_WAVES * NT centroids, y = group of qg queries.  A16: a whole number of workgroups' tiles
// (rows past C are zero).  keepbits / ambbits: [q][keep_words], bit c = row c passes Eq. 5 for sure / is ambiguous;
// tilemax: [q][ceil(C/32)][32].
// The loop over the group's queries is software-pipelined so that no wait covers a score store: the operands of query
// q + 1 are requested before the matrix instructions of query q, moved into the other LDS buffer right after them (by
// then they have arrived), the operands of q + 2 are requested, and only then are the scores of q stored.
// STORE = false: the scores themselves are not written, only the tile maxima and the pruning words (nearest-centroid
// assignment, which re-evaluates the rows of the best tile).
template <int NT, bool STORE>
__global__ __launch_bounds__(H16_THREADS, NT == 2 ? 2 : 4) void scq16_kernel(
    const scq16_half8 *__restrict__ A16, int64_t C, const scq16_half8 *__restrict__ B16, int nq, int qg, float t_lo, float t_hi,
    float *__restrict__ S, uint32_t *__restrict__ keepbits, uint32_t *__restrict__ ambbits, int64_t keep_words,
    float *__restrict__ tilemax)
{
    __shared__ scq16_half8 Bs[2][H16_TILE_VEC];
    constexpr int NPRE = H16_TILE_VEC / H16_THREADS;  // operand vectors a thread moves per query
    const int tid = threadIdx.x, lane = tid & 63, n = lane & 31, h = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int64_t tile0 = ((int64_t)blockIdx.x * H16_WAVES + wave) * NT;
    const int64_t n_blk = (C + 31) >> 5;
    const int q_begin = blockIdx.y * qg, q_end = q_begin + qg < nq ? q_begin + qg : nq;

    scq16_half8 pre[NPRE];
    const scq16_half8 *bsrc = B16 + (int64_t)q_begin * H16_TILE_VEC + tid;
#pragma unroll
    for (int k = 0; k < NPRE; ++k) pre[k] = bsrc[k * H16_THREADS];

    scq16_half8 a[NT][2][H16_STEPS];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int term = 0; term < 2; ++term)
#pragma unroll
            for (int s = 0; s < H16_STEPS; ++s)
                a[t][term][s] = A16[((tile0 + t) * 2 + term) * (H16_STEPS * 64) + s * 64 + lane];

#pragma unroll
    for (int k = 0; k < NPRE; ++k) Bs[0][tid + k * H16_THREADS] = pre[k];
    if (q_begin + 1 < q_end) {
        bsrc += H16_TILE_VEC;
#pragma unroll
        for (int k = 0; k < NPRE; ++k) pre[k] = bsrc[k * H16_THREADS];
    }
    scq16_lds_barrier();

    for (int q = q_begin; q < q_end; ++q) {
        const scq16_half8 *buf = Bs[(q - q_begin) & 1];
        scq16_half8 *nxt = Bs[(q - q_begin + 1) & 1];
        scq16_floatx16 hi[NT], lo[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) hi[t][v] = 0.f, lo[t][v] = 0.f;
#pragma unroll
        for (int s = 0; s < H16_STEPS; ++s) {
            const scq16_half8 b1 = buf[s * 64 + lane], b2 = buf[(H16_STEPS + s) * 64 + lane];
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                hi[t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[t][0][s], b1, hi[t], 0, 0, 0);
                lo[t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[t][0][s], b2, lo[t], 0, 0, 0);
                lo[t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[t][1][s], b1, lo[t], 0, 0, 0);
            }
        }
        // the next query's operands: into the buffer that every wave finished reading before the last barrier
        if (q + 1 < q_end) {
#pragma unroll
            for (int k = 0; k < NPRE; ++k) nxt[tid + k * H16_THREADS] = pre[k];
        }
        if (q + 2 < q_end) {
            bsrc += H16_TILE_VEC;
#pragma unroll
            for (int k = 0; k < NPRE; ++k) pre[k] = bsrc[k * H16_THREADS];
        }
        // Epilogue.  Accumulator v of lane 32 h + n is row 8 (v / 4) + 4 h + v % 4 of the tile, column (query token) n.
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int64_t tile = tile0 + t;
            if (tile >= n_blk) break;  // (uniform) a tile past the end of the table
            const int64_t row0 = tile << 5;
            const int nvalid = C - row0 < 32 ? (int)(C - row0) : 32;
            float *srow = S + ((int64_t)q * C + row0 + 4 * h) * QLEN + n;
            float val[16];
#pragma unroll
            for (int v = 0; v < 16; ++v) val[v] = fmaf(lo[t][v], 1.0f / H16_SCALE, hi[t][v]);
            float cmax = -INFINITY;
            if (nvalid == 32) {  // (uniform) a whole tile: sixteen unconditional stores of two 128-byte rows each, marked
                                 // as streaming (4 GB per launch pass through: nothing of it is worth a cache line)
                if (STORE) {
#pragma unroll
                    for (int v = 0; v < 16; ++v) __builtin_nontemporal_store(val[v], &srow[(8 * (v >> 2) + (v & 3)) * QLEN]);
                }
#pragma unroll
                for (int v = 0; v < 16; ++v) cmax = fmaxf(cmax, val[v]);
            } else {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int r = 8 * (v >> 2) + (v & 3);
                    if (r + 4 * h < nvalid) {
                        if (STORE) srow[r * QLEN] = val[v];
                        cmax = fmaxf(cmax, val[v]);
                    }
                }
            }
            // Eq. 5.  A row can only pass when some lane's maximum reaches t_lo, which no lane's does for all but a few
            // tiles: one comparison settles those.  (Rows past the end hold zeros and are masked below.)
            float lmax = val[0];
#pragma unroll
            for (int v = 1; v < 16; ++v) lmax = fmaxf(lmax, val[v]);
            uint32_t maybe = 0u, sure = 0u;  // uniform: bit = row of the tile with an entry >= t_lo / >= t_hi
            if (__ballot(lmax >= t_lo) != 0ull) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int r = 8 * (v >> 2) + (v & 3);
                    const unsigned long long m = __ballot(val[v] >= t_lo), ms = __ballot(val[v] >= t_hi);
                    maybe |= (((uint32_t)m) ? 1u : 0u) << r;
                    maybe |= (((uint32_t)(m >> 32)) ? 1u : 0u) << (r + 4);
                    sure |= (((uint32_t)ms) ? 1u : 0u) << r;
                    sure |= (((uint32_t)(ms >> 32)) ? 1u : 0u) << (r + 4);
                }
            }
            const uint32_t valid = nvalid == 32 ? 0xFFFFFFFFu : (1u << nvalid) - 1u;  // rows past the end never pass
            cmax = fmaxf(cmax, __shfl_xor(cmax, 32));
            if (tilemax && h == 0) tilemax[((int64_t)q * n_blk + tile) * QLEN + n] = cmax;
            if (lane == 0) {
                keepbits[(int64_t)q * keep_words + tile] = sure & valid;
                ambbits[(int64_t)q * keep_words + tile] = maybe & ~sure & valid;
            }
        }
        scq16_lds_barrier();  // publishes nxt; every wave is done reading buf
    }
}

// ------------------------------------------------------------------ host side
size_t plaid_scq16_centroid_bytes(int64_t C)
{
    const int64_t tiles = ((C + 32 * H16_WG_TILES - 1) / (32 * H16_WG_TILES)) * H16_WG_TILES;
    return (size_t)tiles * H16_TILE_VEC * sizeof(scq16_half8);
}
size_t plaid_scq16_query_bytes(int nq) { return (size_t)nq * H16_TILE_VEC * sizeof(scq16_half8); }

void plaid_launch_scq16_split_centroids(hipStream_t st, const float *centroids, int64_t C, void *A16)
{
    const int64_t tiles = (int64_t)(plaid_scq16_centroid_bytes(C) / (H16_TILE_VEC * sizeof(scq16_half8)));
    int64_t g = (tiles * (H16_STEPS * 64) + 255) / 256;
    if (g > 65536) g = 65536;
    hipLaunchKernelGGL(scq16_split_kernel, dim3((unsigned)g), dim3(256), 0, st, centroids, C, tiles, (scq16_half8 *)A16,
                       (uint32_t *)nullptr, (int64_t)0);
}

void plaid_launch_scq16_split_queries(hipStream_t st, const float *Q, int nq, void *B16, uint32_t *zero, int64_t zero_words)
{
    int64_t work = (int64_t)nq * (H16_STEPS * 64);
    if (work < zero_words) work = zero_words;
    int64_t g = (work + 255) / 256;
    if (g > 4096) g = 4096;
    if (g < 1) g = 1;
    hipLaunchKernelGGL(scq16_split_kernel, dim3((unsigned)g), dim3(256), 0, st, Q, (int64_t)nq * QLEN, (int64_t)nq, (scq16_half8 *)B16,
                       zero, zero_words);
}

void plaid_launch_scq16(hipStream_t st, const void *A16, int64_t C, const void *B16, int nq, float t_cs, float *S,
                        uint32_t *keepbits, uint32_t *ambbits, int64_t keep_words, float *tilemax)
{
    // the two thresholds of the pruning test, rounded away from t_cs (infinite t_cs: both equal it, nothing is ambiguous)
    float t_lo = t_cs, t_hi = t_cs;
    if (t_cs > -INFINITY && t_cs < INFINITY) {
        t_lo = nextafterf(t_cs - PLAID_SCQ16_EPS, -INFINITY);
        t_hi = nextafterf(t_cs + PLAID_SCQ16_EPS, INFINITY);
    }
    const unsigned gx = (unsigned)((C + 32 * H16_WG_TILES - 1) / (32 * H16_WG_TILES));
    // queries per workgroup: enough workgroups to fill the chip several times over, yet many queries per workgroup, since
    // its centroid operands are loaded once
    int qg = (int)(((int64_t)nq * gx + 2047) / 2048);
    if (qg < 8) qg = 8;
    if (qg > 64) qg = 64;
    if (qg > nq) qg = nq;
    const unsigned gy = (unsigned)((nq + qg - 1) / qg);
    if (S)
        hipLaunchKernelGGL((scq16_kernel<H16_NT, true>), dim3(gx, gy), dim3(H16_THREADS), 0, st, (const scq16_half8 *)A16, C,
                           (const scq16_half8 *)B16, nq, qg, t_lo, t_hi, S, keepbits, ambbits, keep_words, tilemax);
    else
        hipLaunchKernelGGL((scq16_kernel<H16_NT, false>), dim3(gx, gy), dim3(H16_THREADS), 0, st, (const scq16_half8 *)A16, C,
                           (const scq16_half8 *)B16, nq, qg, t_lo, t_hi, S, keepbits, ambbits, keep_words, tilemax);
}
