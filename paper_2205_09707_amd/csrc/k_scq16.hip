// S_cq = C . Q^T (Eq. 2) on the half-precision matrix instruction, with both operands split into two fp16 terms.
//
// An fp32 value a is written a = a1 + 2^-11 a2 + d, with a1 = fp16(a), a2 = fp16(2^11 (a - a1)) and |d| <= 2^-22 |a|
// (each rounding keeps 11 significant bits; a1 is taken as 0 below fp16's normal range, so no operand is subnormal but
// for values under 2^-25).  Then 2^11 a b = (2^11 a1) b1 + a1 b2 + a2 b1 + r with |r| <= 3 * 2^-11 |a b|: three
// products of fp16 values, each exact in fp32, accumulated in fp32 by v_mfma_f32_32x32x16_f16 into ONE accumulator,
// which is scaled by 2^-11 on its way out.  (2^11 a1 is formed from a1 next to its use, an exact packed multiplication;
// it needs |a| < 32 on the centroid side.)  Scaling the first product up, rather than the other two down, is what lets
// the three share an accumulator: the cross terms are 2^-11 of the sum, and a rounding of the sum at 2^-24 of its size
// costs them no more than it costs the first product.  For vectors of norm at most one the result differs from the exact
// dot product by at most 3 * 2^-22 (dropped terms) plus the fp32 accumulation error of the 384 products, 384 * 2^-24 in
// the worst case: PLAID_SCQ16_EPS = 2^-15 covers both.  Discrete decisions never rest on these values alone: the probe
// kernel re-evaluates in double, as the definition reads, every entry that lies within the bound of a decision
// (k_scq.hip).
//
// Work split: a workgroup of four waves owns 256 consecutive centroids; a wave keeps the operands of its 64 centroid
// rows (two 32-row tiles) in registers for the whole kernel and walks a group of queries, whose operands (16 KB per
// query, already split and laid out in operand order by scq16_split_kernel) pass through LDS, double-buffered, shared
// by the four waves.  Per query and tile: 24 matrix instructions, then straight from the accumulator: S (a store
// instruction writes two whole 128-byte rows), the tile's column maxima, and the pruning bits of Eq. 5 in
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

// One step of the matrix work: dimensions 16 s .. 16 s + 15 of every tile of the wave, all three products into the one
// accumulator of the tile.  k2048: 2^11 in every half (handed in so that the scaled operands are formed here, next to
// their use, instead of being kept in registers for the whole kernel).
template <int NT>
__device__ __forceinline__ void scq16_step(const scq16_half8 (&a)[NT][2][H16_STEPS], const scq16_half8 *buf, int lane, int s,
                                           scq16_half8 k2048, scq16_floatx16 (&acc)[NT])
{
    const scq16_half8 b1 = buf[s * 64 + lane], b2 = buf[(H16_STEPS + s) * 64 + lane];
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[t][0][s] * k2048, b1, acc[t], 0, 0, 0);
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[t][0][s], b2, acc[t], 0, 0, 0);
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[t][1][s], b1, acc[t], 0, 0, 0);
}

// The score stores of one query, cut into H16_STEPS parts of 2 NT store instructions each (a store instruction writes
// two whole 128-byte rows).  val[t][v] of lane 32 h + n is row 8 (v / 4) + 4 h + v % 4 of tile t, column (query token) n;
// s0: the address of row 4 h, column n of the wave's first tile.  WHOLE: every tile of the wave has its 32 rows; otherwise
// lim[t] = rows of tile t that exist, less 4 h.
template <int NT, bool WHOLE>
__device__ __forceinline__ void scq16_store_part(float *__restrict__ s0, const float (&val)[NT][16], int part, const int (&lim)[NT])
{
#pragma unroll
    for (int j = 0; j < 2 * NT; ++j) {
        const int i = part * 2 * NT + j, t = i >> 4, v = i & 15, r = 8 * (v >> 2) + (v & 3);
        float *dst = s0 + (int64_t)(32 * t + r) * QLEN;
        if (WHOLE)  // marked as streaming: 4 GB per launch pass through, nothing of it is worth a cache line
            __builtin_nontemporal_store(val[t][v], dst);
        else if (r < lim[t])
            *dst = val[t][v];
    }
}

// Out of the accumulators of one query: the scores (val, scaled back), the tiles' column maxima and the pruning words.
template <int NT>
__device__ __forceinline__ void scq16_reduce(const scq16_floatx16 (&acc)[NT], float (&val)[NT][16], const int (&nvalid)[NT],
                                             int64_t tile0, int64_t n_blk, int q, int lane, float t_lo, float t_hi,
                                             uint32_t *__restrict__ keepbits, uint32_t *__restrict__ ambbits, int64_t keep_words,
                                             float *__restrict__ tilemax)
{
    const int n = lane & 31, h = lane >> 5;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
#pragma unroll
        for (int v = 0; v < 16; ++v) val[t][v] = acc[t][v] * (1.0f / H16_SCALE);
        if (nvalid[t] == 0) continue;  // (uniform) a tile past the end of the table
        const int64_t tile = tile0 + t;
        float cmax = -INFINITY;
        if (nvalid[t] == 32) {
#pragma unroll
            for (int v = 0; v < 16; ++v) cmax = fmaxf(cmax, val[t][v]);
        } else {
#pragma unroll
            for (int v = 0; v < 16; ++v)
                if (8 * (v >> 2) + (v & 3) + 4 * h < nvalid[t]) cmax = fmaxf(cmax, val[t][v]);
        }
        // Eq. 5.  A row can only pass when some lane's maximum reaches t_lo, which no lane's does for all but a few
        // tiles: one comparison settles those.  (Rows past the end hold zeros and are masked below.)
        float lmax = val[t][0];
#pragma unroll
        for (int v = 1; v < 16; ++v) lmax = fmaxf(lmax, val[t][v]);
        uint32_t maybe = 0u, sure = 0u;  // uniform: bit = row of the tile with an entry >= t_lo / >= t_hi
        if (__ballot(lmax >= t_lo) != 0ull) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int r = 8 * (v >> 2) + (v & 3);
                const unsigned long long m = __ballot(val[t][v] >= t_lo), ms = __ballot(val[t][v] >= t_hi);
                maybe |= (((uint32_t)m) ? 1u : 0u) << r;
                maybe |= (((uint32_t)(m >> 32)) ? 1u : 0u) << (r + 4);
                sure |= (((uint32_t)ms) ? 1u : 0u) << r;
                sure |= (((uint32_t)(ms >> 32)) ? 1u : 0u) << (r + 4);
            }
        }
        const uint32_t valid = nvalid[t] == 32 ? 0xFFFFFFFFu : (1u << nvalid[t]) - 1u;  // rows past the end never pass
        cmax = fmaxf(cmax, __shfl_xor(cmax, 32));
        if (tilemax && h == 0) tilemax[((int64_t)q * n_blk + tile) * QLEN + n] = cmax;
        if (lane == 0) {
            keepbits[(int64_t)q * keep_words + tile] = sure & valid;
            ambbits[(int64_t)q * keep_words + tile] = maybe & ~sure & valid;
        }
    }
}

// The kernel's body.  WHOLE (uniform over the wave): each of its tiles has all 32 rows, so every score store is
// unconditional.  The two cases are separate instances, and the first query is taken out of the loop, so that the number
// of stores between a request for operands and the wait for them is the same on every path: the memory counter retires
// in order, and a wait sized for the path with the fewest stores would sit out the score stores of the others.
template <int NT, bool STORE, bool WHOLE>
__device__ __forceinline__ void scq16_body(scq16_half8 (&Bs)[2][H16_TILE_VEC], const int (&nvalid)[NT], const scq16_half8 *__restrict__ A16,
                                           int64_t C, const scq16_half8 *__restrict__ B16, int q_begin, int q_end, float t_lo,
                                           float t_hi, float *__restrict__ S, uint32_t *__restrict__ keepbits,
                                           uint32_t *__restrict__ ambbits, int64_t keep_words, float *__restrict__ tilemax)
{
    constexpr int NPRE = H16_TILE_VEC / H16_THREADS;  // operand vectors a thread moves per query
    const int tid = threadIdx.x, lane = tid & 63, n = lane & 31, h = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int64_t tile0 = ((int64_t)blockIdx.x * H16_WAVES + wave) * NT;
    const int64_t n_blk = (C + 31) >> 5;

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

    scq16_floatx16 acc[NT];
    float val[NT][16];
    typedef _Float16 scq16_half2 __attribute__((ext_vector_type(2)));
    // matrix work of query q (operands in Bs[(q - q_begin) & 1]); with_stores: the scores in val go out between the steps
    auto products = [&](int q, float *sdst, auto with_stores) {
        const scq16_half8 *buf = Bs[(q - q_begin) & 1];
        uint32_t kbits;  // 2^11 twice over in fp16, produced here so that the scaled operands are not hoisted out of the loop
        asm volatile("s_mov_b32 %0, 0x68006800" : "=s"(kbits));
        const scq16_half2 k2 = __builtin_bit_cast(scq16_half2, kbits);
        const scq16_half8 k2048 = {k2.x, k2.y, k2.x, k2.y, k2.x, k2.y, k2.x, k2.y};
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;
        int lim[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            lim[t] = nvalid[t] - 4 * h;
            if (!WHOLE) asm volatile("" : "+v"(lim[t]));  // or 32 lane masks would be formed ahead of the loop and kept
        }
#pragma unroll
        for (int s = 0; s < H16_STEPS; ++s) {
            scq16_step<NT>(a, buf, lane, s, k2048, acc);
            if (decltype(with_stores)::value) {
                scq16_store_part<NT, WHOLE>(sdst, val, s, lim);
                // keeps the stores and matrix instructions of a step in that step (the compiler would gather the stores
                // at the end); LDS reads and scalar / vector arithmetic may still move across
                __builtin_amdgcn_sched_barrier(0x0106);
            }
        }
    };
    // after the matrix work of query q: the next query's operands go into the buffer that every wave finished reading
    // before the last barrier, those of the query after it are requested, and the accumulators are reduced into val
    auto finish = [&](int q) {
        scq16_half8 *nxt = Bs[(q - q_begin + 1) & 1];
        if (q + 1 < q_end) {
#pragma unroll
            for (int k = 0; k < NPRE; ++k) nxt[tid + k * H16_THREADS] = pre[k];
        }
        if (q + 2 < q_end) {
            bsrc += H16_TILE_VEC;
#pragma unroll
            for (int k = 0; k < NPRE; ++k) pre[k] = bsrc[k * H16_THREADS];
        }
        scq16_reduce<NT>(acc, val, nvalid, tile0, n_blk, q, lane, t_lo, t_hi, keepbits, ambbits, keep_words, tilemax);
        scq16_lds_barrier();  // publishes nxt; every wave is done reading buf
    };
    struct no_t { enum { value = 0 }; };
    struct yes_t { enum { value = 1 }; };
    float *s0 = STORE ? S + ((int64_t)q_begin * C + (tile0 << 5) + 4 * h) * QLEN + n : nullptr;  // of the query whose stores are due
    products(q_begin, s0, no_t());
    finish(q_begin);
    for (int q = q_begin + 1; q < q_end; ++q) {
        if (STORE) {
            products(q, s0, yes_t());
            s0 += C * QLEN;
        } else {
            products(q, s0, no_t());
        }
        finish(q);
    }
    if (STORE) {  // the last query's scores
        int lim[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t) lim[t] = nvalid[t] - 4 * h;
#pragma unroll
        for (int s = 0; s < H16_STEPS; ++s) scq16_store_part<NT, WHOLE>(s0, val, s, lim);
    }
}

// Grid: x = block of 32 * H16_WAVES * NT centroids, y = group of qg queries.  A16: a whole number of workgroups' tiles
// (rows past C are zero).  keepbits / ambbits: [q][keep_words], bit c = row c passes Eq. 5 for sure / is ambiguous;
// tilemax: [q][ceil(C/32)][32].
// The loop over the group's queries is software-pipelined twice over.  Operands: those of query q + 1 are requested
// before the matrix instructions of query q, moved into the other LDS buffer right after them (by then they have
// arrived), and those of q + 2 are requested.  Scores: the results of query q leave the accumulators (scaled, reduced
// for the tile maxima and the pruning words) into registers of their own, and their stores are issued between the
// matrix instructions of query q + 1, a few per step, so that the store stream and the matrix pipe run side by side.
// STORE = false: the scores themselves are not written, only the tile maxima and the pruning words (nearest-centroid
// assignment, which re-evaluates the rows of the best tile).
template <int NT, bool STORE>
__global__ __launch_bounds__(H16_THREADS, NT == 2 ? 2 : 4) void scq16_kernel(
    const scq16_half8 *__restrict__ A16, int64_t C, const scq16_half8 *__restrict__ B16, int nq, int qg, float t_lo, float t_hi,
    float *__restrict__ S, uint32_t *__restrict__ keepbits, uint32_t *__restrict__ ambbits, int64_t keep_words,
    float *__restrict__ tilemax, unsigned long long *__restrict__ clocks)
{
    __shared__ scq16_half8 Bs[2][H16_TILE_VEC];
    // clocks (may be null): every workgroup adds how far the shader-clock counter and the fixed-rate (100 MHz) timer moved
    // while it ran -- the ratio of the two sums is the clock the chip held during this kernel
    const long long sc0 = clocks ? clock64() : 0, rt0 = clocks ? wall_clock64() : 0;
    const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
    const int64_t tile0 = ((int64_t)blockIdx.x * H16_WAVES + wave) * NT;
    const int q_begin = blockIdx.y * qg, q_end = q_begin + qg < nq ? q_begin + qg : nq;
    int nvalid[NT];  // (uniform) rows of each tile that exist: 0 for a tile past the end of the table
    bool whole = true;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int64_t left = C - ((tile0 + t) << 5);
        nvalid[t] = left >= 32 ? 32 : left > 0 ? (int)left : 0;
        whole = whole && nvalid[t] == 32;
    }
    // (the barriers inside are reached by all four waves in either instance: both run the same loop over the queries)
    if (whole)
        scq16_body<NT, STORE, true>(Bs, nvalid, A16, C, B16, q_begin, q_end, t_lo, t_hi, S, keepbits, ambbits, keep_words, tilemax);
    else
        scq16_body<NT, STORE, false>(Bs, nvalid, A16, C, B16, q_begin, q_end, t_lo, t_hi, S, keepbits, ambbits, keep_words, tilemax);
    if (clocks && threadIdx.x == 0) {
        atomicAdd(&clocks[0], (unsigned long long)(clock64() - sc0));
        atomicAdd(&clocks[1], (unsigned long long)(wall_clock64() - rt0));
    }
}

// max_bits[0] = bit pattern of the largest |value| among n values (a value that is not a number counts as infinite;
// bit patterns of non-negative floats order like the floats).  Zero on entry.
__global__ __launch_bounds__(256) void scq16_max_abs_kernel(const float *__restrict__ x, int64_t n, uint32_t *__restrict__ max_bits)
{
    float m = 0.f;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
        const float a = fabsf(x[i]);
        m = a == a ? fmaxf(m, a) : INFINITY;
    }
    for (int d = 1; d < 64; d <<= 1) m = fmaxf(m, __shfl_xor(m, d));
    if ((threadIdx.x & 63) == 0 && m > 0.f) atomicMax(max_bits, __float_as_uint(m));
}

// ------------------------------------------------------------------ host side
void plaid_launch_scq16_max_abs(hipStream_t st, const float *x, int64_t n, uint32_t *max_bits)
{
    int64_t g = (n + 255) / 256;
    if (g > 2048) g = 2048;
    if (g < 1) g = 1;
    hipLaunchKernelGGL(scq16_max_abs_kernel, dim3((unsigned)g), dim3(256), 0, st, x, n, max_bits);
}

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
                        uint32_t *keepbits, uint32_t *ambbits, int64_t keep_words, float *tilemax, unsigned long long *clocks)
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
                           (const scq16_half8 *)B16, nq, qg, t_lo, t_hi, S, keepbits, ambbits, keep_words, tilemax, clocks);
    else
        hipLaunchKernelGGL((scq16_kernel<H16_NT, false>), dim3(gx, gy), dim3(H16_THREADS), 0, st, (const scq16_half8 *)A16, C,
                           (const scq16_half8 *)B16, nq, qg, t_lo, t_hi, S, keepbits, ambbits, keep_words, tilemax, clocks);
}
