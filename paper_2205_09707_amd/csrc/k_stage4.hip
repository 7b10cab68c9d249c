// Stage 4 (Sections 4.4-4.5): residual decompression fused with exact MaxSim (Eq. 1).
//
// Decompression follows the lookup-table idea of Section 4.5: a packed byte indexes a 256-entry
// table held in LDS.  A reconstructed token is centroid + residual, so its dot product with a query
// token is S_cq[code][i] (already computed, Eq. 2) plus the residual's dot product: the scoring kernel
// gathers the 128-byte S_cq row of each token instead of its 512-byte centroid and contracts only the
// residuals, which take one of 2^nbits bucket weights per dimension.
//
// The contraction runs on the half-precision matrix instruction with both operands split into two fp16
// terms, x = x1 + 2^-11 x2 (|x - x1 - 2^-11 x2| <= 2^-22 |x|): three products per term, each exact in
// fp32, the leading one in one accumulator and the two cross terms in a second, scaled one.  The table
// therefore stores, per byte value, the fp16 terms of the bucket weights of the byte's dimensions, in
// the order the instruction wants them: one 16-byte LDS read yields the operand halves of four
// dimensions (2-bit codes) or the eight leading / eight trailing terms of a byte (1-bit codes), and the
// decoded 32-token x 128 residual tile never leaves registers.  Against fp32 arithmetic the residual's
// dot product loses at most 3 * 2^-22 |r||q|, far inside the score tolerance; it is 16 times cheaper on
// the matrix pipe, which leaves the kernel bound by its gathers and its decoding.
// The standalone decompression kernel below produces the reconstructed vectors themselves
// (centroid + weight, one fp32 addition).
#include "plaid_internal.h"

#include <math.h>

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef _Float16 s4_half8 __attribute__((ext_vector_type(8)));
typedef _Float16 s4_half4 __attribute__((ext_vector_type(4)));
#define S4_RESIDENT_BLOCKS 768
#define S4_SCALE 2048.0f  // 2^11

// The two fp16 terms of x: x1 = fp16(x) (0 below fp16's normal range), x2 = fp16(2^11 (x - x1)).
__device__ __forceinline__ void s4_split(float x, _Float16 &x1, _Float16 &x2)
{
    x1 = fabsf(x) >= 6.103515625e-05f ? (_Float16)x : (_Float16)0.0f;
    x2 = (_Float16)((x - (float)x1) * S4_SCALE);
}

// Table entry (byte v, quad s): weights of dimensions 4s .. 4s+3 of the 8/NBITS dimensions packed in v.
// Bucket indices are stored most-significant first.
template <int NBITS>
__device__ __forceinline__ void build_tables(float4 *wlut, uint32_t *ilut, const float *__restrict__ weights, int tid,
                                             int nthreads)
{
    constexpr int QUADS = NBITS == 2 ? 1 : 2;
    for (int e = tid; e < 256 * QUADS; e += nthreads) {
        const int v = e / QUADS, s = e % QUADS;
        uint32_t idx[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int d = 4 * s + t;  // dimension within the byte
            idx[t] = (v >> (8 - NBITS * (d + 1))) & ((1 << NBITS) - 1);
        }
        wlut[e] = make_float4(weights[idx[0]], weights[idx[1]], weights[idx[2]], weights[idx[3]]);
        if (ilut) ilut[e] = idx[0] | (idx[1] << 8) | (idx[2] << 16) | (idx[3] << 24);
    }
}
// Entry for dimensions 4*quad .. 4*quad+3 of a token whose packed residual starts at r.
template <int NBITS>
__device__ __forceinline__ int table_slot(const uint8_t *__restrict__ r, int quad)
{
    if (NBITS == 2) return r[quad];
    return 2 * r[quad >> 1] + (quad & 1);
}

// Operand table of the scoring kernel.  2-bit codes: hlut[v] = {x1 of the byte's four dimensions, x2 of the same}.
// 1-bit codes: hlut[v] = x1 of the byte's eight dimensions, hlut[256 + v] = their x2.
template <int NBITS>
__device__ __forceinline__ void build_half_tables(s4_half8 *hlut, const float *__restrict__ weights, int tid, int nthreads)
{
    for (int v = tid; v < 256; v += nthreads) {
        s4_half8 a, b;
#pragma unroll
        for (int d = 0; d < 8 / NBITS; ++d) {
            const int idx = (v >> (8 - NBITS * (d + 1))) & ((1 << NBITS) - 1);
            _Float16 x1, x2;
            s4_split(weights[idx], x1, x2);
            if (NBITS == 2) {
                a[d] = x1;
                a[4 + d] = x2;
            } else {
                a[d] = x1;
                b[d] = x2;
            }
        }
        hlut[v] = a;
        if (NBITS == 1) hlut[256 + v] = b;
    }
}

// Passages are scored 32 tokens per step with v_mfma_f32_32x32x16_f16.  Lane = 32 h + r: for the A operand r is the
// passage token of the step, for the B operand and the result r is the query token; both operands hold dimensions
// 16 s + 8 h .. 16 s + 8 h + 7 at step s of the 128 dimensions.
// COOP = false: one wave scores one passage at a time and the waves of the grid stride over the query's list (many
// passages per wave: throughput).  COOP = true: the four waves of a workgroup share a passage, each taking every
// fourth step, and combine their maxima in LDS (short lists: latency).
template <int NBITS, bool COOP>
__global__ __launch_bounds__(256, 3) void decompress_maxsim_kernel(
    const float *__restrict__ Q, const float *__restrict__ S, int64_t C, const int64_t *__restrict__ doc_offsets,
    const int32_t *__restrict__ codes, const uint8_t *__restrict__ residuals, const float *__restrict__ weights,
    const uint64_t *__restrict__ in_keys, int64_t in_stride, const int32_t *__restrict__ in_counts,
    uint64_t *__restrict__ out_keys, int64_t out_stride)
{
    constexpr int RB = 16 * NBITS;
    __shared__ s4_half8 hlut[256 * (NBITS == 2 ? 1 : 2)];
    __shared__ float wmax[4][QLEN];
    const int q = blockIdx.y;
    const int count = in_counts[q];
    if ((int)blockIdx.x * (COOP ? 1 : 4) >= count) return;  // uniform for the workgroup
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r32 = lane & 31, h = lane >> 5;
    build_half_tables<NBITS>(hlut, weights, threadIdx.x, 256);
    const float *Qq = Q + (int64_t)q * QLEN * DIM;
    const float *Sq = S + (int64_t)q * C * QLEN;
    // B operands: the two fp16 terms of query token r32, dimensions 16 s + 8 h .. + 7
    s4_half8 q1[8], q2[8];
#pragma unroll
    for (int s = 0; s < 8; ++s) {
        const float4 *p = reinterpret_cast<const float4 *>(Qq + r32 * DIM + 16 * s + 8 * h);
        const float4 u = p[0], w = p[1];
        const float x[8] = {u.x, u.y, u.z, u.w, w.x, w.y, w.z, w.w};
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            _Float16 x1, x2;
            s4_split(x[j], x1, x2);
            q1[s][j] = x1;
            q2[s][j] = x2;
        }
    }
    __syncthreads();

    for (int j = COOP ? (int)blockIdx.x : (int)blockIdx.x * 4 + wave; j < count; j += (int)gridDim.x * (COOP ? 1 : 4)) {
        // passage id, first token and length are the same in every lane: kept in scalar registers, so that the loops
        // below run with the whole wave active
        const uint32_t pid = (uint32_t)__builtin_amdgcn_readfirstlane((int)(in_keys[(int64_t)q * in_stride + j] & 0xFFFFFFFFu));
        const int64_t t0v = doc_offsets[pid];
        const int64_t t0 = ((int64_t)__builtin_amdgcn_readfirstlane((int)(t0v >> 32)) << 32) |
                           (uint32_t)__builtin_amdgcn_readfirstlane((int)(t0v & 0xFFFFFFFFll));
        const int len = __builtin_amdgcn_readfirstlane((int)(doc_offsets[pid + 1] - t0v));
        float m = -INFINITY;  // running maximum for query token r32 over the rows this lane sees
        // The loop is software-pipelined: the code and packed residual of the next step and the S_cq values of this
        // step are requested before this step's matrix instructions are issued, so their latency runs under them.
        constexpr int STEP = COOP ? 128 : 32;
        int base = COOP ? 32 * wave : 0;
        int32_t code = 0;
        uint32_t rw[RB / 4] = {0};
        auto request = [&](int b, int32_t &c, uint32_t (&r)[RB / 4]) {
            const int row = b + r32;  // this lane's passage token
            const int64_t tok = t0 + (row < len ? row : len - 1);
            c = codes[tok];
            // the token's packed residual: both halves of the wave read all of it, each uses half of the bytes
            const uint4 *rp = reinterpret_cast<const uint4 *>(residuals + tok * RB);
            const uint4 v0 = rp[0];
            r[0] = v0.x, r[1] = v0.y, r[2] = v0.z, r[3] = v0.w;
            if (NBITS == 2) {
                const uint4 v1 = rp[1];
                r[4] = v1.x, r[5] = v1.y, r[6] = v1.z, r[7] = v1.w;
            }
        };
        if (base < len) request(base, code, rw);
        for (; base < len; base += STEP) {
            // the centroid's share of each dot product: row code of S_cq, element r32 (requested now, used after the
            // matrix instructions); acc[v] will hold passage token base + 8 (v/4) + 4h + v%4 against query token r32
            float sv[16];
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int rr = 8 * (v >> 2) + 4 * h + (v & 3);
                const uint32_t cv = (uint32_t)__shfl(code, rr);
                sv[v] = Sq[cv * (uint32_t)QLEN + (uint32_t)r32];
            }
            int32_t code_next = 0;
            uint32_t rw_next[RB / 4] = {0};
            if (base + STEP < len) request(base + STEP, code_next, rw_next);  // uniform
            floatx16 acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
            floatx16 acx = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};  // cross terms, scaled by 2^11
#pragma unroll
            for (int s = 0; s < 8; ++s) {
                // dimensions 16 s + 8 h .. + 7: bytes 4 s + 2 h and 4 s + 2 h + 1 of a 2-bit code, byte 2 s + h of a 1-bit one
                s4_half8 a1, a2;
                if (NBITS == 2) {
                    const uint32_t two = rw[s] >> (16 * h);
                    const s4_half8 e0 = hlut[two & 0xFF], e1 = hlut[(two >> 8) & 0xFF];
                    a1 = s4_half8{e0[0], e0[1], e0[2], e0[3], e1[0], e1[1], e1[2], e1[3]};
                    a2 = s4_half8{e0[4], e0[5], e0[6], e0[7], e1[4], e1[5], e1[6], e1[7]};
                } else {
                    const uint32_t b = (rw[s >> 1] >> (16 * (s & 1) + 8 * h)) & 0xFF;
                    a1 = hlut[b];
                    a2 = hlut[256 + b];
                }
                acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(a1, q1[s], acc, 0, 0, 0);
                acx = __builtin_amdgcn_mfma_f32_32x32x16_f16(a1, q2[s], acx, 0, 0, 0);
                acx = __builtin_amdgcn_mfma_f32_32x32x16_f16(a2, q1[s], acx, 0, 0, 0);
            }
            if (base + 32 <= len) {  // (uniform) a full step: every row counts
#pragma unroll
                for (int v = 0; v < 16; ++v) m = fmaxf(m, fmaf(acx[v], 1.0f / S4_SCALE, acc[v]) + sv[v]);
            } else {
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    if (base + 8 * (v >> 2) + 4 * h + (v & 3) < len) m = fmaxf(m, fmaf(acx[v], 1.0f / S4_SCALE, acc[v]) + sv[v]);
            }
            code = code_next;
#pragma unroll
            for (int e = 0; e < RB / 4; ++e) rw[e] = rw_next[e];
        }
        m = fmaxf(m, __shfl_xor(m, 32));
        if (COOP) {  // j, len are the same in the four waves
            if (h == 0) wmax[wave][r32] = m;
            __syncthreads();
            m = fmaxf(fmaxf(wmax[0][r32], wmax[1][r32]), fmaxf(wmax[2][r32], wmax[3][r32]));
            __syncthreads();
        }
        const float total = plaid_sum32_in_order(m);
        if (lane == 0 && (!COOP || wave == 0))
            out_keys[(int64_t)q * out_stride + j] = plaid_make_key(len > 0 ? total : -INFINITY, pid);
    }
}

// Vanilla ColBERTv2's pruning of an over-large candidate set (Section 4.1): a candidate's score from the embeddings
// of E alone, E = the tokens whose centroid was probed (probebits: bit c = centroid c probed), each decompressed in full
// like in the kernel above.  One wave per candidate; the tokens of E are compacted through a small LDS ring so that
// the matrix instructions run on full 32-token steps whatever share of a passage E covers.  Queries whose candidate
// count does not exceed ncandidates keep every candidate and are not scored: their keys get score 0.
//   cand: [q][cand_stride] ascending candidate pids, n_cand[q] of them;  out_keys[q][j] = key of cand[q][j].
template <int NBITS>
__global__ __launch_bounds__(256, 3) void vanilla_prune_kernel(
    const float *__restrict__ Q, const float *__restrict__ S, int64_t C, const int64_t *__restrict__ doc_offsets,
    const int32_t *__restrict__ codes, const uint8_t *__restrict__ residuals, const float *__restrict__ weights,
    const uint32_t *__restrict__ probebits, int64_t keep_words, const int32_t *__restrict__ cand, int64_t cand_stride,
    const int32_t *__restrict__ n_cand, int32_t ncandidates, uint64_t *__restrict__ out_keys, int64_t out_stride)
{
    constexpr int RB = 16 * NBITS;
    __shared__ s4_half8 hlut[256 * (NBITS == 2 ? 1 : 2)];
    __shared__ int32_t ring_all[4][128];
    const int q = blockIdx.y;
    const int count = n_cand[q];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int32_t *cq = cand + (int64_t)q * cand_stride;
    if (count <= ncandidates) {  // (uniform) no pruning for this query
        for (int j = blockIdx.x * 256 + threadIdx.x; j < count; j += gridDim.x * 256)
            out_keys[(int64_t)q * out_stride + j] = plaid_make_key(0.0f, (uint32_t)cq[j]);
        return;
    }
    const int r32 = lane & 31, h = lane >> 5;
    build_half_tables<NBITS>(hlut, weights, threadIdx.x, 256);
    const float *Qq = Q + (int64_t)q * QLEN * DIM;
    const float *Sq = S + (int64_t)q * C * QLEN;
    const uint32_t *pb = probebits + (int64_t)q * keep_words;
    s4_half8 q1[8], q2[8];
#pragma unroll
    for (int s = 0; s < 8; ++s) {
        const float4 *p = reinterpret_cast<const float4 *>(Qq + r32 * DIM + 16 * s + 8 * h);
        const float4 u = p[0], w = p[1];
        const float x[8] = {u.x, u.y, u.z, u.w, w.x, w.y, w.z, w.w};
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            _Float16 x1, x2;
            s4_split(x[j], x1, x2);
            q1[s][j] = x1;
            q2[s][j] = x2;
        }
    }
    __syncthreads();
    int32_t *ring = ring_all[wave];
    for (int j = (int)blockIdx.x * 4 + wave; j < count; j += (int)gridDim.x * 4) {
        const uint32_t pid = (uint32_t)__builtin_amdgcn_readfirstlane(cq[j]);
        const int64_t t0v = doc_offsets[pid];
        const int64_t t0 = ((int64_t)__builtin_amdgcn_readfirstlane((int)(t0v >> 32)) << 32) |
                           (uint32_t)__builtin_amdgcn_readfirstlane((int)(t0v & 0xFFFFFFFFll));
        const int len = __builtin_amdgcn_readfirstlane((int)(doc_offsets[pid + 1] - t0v));
        float m = -INFINITY;
        int have = 0, done = 0;  // uniform: tokens of E listed so far / scored so far
        for (int src = 0; src < len || done < have; src += 64) {
            if (src < len) {
                const int row = src + lane;
                const int32_t c = row < len ? codes[t0 + row] : 0;
                const bool in = row < len && ((pb[c >> 5] >> (c & 31)) & 1u);
                const unsigned long long mask = __ballot(in);
                if (in) ring[(have + __popcll(mask & ((1ull << lane) - 1ull))) & 127] = row;
                have += __popcll(mask);
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            }
            // full steps while 32 listed tokens wait; the remainder once the passage has been read
            while (have - done >= 32 || (src + 64 >= len && done < have)) {
                const int nrow = have - done < 32 ? have - done : 32;  // uniform
                const int row = ring[(done + (r32 < nrow ? r32 : 0)) & 127];
                const int64_t tok = t0 + row;
                const int32_t code = codes[tok];
                uint32_t rw[RB / 4];
                {
                    const uint4 *rp = reinterpret_cast<const uint4 *>(residuals + tok * RB);
                    const uint4 v0 = rp[0];
                    rw[0] = v0.x, rw[1] = v0.y, rw[2] = v0.z, rw[3] = v0.w;
                    if (NBITS == 2) {
                        const uint4 v1 = rp[1];
                        rw[4] = v1.x, rw[5] = v1.y, rw[6] = v1.z, rw[7] = v1.w;
                    }
                }
                float sv[16];
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int rr = 8 * (v >> 2) + 4 * h + (v & 3);
                    const uint32_t cv = (uint32_t)__shfl(code, rr);
                    sv[v] = Sq[cv * (uint32_t)QLEN + (uint32_t)r32];
                }
                floatx16 acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
                floatx16 acx = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
                for (int s = 0; s < 8; ++s) {
                    s4_half8 a1, a2;
                    if (NBITS == 2) {
                        const uint32_t two = rw[s] >> (16 * h);
                        const s4_half8 e0 = hlut[two & 0xFF], e1 = hlut[(two >> 8) & 0xFF];
                        a1 = s4_half8{e0[0], e0[1], e0[2], e0[3], e1[0], e1[1], e1[2], e1[3]};
                        a2 = s4_half8{e0[4], e0[5], e0[6], e0[7], e1[4], e1[5], e1[6], e1[7]};
                    } else {
                        const uint32_t b = (rw[s >> 1] >> (16 * (s & 1) + 8 * h)) & 0xFF;
                        a1 = hlut[b];
                        a2 = hlut[256 + b];
                    }
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(a1, q1[s], acc, 0, 0, 0);
                    acx = __builtin_amdgcn_mfma_f32_32x32x16_f16(a1, q2[s], acx, 0, 0, 0);
                    acx = __builtin_amdgcn_mfma_f32_32x32x16_f16(a2, q1[s], acx, 0, 0, 0);
                }
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    if (8 * (v >> 2) + 4 * h + (v & 3) < nrow) m = fmaxf(m, fmaf(acx[v], 1.0f / S4_SCALE, acc[v]) + sv[v]);
                done += nrow;
            }
        }
        m = fmaxf(m, __shfl_xor(m, 32));
        const float total = plaid_sum32_in_order(m);
        if (lane == 0) out_keys[(int64_t)q * out_stride + j] = plaid_make_key(have > 0 ? total : -INFINITY, pid);
    }
}

void plaid_launch_vanilla_prune(hipStream_t st, const float *Q, const float *S, int64_t C, const int64_t *doc_offsets,
                                const int32_t *codes, const uint8_t *residuals, const float *bucket_weights, int nbits,
                                const uint32_t *probebits, int64_t keep_words, int nq, const int32_t *cand, int64_t cand_stride,
                                const int32_t *n_cand, int64_t n_upper, int32_t ncandidates, uint64_t *out_keys,
                                int64_t out_stride)
{
    if (n_upper <= 0 || nq <= 0) return;
    int64_t gx = (n_upper + 3) / 4;
    const int64_t cap = (S4_RESIDENT_BLOCKS * 4 + nq - 1) / nq;
    if (gx > cap) gx = cap;
    if (gx < 1) gx = 1;
    if (nbits == 2)
        hipLaunchKernelGGL(vanilla_prune_kernel<2>, dim3((unsigned)gx, nq), dim3(256), 0, st, Q, S, C, doc_offsets, codes, residuals,
                           bucket_weights, probebits, keep_words, cand, cand_stride, n_cand, ncandidates, out_keys, out_stride);
    else
        hipLaunchKernelGGL(vanilla_prune_kernel<1>, dim3((unsigned)gx, nq), dim3(256), 0, st, Q, S, C, doc_offsets, codes, residuals,
                           bucket_weights, probebits, keep_words, cand, cand_stride, n_cand, ncandidates, out_keys, out_stride);
}

void plaid_launch_decompress_maxsim(hipStream_t st, const float *Q, const float *S, int64_t C, const int64_t *doc_offsets,
                                    const int32_t *codes, const uint8_t *residuals, const float *bucket_weights,
                                    int nbits, int nq, const uint64_t *in_keys, int64_t in_stride,
                                    const int32_t *in_counts, int n_upper, uint64_t *out_keys, int64_t out_stride)
{
    if (n_upper <= 0 || nq <= 0) return;
    // few passages in all (short lists of few queries): a workgroup per passage; otherwise waves stride over the lists,
    // several passages each, so that the per-workgroup set-up (table, query operands) is paid rarely
    const bool coop = (int64_t)n_upper * nq <= 2048;
    int gx = coop ? n_upper : (n_upper + 3) / 4;
    // (256 compute units x 3 resident workgroups: one full round of waves, each striding over several passages)
    const int cap = coop ? 2048 : (S4_RESIDENT_BLOCKS + nq - 1) / nq;
    if (gx > cap) gx = cap;
#define PLAID_S4_LAUNCH(NB, CO)                                                                                           \
    hipLaunchKernelGGL((decompress_maxsim_kernel<NB, CO>), dim3(gx, nq), dim3(256), 0, st, Q, S, C, doc_offsets, codes,       \
                       residuals, bucket_weights, in_keys, in_stride, in_counts, out_keys, out_stride)
    if (nbits == 2) {
        if (coop) PLAID_S4_LAUNCH(2, true);
        else PLAID_S4_LAUNCH(2, false);
    } else {
        if (coop) PLAID_S4_LAUNCH(1, true);
        else PLAID_S4_LAUNCH(1, false);
    }
#undef PLAID_S4_LAUNCH
}

// ------------------------------------------------------------------ decompression alone (parity of the codec)
__global__ __launch_bounds__(256) void passage_offsets_kernel(const int64_t *__restrict__ doc_offsets,
                                                              const int32_t *__restrict__ pids, int n,
                                                              int64_t *__restrict__ out_offsets)
{
    // one workgroup; serial carry across chunks of 256 passages
    __shared__ int64_t scan[256];
    __shared__ int64_t carry;
    if (threadIdx.x == 0) {
        carry = 0;
        out_offsets[0] = 0;
    }
    __syncthreads();
    for (int base = 0; base < n; base += 256) {
        const int e = base + threadIdx.x;
        int64_t len = 0;
        if (e < n) len = doc_offsets[pids[e] + 1] - doc_offsets[pids[e]];
        scan[threadIdx.x] = len;
        __syncthreads();
        for (int d = 1; d < 256; d <<= 1) {
            const int64_t t = threadIdx.x >= d ? scan[threadIdx.x - d] : 0;
            __syncthreads();
            scan[threadIdx.x] += t;
            __syncthreads();
        }
        if (e < n) out_offsets[e + 1] = carry + scan[threadIdx.x];
        __syncthreads();
        if (threadIdx.x == 255) carry += scan[255];
        __syncthreads();
    }
}
void plaid_launch_passage_offsets(hipStream_t st, const int64_t *doc_offsets, const int32_t *pids, int n,
                                  int64_t *out_offsets)
{
    hipLaunchKernelGGL(passage_offsets_kernel, dim3(1), dim3(256), 0, st, doc_offsets, pids, n, out_offsets);
}

// Same table, same lookup and same addition as the fused kernel; thread t handles dimensions 4t .. 4t+3.
template <int NBITS>
__global__ __launch_bounds__(256) void decompress_dump_kernel(const float *__restrict__ centroids,
                                                              const int64_t *__restrict__ doc_offsets,
                                                              const int32_t *__restrict__ codes,
                                                              const uint8_t *__restrict__ residuals,
                                                              const float *__restrict__ weights,
                                                              const int32_t *__restrict__ pids,
                                                              const int64_t *__restrict__ out_offsets,
                                                              float *__restrict__ out_vectors,
                                                              uint8_t *__restrict__ out_indices)
{
    constexpr int RB = 16 * NBITS;
    __shared__ float4 wlut[256 * (NBITS == 2 ? 1 : 2)];
    __shared__ uint32_t ilut[256 * (NBITS == 2 ? 1 : 2)];
    build_tables<NBITS>(wlut, ilut, weights, threadIdx.x, 256);
    __syncthreads();
    const int a = blockIdx.x;
    const int32_t pid = pids[a];
    const int64_t t0 = doc_offsets[pid];
    const int len = (int)(doc_offsets[pid + 1] - t0);
    const int64_t o0 = out_offsets[a];
    const int quad = threadIdx.x & 31;
    for (int row = threadIdx.x >> 5; row < len; row += 8) {
        const int64_t tok = t0 + row;
        const float *crow = centroids + (int64_t)codes[tok] * DIM;
        const int slot = table_slot<NBITS>(residuals + tok * RB, quad);
        const float4 c = *reinterpret_cast<const float4 *>(crow + 4 * quad);
        const float4 w = wlut[slot];
        if (out_vectors)
            *reinterpret_cast<float4 *>(out_vectors + (o0 + row) * DIM + 4 * quad) =
                make_float4(c.x + w.x, c.y + w.y, c.z + w.z, c.w + w.w);
        if (out_indices) *reinterpret_cast<uint32_t *>(out_indices + (o0 + row) * DIM + 4 * quad) = ilut[slot];
    }
}
void plaid_launch_decompress_dump(hipStream_t st, const float *centroids, const int64_t *doc_offsets,
                                  const int32_t *codes, const uint8_t *residuals, const float *bucket_weights,
                                  int nbits, const int32_t *pids, int n, const int64_t *out_offsets, float *out_vectors,
                                  uint8_t *out_indices)
{
    if (n <= 0) return;
    if (nbits == 2)
        hipLaunchKernelGGL(decompress_dump_kernel<2>, dim3(n), dim3(256), 0, st, centroids, doc_offsets, codes, residuals,
                           bucket_weights, pids, out_offsets, out_vectors, out_indices);
    else
        hipLaunchKernelGGL(decompress_dump_kernel<1>, dim3(n), dim3(256), 0, st, centroids, doc_offsets, codes, residuals,
                           bucket_weights, pids, out_offsets, out_vectors, out_indices);
}
