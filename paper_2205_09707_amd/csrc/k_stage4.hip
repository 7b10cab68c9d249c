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
#define S4_RESIDENT_BLOCKS 1024
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

// Column maxima of a 32 x 32 result block spread over the wave as the matrix instruction leaves it: lane 32 h + n holds
// mx[v] = the value of query token 8 (v / 4) + 4 h + v % 4 for passage-token column n.  Returns, in lane 32 h + 2 v (and
// its odd neighbour), the maximum over the 32 columns for that query token: a butterfly in which each exchange halves the
// number of values a lane still carries (16 exchanges instead of 16 x 5).
__device__ __forceinline__ float s4_column_maxima(const float (&mx)[16], int lane)
{
    float a8[8], a4[4], a2[2];
    const bool b4 = lane & 16, b3 = lane & 8, b2 = lane & 4, b1 = lane & 2;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const float keep = b4 ? mx[8 + e] : mx[e], send = b4 ? mx[e] : mx[8 + e];
        a8[e] = fmaxf(keep, __shfl_xor(send, 16));
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const float keep = b3 ? a8[4 + e] : a8[e], send = b3 ? a8[e] : a8[4 + e];
        a4[e] = fmaxf(keep, __shfl_xor(send, 8));
    }
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        const float keep = b2 ? a4[2 + e] : a4[e], send = b2 ? a4[e] : a4[2 + e];
        a2[e] = fmaxf(keep, __shfl_xor(send, 4));
    }
    const float keep = b1 ? a2[1] : a2[0], send = b1 ? a2[0] : a2[1];
    const float a1 = fmaxf(keep, __shfl_xor(send, 2));
    return fmaxf(a1, __shfl_xor(a1, 1));
}
// The lane that holds query token i after s4_column_maxima, and the query token of an even lane.
__device__ __forceinline__ constexpr int s4_lane_of_token(int i) { return 32 * ((i >> 2) & 1) + 2 * (4 * (i >> 3) + (i & 3)); }
__device__ __forceinline__ int s4_token_of_lane(int lane)
{
    const int v = (lane >> 1) & 15;
    return 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
}

// Passages are scored 32 tokens per step with v_mfma_f32_32x32x16_f16: rows = the 32 query tokens (A operand), columns
// = 32 passage tokens (B operand); lane 32 h + r holds row / column r of its operand, dimensions 16 s + 8 h .. + 7 at
// step s of the 128 dimensions.  A lane therefore decodes the residual of one passage token, gets the results of that
// token's column (16 query tokens: 8 g + 4 h + 0..3), and adds the centroid's share from its own token's row of S_cq
// (four 16-byte loads, no exchange between lanes).  It keeps 16 running maxima over the steps of a passage; the maxima
// over the columns are taken once per passage (s4_column_maxima).
// COOP = false: one wave scores one passage at a time and the waves of the grid stride over the query's list (many
// passages per wave: throughput).  COOP = true: the four waves of a workgroup share a passage, each taking every
// fourth step, and combine their maxima in LDS (short lists: latency).
// The grid is one-dimensional; with eight queries or more (spread = 0) workgroup L serves query 8 (L / 8 / gx) + L % 8:
// consecutive workgroups go to the chip's eight partitions in turn, so a query's workgroups share one partition's
// second-level cache and the rows of S_cq its passages have in common are fetched once.
// RN: the storage variant in which a reconstructed vector is scaled to unit length: its dot products are multiplied by
// the token's factor inv_norm[token] = 1 / |centroid + residual| (plaid_launch_token_inv_norm).
template <int NBITS, bool COOP, bool RN>
__global__ __launch_bounds__(256, 4) void decompress_maxsim_kernel(
    const float *__restrict__ Q, const float *__restrict__ S, int64_t C, const int64_t *__restrict__ doc_offsets,
    const int32_t *__restrict__ codes, const uint8_t *__restrict__ residuals, const float *__restrict__ weights,
    const float *__restrict__ inv_norm,
    const uint64_t *__restrict__ in_keys, int64_t in_stride, const int32_t *__restrict__ in_counts, int nq, int gx,
    int spread, uint64_t *__restrict__ out_keys, int64_t out_stride)
{
    constexpr int RB = 16 * NBITS;
    __shared__ s4_half8 hlut[256 * (NBITS == 2 ? 1 : 2)];
    __shared__ float wmax[4][QLEN];
    __shared__ s4_half8 qs[2][8][64];  // [term][step of 16 dimensions][lane]
    int q, bx;
    if (spread) {
        q = blockIdx.x / gx;
        bx = blockIdx.x % gx;
    } else {
        const int k = blockIdx.x >> 3;
        q = 8 * (k / gx) + (blockIdx.x & 7);
        bx = k % gx;
    }
    if (q >= nq) return;
    const int count = in_counts[q];
    if (bx * (COOP ? 1 : 4) >= count) return;  // uniform for the workgroup
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r32 = lane & 31, h = lane >> 5;
    build_half_tables<NBITS>(hlut, weights, threadIdx.x, 256);
    const float *Qq = Q + (int64_t)q * QLEN * DIM;
    const char *Sq = reinterpret_cast<const char *>(S + (int64_t)q * C * QLEN);
    // A operands: the two fp16 terms of query token r32, dimensions 16 s + 8 h .. + 7.  They are the same for the four
    // waves and stay in LDS (16 KB), from where each matrix step reads them: 64 registers less per lane, which buys a
    // third wave per SIMD to cover the latency of the gathers.
    for (int e = threadIdx.x; e < 8 * 64; e += 256) {
        const int s = e >> 6, l = e & 63;
        const float4 *p = reinterpret_cast<const float4 *>(Qq + (l & 31) * DIM + 16 * s + 8 * (l >> 5));
        const float4 u = p[0], w = p[1];
        const float x[8] = {u.x, u.y, u.z, u.w, w.x, w.y, w.z, w.w};
        s4_half8 t1, t2;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            _Float16 x1, x2;
            s4_split(x[j], x1, x2);
            t1[j] = x1;
            t2[j] = x2;
        }
        qs[0][s][l] = t1;
        qs[1][s][l] = t2;
    }
    __syncthreads();

    // In front of a passage's first step stands a chain of dependent loads: its id (from the key list), its token range,
    // its first codes and residuals.  The chain is started three passages ahead and advanced one link per passage, and the
    // first step's operands of the next passage are requested during the last step of this one, so that a wave never
    // waits for the whole chain.  Ids and ranges are the same in every lane; they are still fetched with vector loads
    // (a zero the compiler cannot see through is added to the index), which return in order and are counted apart from
    // LDS reads.  List positions past the end repeat the last passage (loaded, not scored).
    int vz;
    asm volatile("v_mov_b32 %0, 0" : "=v"(vz));
    const uint32_t *ik = reinterpret_cast<const uint32_t *>(in_keys + (int64_t)q * in_stride);  // low word: passage id
    const int j0 = COOP ? bx : bx * 4 + wave, jstride = gx * (COOP ? 1 : 4);
    auto load_id = [&](int n) -> uint32_t {
        const int64_t jj = (int64_t)j0 + (int64_t)n * jstride;
        return ik[2 * (jj < count ? jj : (int64_t)count - 1) + vz];
    };
    auto uniform64 = [](int64_t v) -> int64_t {
        return ((int64_t)__builtin_amdgcn_readfirstlane((int)(v >> 32)) << 32) |
               (uint32_t)__builtin_amdgcn_readfirstlane((int)(v & 0xFFFFFFFFll));
    };
    constexpr int RW = RB / 4;
    auto request = [&](int64_t t0, int len, int b, int32_t &c, float &nf, uint32_t (&r)[RW]) {
        const int row = b + r32;  // this lane's passage token
        const int64_t tok = t0 + (row < len ? row : len - 1);
        c = codes[tok];
        if (RN) nf = inv_norm[tok];
        // the token's packed residual: both halves of the wave read all of it, each uses half of the bytes
        const uint4 *rp = reinterpret_cast<const uint4 *>(residuals + tok * RB);
        const uint4 v0 = rp[0];
        r[0] = v0.x, r[1] = v0.y, r[2] = v0.z, r[3] = v0.w;
        if (NBITS == 2) {
            const uint4 v1 = rp[1];
            r[4] = v1.x, r[5] = v1.y, r[6] = v1.z, r[7] = v1.w;
        }
    };
    constexpr int STEP = COOP ? 128 : 32;
    const int base0 = COOP ? 32 * wave : 0;
    // warm-up: passage 0 completely, passage 1 up to its token range, passage 2's id
    uint32_t pid = (uint32_t)__builtin_amdgcn_readfirstlane((int)load_id(0));
    int64_t t0 = uniform64(doc_offsets[(int64_t)pid + vz]);
    int len = (int)(uniform64(doc_offsets[(int64_t)pid + 1 + vz]) - t0);
    int32_t code = 0;
    float nf = 1.0f;  // this lane's token's scaling factor (RN)
    uint32_t rw[RW] = {0};
    if (base0 < len) request(t0, len, base0, code, nf, rw);
    uint32_t pid1 = (uint32_t)__builtin_amdgcn_readfirstlane((int)load_id(1));
    int64_t o1a = doc_offsets[(int64_t)pid1 + vz], o1b = doc_offsets[(int64_t)pid1 + 1 + vz];  // as loaded (same in every lane)
    uint32_t id2 = load_id(2);
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): the loop's waits then cover only what the loop itself requests

    for (int n = 0; (int64_t)j0 + (int64_t)n * jstride < count; ++n) {
        const int j = j0 + n * jstride;
        // one link further for the passages ahead
        const int64_t t0_next = uniform64(o1a);
        const int len_next = (int)(uniform64(o1b) - t0_next);
        const uint32_t pid2 = (uint32_t)__builtin_amdgcn_readfirstlane((int)id2);
        const int64_t o2a = doc_offsets[(int64_t)pid2 + vz], o2b = doc_offsets[(int64_t)pid2 + 1 + vz];
        const uint32_t id3 = load_id(n + 3);
        int32_t code_next = 0;
        float nf_next = 1.0f;
        uint32_t rw_next[RW] = {0};
        bool next_requested = false;
        float mx[16];  // running maxima of this lane's column class: query token 8 (v / 4) + 4 h + v % 4
#pragma unroll
        for (int v = 0; v < 16; ++v) mx[v] = -INFINITY;
        // The step loop is software-pipelined too: the code and packed residual of the next step and the S_cq values of
        // this step are requested before this step's matrix instructions are issued.
        for (int base = base0; base < len; base += STEP) {
            // the centroid's share of each dot product: the token's row of S_cq, elements 8 g + 4 h .. + 3 (requested now,
            // used after the matrix instructions)
            float4 sv[4];
            {
                const uint32_t off = (uint32_t)code * (uint32_t)(QLEN * 4) + 16u * (uint32_t)h;
#pragma unroll
                for (int g = 0; g < 4; ++g) sv[g] = *reinterpret_cast<const float4 *>(Sq + off + 32u * g);
            }
            if (base + STEP < len) {  // uniform
                request(t0, len, base + STEP, code_next, nf_next, rw_next);
            } else {  // last step: the first step of the next passage
                if (base0 < len_next) request(t0_next, len_next, base0, code_next, nf_next, rw_next);
                next_requested = true;
            }
            floatx16 acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
            floatx16 acx = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};  // cross terms, scaled by 2^11
            // (the query operands are read anew in every step, through an index the compiler cannot tell from the last
            // step's: kept across steps they would take the 64 registers again)
            int ql = lane;
            asm volatile("" : "+v"(ql));
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
                const s4_half8 q1 = qs[0][s][ql], q2 = qs[1][s][ql];
                acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(q1, a1, acc, 0, 0, 0);
                acx = __builtin_amdgcn_mfma_f32_32x32x16_f16(q2, a1, acx, 0, 0, 0);
                acx = __builtin_amdgcn_mfma_f32_32x32x16_f16(q1, a2, acx, 0, 0, 0);
            }
            const float svf[16] = {sv[0].x, sv[0].y, sv[0].z, sv[0].w, sv[1].x, sv[1].y, sv[1].z, sv[1].w,
                                   sv[2].x, sv[2].y, sv[2].z, sv[2].w, sv[3].x, sv[3].y, sv[3].z, sv[3].w};
            // (med3(a, b, +inf) = max(a, b) for ordered operands, without the canonicalising copies of fmaxf)
            if (base + 32 <= len) {  // (uniform) a full step: every column counts
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    float x = fmaf(acx[v], 1.0f / S4_SCALE, acc[v]) + svf[v];
                    if (RN) x *= nf;
                    mx[v] = __builtin_amdgcn_fmed3f(mx[v], x, INFINITY);
                }
            } else if (base + r32 < len) {  // this lane's column is a token of the passage
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    float x = fmaf(acx[v], 1.0f / S4_SCALE, acc[v]) + svf[v];
                    if (RN) x *= nf;
                    mx[v] = __builtin_amdgcn_fmed3f(mx[v], x, INFINITY);
                }
            }
            code = code_next;
            nf = nf_next;
#pragma unroll
            for (int e = 0; e < RW; ++e) rw[e] = rw_next[e];
        }
        if (!next_requested && base0 < len_next) request(t0_next, len_next, base0, code, nf, rw);  // (uniform) no step was taken
        const float cm = s4_column_maxima(mx, lane);  // query token s4_token_of_lane(lane), in even and odd lane alike
        float total;
        if (COOP) {  // j, len are the same in the four waves
            if (!(lane & 1)) wmax[wave][s4_token_of_lane(lane)] = cm;
            __syncthreads();
            const float m = fmaxf(fmaxf(wmax[0][r32], wmax[1][r32]), fmaxf(wmax[2][r32], wmax[3][r32]));
            __syncthreads();
            total = plaid_sum32_in_order(m);
        } else {
            // the sum over the query tokens of Eq. 1, in double, in index order
            double d = 0.0;
#pragma unroll
            for (int i = 0; i < QLEN; ++i)
                d += (double)__int_as_float(__builtin_amdgcn_readlane(__float_as_int(cm), s4_lane_of_token(i)));
            total = (float)d;
        }
        if (lane == 0 && (!COOP || wave == 0))
            out_keys[(int64_t)q * out_stride + j] = plaid_make_key(len > 0 ? total : -INFINITY, pid);
        // the passages ahead move up
        pid = pid1, t0 = t0_next, len = len_next;
        pid1 = pid2, o1a = o2a, o1b = o2b;
        id2 = id3;
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
                                    const int32_t *in_counts, int n_upper, uint64_t *out_keys, int64_t out_stride,
                                    const float *inv_norm)
{
    if (n_upper <= 0 || nq <= 0) return;
    // few passages in all (short lists of few queries): a workgroup per passage; otherwise waves stride over the lists,
    // several passages each, so that the per-workgroup set-up (table, query operands) is paid rarely
    const bool coop = (int64_t)n_upper * nq <= 2048;
    int gx = coop ? n_upper : (n_upper + 3) / 4;
    // (256 compute units x 4 resident workgroups: one full round of waves, each striding over several passages)
    const int cap = coop ? 2048 : (S4_RESIDENT_BLOCKS + nq - 1) / nq;
    if (gx > cap) gx = cap;
    const int spread = nq < 8 ? 1 : 0;
    const int64_t slots = spread ? nq : 8 * (((int64_t)nq + 7) / 8);  // query slots of the one-dimensional grid
    if (slots * gx > (1ll << 23)) gx = (int)((1ll << 23) / slots);  // (the waves stride over longer lists)
    if (gx < 1) gx = 1;
#define PLAID_S4_LAUNCH(NB, CO, RN)                                                                                       \
    hipLaunchKernelGGL((decompress_maxsim_kernel<NB, CO, RN>), dim3((unsigned)(slots * gx)), dim3(256), 0, st, Q, S, C,      \
                       doc_offsets, codes, residuals, bucket_weights, inv_norm, in_keys, in_stride, in_counts, nq, gx,       \
                       spread, out_keys, out_stride)
#define PLAID_S4_LAUNCH_RN(NB, CO)                                                                                        \
    do {                                                                                                                  \
        if (inv_norm) PLAID_S4_LAUNCH(NB, CO, true);                                                                      \
        else PLAID_S4_LAUNCH(NB, CO, false);                                                                              \
    } while (0)
    if (nbits == 2) {
        if (coop) PLAID_S4_LAUNCH_RN(2, true);
        else PLAID_S4_LAUNCH_RN(2, false);
    } else {
        if (coop) PLAID_S4_LAUNCH_RN(1, true);
        else PLAID_S4_LAUNCH_RN(1, false);
    }
#undef PLAID_S4_LAUNCH_RN
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
                                                              uint8_t *__restrict__ out_indices,
                                                              const float *__restrict__ inv_norm)
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
        if (out_vectors) {
            float4 d = make_float4(c.x + w.x, c.y + w.y, c.z + w.z, c.w + w.w);
            if (inv_norm) {  // scaled to unit length: one fp32 factor per token, one rounding per component
                const float f = inv_norm[tok];
                d = make_float4(d.x * f, d.y * f, d.z * f, d.w * f);
            }
            *reinterpret_cast<float4 *>(out_vectors + (o0 + row) * DIM + 4 * quad) = d;
        }
        if (out_indices) *reinterpret_cast<uint32_t *>(out_indices + (o0 + row) * DIM + 4 * quad) = ilut[slot];
    }
}
void plaid_launch_decompress_dump(hipStream_t st, const float *centroids, const int64_t *doc_offsets,
                                  const int32_t *codes, const uint8_t *residuals, const float *bucket_weights,
                                  int nbits, const int32_t *pids, int n, const int64_t *out_offsets, float *out_vectors,
                                  uint8_t *out_indices, const float *inv_norm)
{
    if (n <= 0) return;
    if (nbits == 2)
        hipLaunchKernelGGL(decompress_dump_kernel<2>, dim3(n), dim3(256), 0, st, centroids, doc_offsets, codes, residuals,
                           bucket_weights, pids, out_offsets, out_vectors, out_indices, inv_norm);
    else
        hipLaunchKernelGGL(decompress_dump_kernel<1>, dim3(n), dim3(256), 0, st, centroids, doc_offsets, codes, residuals,
                           bucket_weights, pids, out_offsets, out_vectors, out_indices, inv_norm);
}

// Storage variant "reconstructed vectors scaled to unit length" (the other reading of Section 4.5's reconstruction):
// inv_norm[t] = fl32(1 / sqrt(sum_x fl32(centroid[code_t][x] + weight[index(t, x)])^2)), the squares (exact in double)
// added in double in index order; 0 for a zero vector.  One thread per token; run once, when the variant is switched on.
template <int NBITS>
__global__ __launch_bounds__(256) void token_inv_norm_kernel(const float *__restrict__ centroids,
                                                             const int32_t *__restrict__ codes,
                                                             const uint8_t *__restrict__ residuals,
                                                             const float *__restrict__ weights, int64_t N,
                                                             float *__restrict__ inv_norm)
{
    constexpr int RB = 16 * NBITS;
    __shared__ float4 wlut[256 * (NBITS == 2 ? 1 : 2)];
    build_tables<NBITS>(wlut, nullptr, weights, threadIdx.x, 256);
    __syncthreads();
    for (int64_t tok = (int64_t)blockIdx.x * 256 + threadIdx.x; tok < N; tok += (int64_t)gridDim.x * 256) {
        const float *crow = centroids + (int64_t)codes[tok] * DIM;
        const uint8_t *r = residuals + tok * RB;
        double n2 = 0.0;
        for (int quad = 0; quad < DIM / 4; ++quad) {
            const float4 c = *reinterpret_cast<const float4 *>(crow + 4 * quad);
            const float4 w = wlut[table_slot<NBITS>(r, quad)];
            const float d0 = c.x + w.x, d1 = c.y + w.y, d2 = c.z + w.z, d3 = c.w + w.w;
            n2 = fma((double)d0, (double)d0, n2);
            n2 = fma((double)d1, (double)d1, n2);
            n2 = fma((double)d2, (double)d2, n2);
            n2 = fma((double)d3, (double)d3, n2);
        }
        inv_norm[tok] = n2 > 0.0 ? (float)(1.0 / sqrt(n2)) : 0.0f;
    }
}
void plaid_launch_token_inv_norm(hipStream_t st, const float *centroids, const int32_t *codes, const uint8_t *residuals,
                                 const float *bucket_weights, int nbits, int64_t N, float *inv_norm)
{
    if (N <= 0) return;
    int64_t g = (N + 255) / 256;
    if (g > 65536) g = 65536;
    if (nbits == 2)
        hipLaunchKernelGGL(token_inv_norm_kernel<2>, dim3((unsigned)g), dim3(256), 0, st, centroids, codes, residuals,
                           bucket_weights, N, inv_norm);
    else
        hipLaunchKernelGGL(token_inv_norm_kernel<1>, dim3((unsigned)g), dim3(256), 0, st, centroids, codes, residuals,
                           bucket_weights, N, inv_norm);
}
