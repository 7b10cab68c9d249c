// Candidate generation, first half (Section 4.1): for each query token the nprobe centroids with the
// largest S_cq entries, ranked by (score descending, centroid id ascending), and the ascending
// duplicate-free union of those ids for the inverted-list scan.
//
// nprobe <= 8 (every operating point of Table 2): S is streamed once, coalesced; each thread keeps
// a register-resident sorted list for one (token, row phase), lists are merged through LDS per
// workgroup and then per query.  Larger nprobe: ranking keys of each S column go through the
// generic selection.
#include "plaid_internal.h"

#define PROBE_MAX_FAST 8
#define PROBE_THREADS 256

template <int NP>
__device__ __forceinline__ void insert_key(uint64_t (&best)[NP], uint64_t key)
{
    if (key < best[NP - 1]) {
#pragma unroll
        for (int j = NP - 1; j >= 0; --j) {
            if (key < best[j]) {
                if (j + 1 < NP) best[j + 1] = best[j];
                best[j] = key;
            }
        }
    }
}

// partial[q][b][i][NP]: the NP best keys of token i among the rows of block b
template <int NP>
__global__ __launch_bounds__(PROBE_THREADS) void probe_partial_kernel(const float *__restrict__ S, int64_t C,
                                                                      int rows_per_block, uint64_t *__restrict__ partial)
{
    __shared__ uint64_t lk[8][QLEN][NP];
    const int q = blockIdx.y, b = blockIdx.x;
    const int i = threadIdx.x & 31, g = threadIdx.x >> 5;
    const float *Sq = S + (int64_t)q * C * QLEN;
    const int64_t r0 = (int64_t)b * rows_per_block;
    int64_t r1 = r0 + rows_per_block;
    if (r1 > C) r1 = C;
    uint64_t best[NP];
#pragma unroll
    for (int j = 0; j < NP; ++j) best[j] = PLAID_KEY_MAX;
    int64_t c = r0 + g;
    for (; c + 24 < r1; c += 32) {  // four independent loads in flight
        const float v0 = Sq[c * QLEN + i], v1 = Sq[(c + 8) * QLEN + i], v2 = Sq[(c + 16) * QLEN + i],
                    v3 = Sq[(c + 24) * QLEN + i];
        insert_key<NP>(best, plaid_make_key(v0, (uint32_t)c));
        insert_key<NP>(best, plaid_make_key(v1, (uint32_t)(c + 8)));
        insert_key<NP>(best, plaid_make_key(v2, (uint32_t)(c + 16)));
        insert_key<NP>(best, plaid_make_key(v3, (uint32_t)(c + 24)));
    }
    for (; c < r1; c += 8) insert_key<NP>(best, plaid_make_key(Sq[c * QLEN + i], (uint32_t)c));
#pragma unroll
    for (int j = 0; j < NP; ++j) lk[g][i][j] = best[j];
    __syncthreads();
    if (g == 0) {
        for (int gg = 1; gg < 8; ++gg)
#pragma unroll
            for (int j = 0; j < NP; ++j) insert_key<NP>(best, lk[gg][i][j]);
        uint64_t *o = partial + (((int64_t)q * gridDim.x + b) * QLEN + i) * NP;
#pragma unroll
        for (int j = 0; j < NP; ++j) o[j] = best[j];
    }
}

// One workgroup per query: merge the per-block lists, emit probed[q][i][0..nprobe) in rank order and
// the ascending unique union uniq[q][0..n_uniq[q]).
template <int NP>
__global__ __launch_bounds__(1024) void probe_merge_kernel(const uint64_t *__restrict__ partial, int nblocks, int nprobe,
                                                           int32_t *__restrict__ probed, int32_t *__restrict__ uniq,
                                                           int uniq_stride, int32_t *__restrict__ n_uniq)
{
    __shared__ uint64_t lk[QLEN][32][NP];
    __shared__ int32_t ids[QLEN * PROBE_MAX_FAST];
    const int q = blockIdx.x;
    const int i = threadIdx.x >> 5, l = threadIdx.x & 31;
    uint64_t best[NP];
#pragma unroll
    for (int j = 0; j < NP; ++j) best[j] = PLAID_KEY_MAX;
    const uint64_t *pq = partial + (int64_t)q * nblocks * QLEN * NP;
    for (int b = l; b < nblocks; b += 32) {
        const uint64_t *src = pq + ((int64_t)b * QLEN + i) * NP;
#pragma unroll
        for (int j = 0; j < NP; ++j) insert_key<NP>(best, src[j]);
    }
#pragma unroll
    for (int j = 0; j < NP; ++j) lk[i][l][j] = best[j];
    __syncthreads();
    if (l == 0) {
        for (int ll = 1; ll < 32; ++ll)
#pragma unroll
            for (int j = 0; j < NP; ++j) insert_key<NP>(best, lk[i][ll][j]);
#pragma unroll
        for (int j = 0; j < NP; ++j)
            if (j < nprobe) {
                const int32_t id = (int32_t)(best[j] & 0xFFFFFFFFu);
                probed[((int64_t)q * QLEN + i) * nprobe + j] = id;
                ids[i * nprobe + j] = id;
            }
    }
    __syncthreads();
    // sort the 32*nprobe (<= 256) ids and drop duplicates
    const int n = QLEN * nprobe;
    int n2 = 1;
    while (n2 < n) n2 <<= 1;
    for (int t = n + threadIdx.x; t < n2; t += blockDim.x) ids[t] = 0x7FFFFFFF;
    __syncthreads();
    for (int k = 2; k <= n2; k <<= 1)
        for (int j = k >> 1; j > 0; j >>= 1) {
            const int t = threadIdx.x;
            if (t < n2) {
                const int p = t ^ j;
                if (p > t) {
                    const int32_t a = ids[t], b = ids[p];
                    if ((a > b) == ((t & k) == 0)) {
                        ids[t] = b;
                        ids[p] = a;
                    }
                }
            }
            __syncthreads();
        }
    if (threadIdx.x == 0) {
        int cnt = 0;
        for (int t = 0; t < n; ++t)
            if (t == 0 || ids[t] != ids[t - 1]) uniq[(int64_t)q * uniq_stride + cnt++] = ids[t];
        n_uniq[q] = cnt;
    }
}

// ------------------------------------------------------------------ general path (nprobe > 8)
__global__ void probe_keys_kernel(const float *__restrict__ S, int64_t C, uint64_t *__restrict__ keys,
                                  int32_t *__restrict__ counts)
{
    const int q = blockIdx.y;
    const float *Sq = S + (int64_t)q * C * QLEN;
    uint64_t *kq = keys + (int64_t)q * QLEN * C;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < C * QLEN; e += (int64_t)gridDim.x * blockDim.x) {
        const int64_t c = e >> 5;
        const int i = (int)(e & 31);
        kq[(int64_t)i * C + c] = plaid_make_key(Sq[e], (uint32_t)c);
    }
    if (blockIdx.x == 0 && threadIdx.x < QLEN) counts[q * QLEN + threadIdx.x] = (int32_t)C;
}

__global__ void probe_general_finalize_kernel(const uint64_t *__restrict__ sel, int nprobe, int32_t *__restrict__ probed,
                                              uint32_t *__restrict__ bits, int64_t words)
{
    const int q = blockIdx.y;
    const int64_t n = (int64_t)QLEN * nprobe;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < n; e += (int64_t)gridDim.x * blockDim.x) {
        const uint32_t id = (uint32_t)(sel[(int64_t)q * n + e] & 0xFFFFFFFFu);
        probed[(int64_t)q * n + e] = (int32_t)id;
        atomicOr(&bits[(int64_t)q * words + (id >> 5)], 1u << (id & 31));
    }
}

static inline size_t a256(size_t x) { return (x + 255) & ~(size_t)255; }
static int probe_blocks(int64_t C)
{
    int64_t b = C / 512;
    if (b < 1) b = 1;
    if (b > 128) b = 128;
    return (int)b;
}

size_t plaid_top_nprobe_scratch_bytes(int64_t C, int nq, int nprobe)
{
    if (nprobe <= PROBE_MAX_FAST) return a256((size_t)nq * probe_blocks(C) * QLEN * PROBE_MAX_FAST * 8);
    const int nseg = nq * QLEN;
    const int64_t words = (C + 31) / 32;
    return a256((size_t)nseg * C * 8) + a256((size_t)nseg * 4) + a256((size_t)nseg * nprobe * 8) + a256((size_t)nseg * 4) +
           a256((size_t)nq * words * 4) + plaid_select_scratch_bytes(nseg, C, nprobe);
}

template <int NP>
static void launch_fast(hipStream_t st, const float *S, int64_t C, int nq, int nprobe, int32_t *probed, int32_t *uniq,
                        int uniq_stride, int32_t *n_uniq, uint64_t *partial)
{
    const int nb = probe_blocks(C);
    int rows = (int)((C + nb - 1) / nb);
    rows = (rows + 7) & ~7;
    hipLaunchKernelGGL(probe_partial_kernel<NP>, dim3(nb, nq), dim3(PROBE_THREADS), 0, st, S, C, rows, partial);
    hipLaunchKernelGGL(probe_merge_kernel<NP>, dim3(nq), dim3(1024), 0, st, partial, nb, nprobe, probed, uniq,
                       uniq_stride, n_uniq);
}

void plaid_launch_top_nprobe(hipStream_t st, const float *S, int64_t C, int nq, int nprobe, int32_t *probed,
                             int32_t *uniq, int uniq_stride, int32_t *n_uniq, void *scratch, size_t scratch_bytes)
{
    (void)scratch_bytes;
    if (nprobe <= PROBE_MAX_FAST) {
        uint64_t *partial = (uint64_t *)scratch;
        if (nprobe == 1) launch_fast<1>(st, S, C, nq, nprobe, probed, uniq, uniq_stride, n_uniq, partial);
        else if (nprobe == 2) launch_fast<2>(st, S, C, nq, nprobe, probed, uniq, uniq_stride, n_uniq, partial);
        else if (nprobe <= 4) launch_fast<4>(st, S, C, nq, nprobe, probed, uniq, uniq_stride, n_uniq, partial);
        else launch_fast<8>(st, S, C, nq, nprobe, probed, uniq, uniq_stride, n_uniq, partial);
        return;
    }
    // general: rank every column of S with the generic selection
    const int nseg = nq * QLEN;
    const int64_t words = (C + 31) / 32;
    char *p = (char *)scratch;
    uint64_t *keys = (uint64_t *)p;
    p += a256((size_t)nseg * C * 8);
    int32_t *counts = (int32_t *)p;
    p += a256((size_t)nseg * 4);
    uint64_t *sel = (uint64_t *)p;
    p += a256((size_t)nseg * nprobe * 8);
    int32_t *sel_counts = (int32_t *)p;
    p += a256((size_t)nseg * 4);
    uint32_t *bits = (uint32_t *)p;
    p += a256((size_t)nq * words * 4);
    SelScratch sc = plaid_select_scratch_carve(p, nseg, C, nprobe);
    plaid_launch_fill_u32(st, (uint32_t *)sc.state, (int64_t)(plaid_select_zero_bytes(nseg) / 4), 0u);
    plaid_launch_fill_u32(st, bits, (int64_t)nq * words, 0u);
    int gx = (int)((C * QLEN + 255) / 256);
    if (gx > 2048) gx = 2048;
    hipLaunchKernelGGL(probe_keys_kernel, dim3(gx, nq), dim3(256), 0, st, S, C, keys, counts);
    plaid_launch_select(st, keys, C, counts, nseg, C, nprobe, sel, nprobe, sel_counts, 1, sc, 0);
    int gf = (int)(((int64_t)QLEN * nprobe + 255) / 256);
    if (gf > 256) gf = 256;
    hipLaunchKernelGGL(probe_general_finalize_kernel, dim3(gf, nq), dim3(256), 0, st, sel, nprobe, probed, bits, words);
    plaid_launch_bitmap_to_list(st, bits, words, C, nq, uniq, uniq_stride, n_uniq);
}
