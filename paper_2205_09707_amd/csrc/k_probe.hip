// Candidate generation, first half (Section 4.1), general form: for each query token the nprobe
// centroids with the largest S_cq entries, ranked by (score descending, centroid id ascending),
// and the ascending duplicate-free union of those ids for the inverted-list scan.
//
// Table 2's operating points (nprobe <= 8) never get here: the stage-1 kernel ranks them in
// registers.  For larger nprobe the ranking keys of each S column go through the generic selection.
#include "plaid_internal.h"

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

size_t plaid_top_nprobe_scratch_bytes(int64_t C, int nq, int nprobe)
{
    if (nprobe <= PLAID_PROBE_FAST_MAX) return 256;
    const int nseg = nq * QLEN;
    const int64_t words = (C + 31) / 32;
    return a256((size_t)nseg * C * 8) + a256((size_t)nseg * 4) + a256((size_t)nseg * nprobe * 8) + a256((size_t)nseg * 4) +
           a256((size_t)nq * words * 4) + plaid_select_scratch_bytes(nseg, C, nprobe);
}

void plaid_launch_top_nprobe_general(hipStream_t st, const float *S, int64_t C, int nq, int nprobe, int32_t *probed,
                                     int32_t *uniq, int uniq_stride, int32_t *n_uniq, void *scratch, size_t scratch_bytes)
{
    (void)scratch_bytes;
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
