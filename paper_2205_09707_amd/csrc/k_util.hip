// Small helper kernels: fills, key -> (id, score) conversion, bitmap -> ascending id list.
#include "plaid_internal.h"

#include <math.h>

__global__ void fill_u32_kernel(uint32_t *__restrict__ p, int64_t n, uint32_t v)
{
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = v;
}
void plaid_launch_fill_u32(hipStream_t st, uint32_t *p, int64_t n, uint32_t v)
{
    if (n <= 0) return;
    int64_t g = (n + 255) / 256;
    if (g > 4096) g = 4096;
    hipLaunchKernelGGL(fill_u32_kernel, dim3((int)g), dim3(256), 0, st, p, n, v);
}

// Final ranking -> caller buffers: ids[q][j], scores[q][j] for j < counts[q] (capped at k), (-1, -inf) beyond.
__global__ void keys_to_output_kernel(const uint64_t *__restrict__ keys, int64_t key_stride,
                                      const int32_t *__restrict__ counts, int32_t k, int32_t *__restrict__ out_ids,
                                      float *__restrict__ out_scores)
{
    const int q = blockIdx.y;
    const int n = counts[q] < k ? counts[q] : k;
    for (int j = blockIdx.x * blockDim.x + threadIdx.x; j < k; j += gridDim.x * blockDim.x) {
        int32_t id = -1;
        float sc = -INFINITY;
        if (j < n) {
            const uint64_t key = keys[(int64_t)q * key_stride + j];
            id = (int32_t)(key & 0xFFFFFFFFu);
            sc = plaid_ord_to_score((uint32_t)(key >> 32));
        }
        out_ids[(int64_t)q * k + j] = id;
        out_scores[(int64_t)q * k + j] = sc;
    }
}
void plaid_launch_keys_to_output(hipStream_t st, const uint64_t *keys, int64_t key_stride, const int32_t *counts, int nq,
                                 int32_t k, int32_t *out_ids, float *out_scores)
{
    int g = (k + 255) / 256;
    if (g > 64) g = 64;
    hipLaunchKernelGGL(keys_to_output_kernel, dim3(g, nq), dim3(256), 0, st, keys, key_stride, counts, k, out_ids,
                       out_scores);
}

// Debug dump of a key list as (id, score) pairs; any output pointer may be null.
__global__ void keys_to_pairs_kernel(const uint64_t *__restrict__ keys, int64_t key_stride,
                                     const int32_t *__restrict__ counts, int32_t cap, int32_t *__restrict__ out_ids,
                                     float *__restrict__ out_scores, int32_t *__restrict__ out_counts)
{
    const int q = blockIdx.y;
    const int n = counts[q] < cap ? counts[q] : cap;
    for (int j = blockIdx.x * blockDim.x + threadIdx.x; j < n; j += gridDim.x * blockDim.x) {
        const uint64_t key = keys[(int64_t)q * key_stride + j];
        if (out_ids) out_ids[(int64_t)q * cap + j] = (int32_t)(key & 0xFFFFFFFFu);
        if (out_scores) out_scores[(int64_t)q * cap + j] = plaid_ord_to_score((uint32_t)(key >> 32));
    }
    if (out_counts && blockIdx.x == 0 && threadIdx.x == 0) out_counts[q] = n;
}
void plaid_launch_keys_to_pairs(hipStream_t st, const uint64_t *keys, int64_t key_stride, const int32_t *counts, int nq,
                                int32_t cap, int32_t *out_ids, float *out_scores, int32_t *out_counts)
{
    int g = (cap + 255) / 256;
    if (g > 64) g = 64;
    if (g < 1) g = 1;
    hipLaunchKernelGGL(keys_to_pairs_kernel, dim3(g, nq), dim3(256), 0, st, keys, key_stride, counts, cap, out_ids,
                       out_scores, out_counts);
}

// Ascending list of the set bits of bits[q][0..words): one workgroup per query, chunked prefix sums.
__global__ __launch_bounds__(1024) void bitmap_to_list_kernel(const uint32_t *__restrict__ bits, int64_t words,
                                                              int64_t nvalid, int32_t *__restrict__ out,
                                                              int64_t out_stride, int32_t *__restrict__ out_counts)
{
    __shared__ int32_t scan[1024];
    __shared__ int32_t base_s;
    const int q = blockIdx.x;
    const uint32_t *b = bits + (int64_t)q * words;
    int32_t *o = out ? out + (int64_t)q * out_stride : nullptr;
    if (threadIdx.x == 0) base_s = 0;
    __syncthreads();
    for (int64_t w0 = 0; w0 < words; w0 += 1024) {
        const int64_t w = w0 + threadIdx.x;
        uint32_t v = w < words ? b[w] : 0u;
        if (w < words && (w + 1) * 32 > nvalid) {  // mask bits beyond the valid range
            const int64_t keep = nvalid - w * 32;
            v = keep <= 0 ? 0u : (keep >= 32 ? v : (v & ((1u << keep) - 1u)));
        }
        const int cnt = __popc(v);
        scan[threadIdx.x] = cnt;
        __syncthreads();
        for (int d = 1; d < 1024; d <<= 1) {
            const int t = threadIdx.x >= d ? scan[threadIdx.x - d] : 0;
            __syncthreads();
            scan[threadIdx.x] += t;
            __syncthreads();
        }
        int pos = base_s + scan[threadIdx.x] - cnt;
        if (o)
            while (v) {
                const int bit = __ffs(v) - 1;
                v &= v - 1;
                o[pos++] = (int32_t)(w * 32 + bit);
            }
        __syncthreads();
        if (threadIdx.x == 1023) base_s += scan[1023];
        __syncthreads();
    }
    if (threadIdx.x == 0 && out_counts) out_counts[q] = base_s;
}
void plaid_launch_bitmap_to_list(hipStream_t st, const uint32_t *bits, int64_t words, int64_t nbits_valid, int nq,
                                 int32_t *out, int64_t out_stride, int32_t *out_counts)
{
    hipLaunchKernelGGL(bitmap_to_list_kernel, dim3(nq), dim3(1024), 0, st, bits, words, nbits_valid, out, out_stride,
                       out_counts);
}

// ------------------------------------------------------------------ structural validation of a device-resident index
// The search kernels index memory with the index's own offsets, codes and passage ids, so an index whose arrays arrive
// in device memory is checked once, when the handle is made: doc_offsets from 0 to N without a decrease, codes in
// [0, C), ivf_offsets from 0 to ivf_len without a decrease, passage ids in [0, P) and strictly ascending inside each
// list.  bad[0] receives the OR of: 1 doc_offsets, 2 codes, 4 ivf_offsets, 8 passage id out of range, 16 list not
// strictly ascending.  Grid-stride loops over each array; the list test looks up the list of entry e by binary search
// in ivf_offsets only when e follows a larger-or-equal id (a list boundary or an error), so it costs one pass over
// the ids.
__global__ __launch_bounds__(256) void index_validate_kernel(const int64_t *__restrict__ doc_offsets, int64_t P, int64_t N,
                                                             const int32_t *__restrict__ codes, int64_t C,
                                                             const int64_t *__restrict__ ivf_offsets,
                                                             const int32_t *__restrict__ ivf_pids, int64_t ivf_len,
                                                             int32_t *__restrict__ bad)
{
    const int64_t t0 = (int64_t)blockIdx.x * blockDim.x + threadIdx.x, step = (int64_t)gridDim.x * blockDim.x;
    int flags = 0;
    for (int64_t p = t0; p <= P; p += step) {
        const int64_t o = doc_offsets[p];
        if (o < 0 || o > N || (p == 0 && o != 0) || (p == P && o != N)) flags |= 1;
        if (p < P && doc_offsets[p + 1] < o) flags |= 1;
    }
    for (int64_t j = t0; j < N; j += step) {
        const int32_t c = codes[j];
        if (c < 0 || c >= C) flags |= 2;
    }
    for (int64_t c = t0; c <= C; c += step) {
        const int64_t o = ivf_offsets[c];
        if (o < 0 || o > ivf_len || (c == 0 && o != 0) || (c == C && o != ivf_len)) flags |= 4;
        if (c < C && ivf_offsets[c + 1] < o) flags |= 4;
    }
    for (int64_t e = t0; e < ivf_len; e += step) {
        const int32_t pid = ivf_pids[e];
        if (pid < 0 || pid >= P) flags |= 8;
        if (e > 0 && ivf_pids[e - 1] >= pid) {
            // allowed only when e is the first entry of a list: some offset equals e
            int64_t lo = 0, hi = C;  // largest lo with ivf_offsets[lo] <= e (offsets validated by other threads: a
            while (lo < hi) {        // malformed table can only produce a wrong verdict here, and sets flag 4 there)
                const int64_t mid = (lo + hi + 1) >> 1;
                if (ivf_offsets[mid] <= e) lo = mid;
                else hi = mid - 1;
            }
            if (ivf_offsets[lo] != e) flags |= 16;
        }
    }
    if (flags) atomicOr(bad, flags);
}
void plaid_launch_index_validate(hipStream_t st, const int64_t *doc_offsets, int64_t P, int64_t N, const int32_t *codes,
                                 int64_t C, const int64_t *ivf_offsets, const int32_t *ivf_pids, int64_t ivf_len, int32_t *bad)
{
    int64_t work = N > ivf_len ? N : ivf_len;
    if (work < P + 1) work = P + 1;
    if (work < C + 1) work = C + 1;
    int64_t g = (work + 255) / 256;
    if (g > 8192) g = 8192;
    if (g < 1) g = 1;
    hipLaunchKernelGGL(index_validate_kernel, dim3((unsigned)g), dim3(256), 0, st, doc_offsets, P, N, codes, C, ivf_offsets,
                       ivf_pids, ivf_len, bad);
}
