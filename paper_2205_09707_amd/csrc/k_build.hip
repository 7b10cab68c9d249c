// Index construction, the step before the search path (Section 3.1 for the residual encoding, Section 4.1 for the
// passage-level inverted lists): what turns vectors and their centroid ids into the arrays a search reads.
//
//  * residual encoding: r = x - centroid per dimension (one fp32 subtraction), bucket = number of cut-offs strictly
//    below r, 8 / nbits bucket indices per byte, most significant first -- the inverse of Section 4.5's byte table.
//  * inverted lists: list c = the ascending unique ids of the passages that hold a token coded c.  Passages are
//    split into groups of consecutive ids.  Pass 1 counts, per (group, centroid), the passages of the group that
//    contain the centroid (a token counts when no earlier token of its passage has the same code).  A scan over
//    (centroid major, group minor) turns the counts into the position where each group starts writing inside each
//    list.  Pass 2 gives every group to ONE wave, which walks its passages in ascending id order and appends each
//    passage to the lists of its distinct codes: a list receives the groups' contributions at disjoint, ordered
//    positions and, inside a group, in id order -- ascending and deterministic without any sort.
//
// (Nearest-centroid assignment needs no kernel of its own: it is S_cq with 32 vectors in the place of a query's 32
// tokens, followed by the top-1 probe of every "token".)
#include "plaid_internal.h"

// ------------------------------------------------------------------ residual encoding
// One thread per 32-bit output word: 32 / NBITS dimensions of one vector.
template <int NBITS>
__global__ __launch_bounds__(256) void encode_residuals_kernel(const float *__restrict__ centroids, int64_t C,
                                                               const float *__restrict__ x,
                                                               const int32_t *__restrict__ codes, int64_t n,
                                                               const float *__restrict__ cutoffs,
                                                               uint32_t *__restrict__ out, int32_t *__restrict__ bad)
{
    constexpr int WORDS = DIM * NBITS / 32;  // per vector
    constexpr int DPW = 32 / NBITS;          // dimensions per word
    constexpr int NCUT = (1 << NBITS) - 1;
    float cut[NCUT];
#pragma unroll
    for (int q = 0; q < NCUT; ++q) cut[q] = cutoffs[q];
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < n * WORDS; e += (int64_t)gridDim.x * blockDim.x) {
        const int64_t j = e / WORDS;
        const int w = (int)(e % WORDS);
        const int32_t c = codes[j];
        if (c < 0 || c >= C) {  // reported to the host; the word is written as zero
            *bad = 1;
            out[e] = 0u;
            continue;
        }
        const float4 *xv = reinterpret_cast<const float4 *>(x + j * DIM + w * DPW);
        const float4 *cv = reinterpret_cast<const float4 *>(centroids + (int64_t)c * DIM + w * DPW);
        uint32_t word = 0u;  // byte m of the word = output byte 4 w + m (little endian), dimensions most significant first
#pragma unroll
        for (int g = 0; g < DPW / 4; ++g) {
            const float4 a = xv[g], b = cv[g];
            const float r[4] = {a.x - b.x, a.y - b.y, a.z - b.z, a.w - b.w};
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                uint32_t bk = 0u;
#pragma unroll
                for (int q = 0; q < NCUT; ++q) bk += cut[q] < r[t] ? 1u : 0u;
                const int d = 4 * g + t;                   // dimension within the word
                const int byte = d / (8 / NBITS), pos = d % (8 / NBITS);
                word |= bk << (8 * byte + 8 - NBITS * (pos + 1));
            }
        }
        out[e] = word;
    }
}

void plaid_launch_encode_residuals(hipStream_t st, const float *centroids, int64_t C, const float *x, const int32_t *codes,
                                   int64_t n, const float *cutoffs, int nbits, uint8_t *residuals, int32_t *bad)
{
    if (n <= 0) return;
    const int64_t words = n * (DIM * nbits / 32);
    int64_t blocks = (words + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    if (nbits == 2)
        hipLaunchKernelGGL(encode_residuals_kernel<2>, dim3((unsigned)blocks), dim3(256), 0, st, centroids, C, x, codes, n, cutoffs,
                           (uint32_t *)residuals, bad);
    else
        hipLaunchKernelGGL(encode_residuals_kernel<1>, dim3((unsigned)blocks), dim3(256), 0, st, centroids, C, x, codes, n, cutoffs,
                           (uint32_t *)residuals, bad);
}

// ------------------------------------------------------------------ inverted lists
// Whether token j (tokens [t0, t1) form its passage) is the first of its passage with its code.
__device__ __forceinline__ bool ivb_first_in_passage(const int32_t *__restrict__ codes, int64_t t0, int64_t j, int32_t c)
{
    for (int64_t e = t0; e < j; ++e)
        if (codes[e] == c) return false;
    return true;
}

// Passages [g * per, (g + 1) * per) form group g.  bad[0] is set when a code or an offset is out of range.
__device__ __forceinline__ bool ivb_passage(const int64_t *__restrict__ doc_offsets, int64_t p, int64_t N, int64_t &t0,
                                            int64_t &t1, int32_t *bad)
{
    t0 = doc_offsets[p];
    t1 = doc_offsets[p + 1];
    if (t0 < 0 || t1 < t0 || t1 > N) {
        *bad = 1;
        return false;
    }
    return true;
}

// Pass 1: counts[g][c] += 1 for every distinct code c of every passage of group g.  One wave per passage.
__global__ __launch_bounds__(256) void ivb_count_kernel(const int32_t *__restrict__ codes,
                                                        const int64_t *__restrict__ doc_offsets, int64_t P, int64_t N,
                                                        int64_t C, int64_t per, int32_t *__restrict__ counts,
                                                        int32_t *__restrict__ bad)
{
    const int lane = threadIdx.x & 63;
    const int64_t wave = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const int64_t nwaves = (int64_t)gridDim.x * (blockDim.x >> 6);
    for (int64_t p = wave; p < P; p += nwaves) {
        int64_t t0, t1;
        if (!ivb_passage(doc_offsets, p, N, t0, t1, bad)) continue;
        int32_t *row = counts + (p / per) * C;
        for (int64_t j = t0 + lane; j < t1; j += 64) {
            const int32_t c = codes[j];
            if (c < 0 || c >= C) {
                *bad = 1;
                continue;
            }
            if (ivb_first_in_passage(codes, t0, j, c)) atomicAdd(&row[c], 1);
        }
    }
}

// One pass over the count table: counts[g][c] <- sum of counts[g'][c] over g' < g (the 32-bit position inside list c at
// which group g starts writing), total[c] = the sum over all groups (the list's length).
__global__ __launch_bounds__(256) void ivb_totals_kernel(int32_t *__restrict__ counts, int64_t C, int64_t G,
                                                         int64_t *__restrict__ total)
{
    const int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= C) return;
    int32_t run = 0;  // (a list has at most P < 2^31 entries)
    for (int64_t g = 0; g < G; ++g) {
        const int32_t v = counts[g * C + c];
        counts[g * C + c] = run;
        run += v;
    }
    total[c] = run;
}
// One workgroup: ivf_offsets[0 .. C] = exclusive prefix sum of total[0 .. C).
__global__ __launch_bounds__(1024) void ivb_scan_kernel(const int64_t *__restrict__ total, int64_t C,
                                                        int64_t *__restrict__ ivf_offsets)
{
    __shared__ int64_t part[1024];
    const int tid = threadIdx.x;
    const int64_t per = (C + 1023) / 1024;
    const int64_t a = tid * per, b = a + per < C ? a + per : C;
    int64_t s = 0;
    for (int64_t c = a; c < b; ++c) s += total[c];
    part[tid] = s;
    __syncthreads();
    if (tid == 0) {
        int64_t run = 0;
        for (int t = 0; t < 1024; ++t) {
            const int64_t v = part[t];
            part[t] = run;
            run += v;
        }
        ivf_offsets[C] = run;
    }
    __syncthreads();
    int64_t run = part[tid];
    for (int64_t c = a; c < b; ++c) {
        ivf_offsets[c] = run;
        run += total[c];
    }
}
// Pass 2: one wave per group, passages in ascending id order.  The position comes back from the atomic before the
// passage id is stored, so the wave has finished one passage before it starts the next: every (group, centroid)
// cursor hands out its positions in passage order.
__global__ __launch_bounds__(64) void ivb_fill_kernel(const int32_t *__restrict__ codes,
                                                      const int64_t *__restrict__ doc_offsets, int64_t P, int64_t N, int64_t C,
                                                      int64_t per, int32_t *__restrict__ starts,
                                                      const int64_t *__restrict__ ivf_offsets, int32_t *__restrict__ ivf_pids,
                                                      int64_t capacity)
{
    const int lane = threadIdx.x;
    const int64_t g = blockIdx.x;
    const int64_t p0 = g * per, p1 = p0 + per < P ? p0 + per : P;
    int32_t *row = starts + g * C;
    for (int64_t p = p0; p < p1; ++p) {
        const int64_t t0 = doc_offsets[p], t1 = doc_offsets[p + 1];
        if (t0 < 0 || t1 < t0 || t1 > N) continue;  // (reported by pass 1)
        for (int64_t j = t0 + lane; j < t1; j += 64) {
            const int32_t c = codes[j];
            if (c < 0 || c >= C) continue;
            if (ivb_first_in_passage(codes, t0, j, c)) {
                const int64_t at = ivf_offsets[c] + atomicAdd(&row[c], 1);
                if (at < capacity) ivf_pids[at] = (int32_t)p;
            }
        }
    }
}

int64_t plaid_ivf_build_groups(int64_t P)
{
    int64_t G = P < 2048 ? P : 2048;
    return G < 1 ? 1 : G;
}
size_t plaid_ivf_build_scratch_bytes(int64_t P, int64_t C)
{
    return (size_t)plaid_ivf_build_groups(P) * (size_t)C * 4 + (size_t)C * 8 + 256;
}
// scratch: plaid_ivf_build_scratch_bytes(P, C) bytes, zero on entry (counts first, totals after them).
void plaid_launch_ivf_build_offsets(hipStream_t st, const int32_t *codes, const int64_t *doc_offsets, int64_t P, int64_t N,
                                    int64_t C, void *scratch, int64_t *ivf_offsets, int32_t *bad)
{
    const int64_t G = plaid_ivf_build_groups(P), per = (P + G - 1) / G;
    int32_t *counts = (int32_t *)scratch;
    int64_t *total = (int64_t *)((char *)scratch + ((size_t)G * (size_t)C * 4 + 255) / 256 * 256);
    int64_t blocks = (P + 3) / 4;
    if (blocks > 16384) blocks = 16384;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(ivb_count_kernel, dim3((unsigned)blocks), dim3(256), 0, st, codes, doc_offsets, P, N, C, per, counts, bad);
    hipLaunchKernelGGL(ivb_totals_kernel, dim3((unsigned)((C + 255) / 256)), dim3(256), 0, st, counts, C, G, total);
    hipLaunchKernelGGL(ivb_scan_kernel, dim3(1), dim3(1024), 0, st, total, C, ivf_offsets);
}
void plaid_launch_ivf_build_fill(hipStream_t st, const int32_t *codes, const int64_t *doc_offsets, int64_t P, int64_t N,
                                 int64_t C, void *scratch, const int64_t *ivf_offsets, int32_t *ivf_pids, int64_t capacity)
{
    const int64_t G = plaid_ivf_build_groups(P), per = (P + G - 1) / G;
    hipLaunchKernelGGL(ivb_fill_kernel, dim3((unsigned)G), dim3(64), 0, st, codes, doc_offsets, P, N, C, per, (int32_t *)scratch,
                       ivf_offsets, ivf_pids, capacity);
}

// ------------------------------------------------------------------ embedding-level inverted lists (vanilla ColBERTv2 retrieval)
// list c = the ascending indices of the tokens coded c (Section 4.1 describes vanilla's lists as centroid -> embedding
// ids).  Same plan as above with groups of consecutive TOKENS: counts per (group, centroid), the same scans, then one
// wave per group walks its tokens 64 at a time; a lane's position is the cursor of its code plus the number of earlier
// lanes of the chunk with the same code, so the list comes out in token order without a sort and without atomics.
__global__ __launch_bounds__(256) void evb_count_kernel(const int32_t *__restrict__ codes, int64_t N, int64_t C, int64_t per,
                                                        int32_t *__restrict__ counts, int32_t *__restrict__ bad)
{
    for (int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; j < N; j += (int64_t)gridDim.x * blockDim.x) {
        const int32_t c = codes[j];
        if (c < 0 || c >= C) {
            *bad = 1;
            continue;
        }
        atomicAdd(&counts[(j / per) * C + c], 1);
    }
}
__global__ __launch_bounds__(64) void evb_fill_kernel(const int32_t *__restrict__ codes, int64_t N, int64_t C, int64_t per,
                                                      int32_t *__restrict__ starts, const int64_t *__restrict__ offsets,
                                                      int32_t *__restrict__ eids)
{
    const int lane = threadIdx.x;
    const int64_t g = blockIdx.x;
    const int64_t j0 = g * per, j1 = j0 + per < N ? j0 + per : N;
    int32_t *row = starts + g * C;
    for (int64_t base = j0; base < j1; base += 64) {
        const int64_t j = base + lane;
        int32_t c = j < j1 ? codes[j] : -1;
        if (c >= C) c = -1;  // (reported by the counting pass)
        // earlier lanes of this chunk with my code, and whether I am the last lane with it
        int before = 0, after = 0;
        for (int l = 0; l < 64; ++l) {
            const int32_t cl = __builtin_amdgcn_readlane(c, l);
            before += (cl == c && l < lane) ? 1 : 0;
            after += (cl == c && l > lane) ? 1 : 0;
        }
        if (c >= 0) {
            const int32_t at = row[c] + before;   // the cursor of (group, c): only this wave touches it
            eids[offsets[c] + at] = (int32_t)j;
            if (after == 0) row[c] = at + 1;      // the last lane with this code moves the cursor past the chunk
        }
        // (the next chunk's reads of row[] follow this chunk's writes in program order: one wave, in-order memory)
        __threadfence_block();
    }
}
// scratch: plaid_ivf_build_scratch_bytes(N, C) bytes, zero on entry.  offsets [C+1], eids [N] (N < 2^31).
void plaid_launch_embedding_lists(hipStream_t st, const int32_t *codes, int64_t N, int64_t C, void *scratch, int64_t *offsets,
                                  int32_t *eids, int32_t *bad)
{
    const int64_t G = plaid_ivf_build_groups(N), per = (N + G - 1) / G;
    int32_t *counts = (int32_t *)scratch;
    int64_t *total = (int64_t *)((char *)scratch + ((size_t)G * (size_t)C * 4 + 255) / 256 * 256);
    int64_t blocks = (N + 255) / 256;
    if (blocks > 16384) blocks = 16384;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(evb_count_kernel, dim3((unsigned)blocks), dim3(256), 0, st, codes, N, C, per > 0 ? per : 1, counts, bad);
    hipLaunchKernelGGL(ivb_totals_kernel, dim3((unsigned)((C + 255) / 256)), dim3(256), 0, st, counts, C, G, total);
    hipLaunchKernelGGL(ivb_scan_kernel, dim3(1), dim3(1024), 0, st, total, C, offsets);
    if (N > 0)
        hipLaunchKernelGGL(evb_fill_kernel, dim3((unsigned)G), dim3(64), 0, st, codes, N, C, per, counts, offsets, eids);
}

// tok2pid[j] = the passage token j belongs to (binary search in the passage offsets; empty passages own no token).
__global__ __launch_bounds__(256) void tok2pid_kernel(const int64_t *__restrict__ doc_offsets, int64_t P, int64_t N,
                                                      int32_t *__restrict__ tok2pid)
{
    for (int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; j < N; j += (int64_t)gridDim.x * blockDim.x) {
        int64_t lo = 0, hi = P;  // largest lo with doc_offsets[lo] <= j
        while (hi - lo > 1) {
            const int64_t mid = (lo + hi) >> 1;
            if (doc_offsets[mid] <= j) lo = mid;
            else hi = mid;
        }
        tok2pid[j] = (int32_t)lo;
    }
}
void plaid_launch_tok2pid(hipStream_t st, const int64_t *doc_offsets, int64_t P, int64_t N, int32_t *tok2pid)
{
    if (N <= 0) return;
    int64_t blocks = (N + 255) / 256;
    if (blocks > 16384) blocks = 16384;
    hipLaunchKernelGGL(tok2pid_kernel, dim3((unsigned)blocks), dim3(256), 0, st, doc_offsets, P, N, tok2pid);
}
