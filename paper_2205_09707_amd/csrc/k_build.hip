// Index construction, the step before the search path (Section 3.1 for the residual encoding, Section 4.1 for the
// passage-level inverted lists): what turns vectors and their centroid ids into the arrays a search reads.
//
//  * residual encoding: r = x - centroid per dimension (one fp32 subtraction), bucket = number of cut-offs strictly
//    below r, 8 / nbits bucket indices per byte, most significant first -- the inverse of Section 4.5's byte table.
//  * inverted lists: list c = the ascending unique ids of the passages that hold a token coded c.  A token counts when
//    no earlier token of its passage has the same code.  Pass 1 gives every such token its arrival rank among the
//    tokens of its (stripe, centroid) -- passages are dealt round-robin to up to 64 stripes, each with its own table of
//    C counters, because centroid popularity is heavily skewed (the most popular centroid occurs in nearly every
//    passage) and atomics on one address are served one after the other.  The counters end as lengths; a prefix over
//    the stripes and a scan over the centroids turn them into offsets; pass 2 stores the passage of every ranked token
//    at offset + stripe start + rank in a staging buffer: the lists are complete but in arrival order.  Pass 3 sorts
//    each list on its way to the output -- a wave per list with a bitonic network in LDS, or, for the long lists, a
//    workgroup that marks the list's passages in an LDS bitmap of 2^20 passage ids at a time and reads the marks back in
//    order.  The ids of a list are distinct, so the sorted list is the one list there is: deterministic whatever
//    order the atomics were served in.
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
#define IVB_SHORT_MAX 2048                 // longest list a single wave sorts in LDS
#define IVB_RANGE_SHIFT 20                 // the bitmap of the long-list kernel covers 2^20 passage ids
#define IVB_RANGE_WORDS (1 << (IVB_RANGE_SHIFT - 5))

// Tokens [t0, t1) of passage p.  bad[0] is set when the offsets are not monotone within [0, N].
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

// A wave holds tokens base .. base + 63 of a passage that starts at t0, c = the code of the lane's token (-1: none).
// Whether an earlier token of the passage has the same code.
__device__ __forceinline__ bool ivb_seen_before(const int32_t *__restrict__ codes, int64_t t0, int64_t base, int lane, int32_t c)
{
    int dup = 0;
    for (int64_t e0 = t0; e0 < base; e0 += 64) {  // the (whole) chunks before this one
        const int32_t prev = codes[e0 + lane];
#pragma unroll 8
        for (int l = 0; l < 64; ++l) dup |= (__builtin_amdgcn_readlane(prev, l) == c) ? 1 : 0;
    }
#pragma unroll 8
    for (int l = 0; l < 64; ++l) dup |= (__builtin_amdgcn_readlane(c, l) == c && l < lane) ? 1 : 0;
    return dup != 0;
}

// Pass 1, one wave per passage, 64 tokens at a time; passage p belongs to stripe p % stripes (a power of two).
// rank[j] = how many tokens were counted into counts[stripe][codes[j]] before token j, or -1 for a token whose code an
// earlier token of the passage already has (or whose code is out of range: bad[0] is set).  counts[s][c] ends as the
// number of passages of stripe s in list c.
__global__ __launch_bounds__(256) void ivb_rank_kernel(const int32_t *__restrict__ codes, const int64_t *__restrict__ doc_offsets,
                                                       int64_t P, int64_t N, int64_t C, int stripes, int32_t *__restrict__ counts,
                                                       int32_t *__restrict__ rank, int32_t *__restrict__ bad)
{
    const int lane = threadIdx.x & 63;
    const int64_t wave = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const int64_t nwaves = (int64_t)gridDim.x * (blockDim.x >> 6);
    for (int64_t p = wave; p < P; p += nwaves) {
        int64_t t0, t1;
        if (!ivb_passage(doc_offsets, p, N, t0, t1, bad)) continue;
        int32_t *row = counts + (p & (stripes - 1)) * C;
        for (int64_t base = t0; base < t1; base += 64) {
            const int64_t j = base + lane;
            int32_t c = j < t1 ? codes[j] : -1;
            if (j < t1 && (c < 0 || c >= C)) {
                *bad = 1;
                c = -1;
            }
            const bool dup = ivb_seen_before(codes, t0, base, lane, c);
            if (j < t1) rank[j] = (c < 0 || dup) ? -1 : atomicAdd(&row[c], 1);
        }
    }
}

// counts[s][c] <- the sum over the stripes before s (where stripe s starts inside list c), total[c] = the list's length.
__global__ __launch_bounds__(256) void ivb_stripe_totals_kernel(int32_t *__restrict__ counts, int64_t C, int stripes,
                                                                int32_t *__restrict__ total)
{
    const int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= C) return;
    int32_t run = 0;  // (a list has at most P < 2^31 entries)
    for (int s = 0; s < stripes; ++s) {
        const int32_t v = counts[s * C + c];
        counts[s * C + c] = run;
        run += v;
    }
    total[c] = run;
}

// One workgroup: ivf_offsets[0 .. C] = exclusive prefix sum of total[0 .. C); the lists longer than IVB_SHORT_MAX are
// appended to long_lists (n_long counts them, zero on entry).
__global__ __launch_bounds__(1024) void ivb_offsets_kernel(const int32_t *__restrict__ total, int64_t C,
                                                           int64_t *__restrict__ ivf_offsets, int32_t *__restrict__ long_lists,
                                                           int32_t *__restrict__ n_long)
{
    __shared__ long long wave_sum[16];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    long long carry = 0;
    for (int64_t base = 0; base < C; base += 4096) {  // four consecutive lists per thread and round
        const int64_t c0 = base + 4 * tid;
        int32_t v[4];
        long long mine = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            v[e] = c0 + e < C ? total[c0 + e] : 0;
            if (v[e] > IVB_SHORT_MAX) long_lists[atomicAdd(n_long, 1)] = (int32_t)(c0 + e);
            mine += v[e];
        }
        long long incl = mine;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const long long up = __shfl_up(incl, d);
            if (lane >= d) incl += up;
        }
        if (lane == 63) wave_sum[w] = incl;
        __syncthreads();
        long long before = 0, all = 0;
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            const long long x = wave_sum[k];
            before += k < w ? x : 0;
            all += x;
        }
        long long at = carry + before + incl - mine;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (c0 + e < C) ivf_offsets[c0 + e] = at;
            at += v[e];
        }
        carry += all;
        __syncthreads();
    }
    if (tid == 0) ivf_offsets[C] = carry;
}

// Pass 2, one wave per passage: the passage id of every ranked token goes to its list's staging area, at the start of
// its stripe plus its rank.
__global__ __launch_bounds__(256) void ivb_scatter_kernel(const int32_t *__restrict__ codes, const int64_t *__restrict__ doc_offsets,
                                                          int64_t P, int64_t N, int64_t C, int stripes,
                                                          const int32_t *__restrict__ stripe_start,
                                                          const int64_t *__restrict__ ivf_offsets, const int32_t *__restrict__ rank,
                                                          int32_t *__restrict__ staged, int64_t capacity)
{
    const int lane = threadIdx.x & 63;
    const int64_t wave = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const int64_t nwaves = (int64_t)gridDim.x * (blockDim.x >> 6);
    for (int64_t p = wave; p < P; p += nwaves) {
        const int64_t t0 = doc_offsets[p], t1 = doc_offsets[p + 1];
        if (t0 < 0 || t1 < t0 || t1 > N) continue;  // (reported by pass 1)
        const int32_t *row = stripe_start + (p & (stripes - 1)) * C;
        for (int64_t j = t0 + lane; j < t1; j += 64) {
            const int32_t r = rank[j];
            if (r < 0) continue;
            const int32_t c = codes[j];  // (a ranked token's code is in range)
            const int64_t at = ivf_offsets[c] + row[c] + r;
            if (at < capacity) staged[at] = (int32_t)p;
        }
    }
}

// Pass 3 for lists of at most IVB_SHORT_MAX entries: one wave per list, bitonic network in the wave's LDS area.
__global__ __launch_bounds__(256) void ivb_sort_short_kernel(const int64_t *__restrict__ ivf_offsets, int64_t C,
                                                             const int32_t *__restrict__ staged, int32_t *__restrict__ ivf_pids)
{
    __shared__ int32_t area[4][IVB_SHORT_MAX];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    int32_t *buf = area[w];
    for (int64_t c = (int64_t)blockIdx.x * 4 + w; c < C; c += (int64_t)gridDim.x * 4) {
        const int64_t off = ivf_offsets[c];
        const int64_t len = ivf_offsets[c + 1] - off;
        if (len <= 0 || len > IVB_SHORT_MAX) continue;
        const int L = (int)len;
        if (L == 1) {
            if (lane == 0) ivf_pids[off] = staged[off];
            continue;
        }
        int n = 2;
        while (n < L) n <<= 1;
        for (int i = lane; i < n; i += 64) buf[i] = i < L ? staged[off + i] : 0x7FFFFFFF;
        for (int k = 2; k <= n; k <<= 1)
            for (int j = k >> 1; j > 0; j >>= 1) {
                // (one wave: its LDS accesses are served in order; the fences keep the compiler from moving them)
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                for (int i = lane; i < (n >> 1); i += 64) {
                    const int a = ((i & ~(j - 1)) << 1) | (i & (j - 1)), b = a | j;
                    const int32_t x = buf[a], y = buf[b];
                    const bool up = (a & k) == 0;
                    if ((x > y) == up) {
                        buf[a] = y;
                        buf[b] = x;
                    }
                }
            }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        for (int i = lane; i < L; i += 64) ivf_pids[off + i] = buf[i];
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");  // the next list's loads into buf come after these reads
        __builtin_amdgcn_wave_barrier();
    }
}

// Pass 3 for the long lists: one workgroup per list.  For each range of 2^20 passage ids in turn: mark the list's ids of
// the range in an LDS bitmap, then read the marks back in ascending order (a thread owns a stretch of consecutive words,
// counts them, a scan over the workgroup gives its first output position).
__global__ __launch_bounds__(1024) void ivb_sort_long_kernel(const int64_t *__restrict__ ivf_offsets, const int32_t *__restrict__ long_lists,
                                                             const int32_t *__restrict__ n_long, int64_t P,
                                                             const int32_t *__restrict__ staged, int32_t *__restrict__ ivf_pids)
{
    __shared__ uint32_t marks[IVB_RANGE_WORDS];
    __shared__ int32_t wave_sum[16];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int nl = *n_long;
    for (int li = blockIdx.x; li < nl; li += gridDim.x) {
        const int64_t c = long_lists[li];
        const int64_t off = ivf_offsets[c], len = ivf_offsets[c + 1] - off;
        int64_t out = off;
        for (int64_t r = 0; (r << IVB_RANGE_SHIFT) < P; ++r) {
            // words of this range that can hold a mark, and how many of them a thread owns (consecutive ones)
            const int64_t left = P - (r << IVB_RANGE_SHIFT);
            const int words = left >= (1 << IVB_RANGE_SHIFT) ? IVB_RANGE_WORDS : (int)((left + 31) >> 5);
            const int each = ((words + 1023) >> 10) | 1;  // odd: the lanes of a wave then read distinct LDS banks
            for (int i = tid; i < words; i += 1024) marks[i] = 0u;
            __syncthreads();
            for (int64_t i = tid; i < len; i += 1024) {
                const int32_t p = staged[off + i];
                if ((int64_t)(p >> IVB_RANGE_SHIFT) == r)
                    atomicOr(&marks[(p & ((1 << IVB_RANGE_SHIFT) - 1)) >> 5], 1u << (p & 31));
            }
            __syncthreads();
            const int w0 = tid * each, w1 = w0 + each < words ? w0 + each : words;
            int cnt = 0;
            for (int i = w0; i < w1; ++i) cnt += __popc(marks[i]);
            int incl = cnt;
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                const int up = __shfl_up(incl, d);
                if (lane >= d) incl += up;
            }
            if (lane == 63) wave_sum[w] = incl;
            __syncthreads();
            int before = 0, all = 0;
#pragma unroll
            for (int k = 0; k < 16; ++k) {
                const int x = wave_sum[k];
                before += k < w ? x : 0;
                all += x;
            }
            if (cnt > 0) {
                int64_t at = out + before + incl - cnt;
                for (int i = w0; i < w1; ++i) {
                    uint32_t m = marks[i];
                    const int32_t first = (int32_t)((r << IVB_RANGE_SHIFT) + 32 * i);
                    while (m) {
                        ivf_pids[at++] = first + __builtin_ctz(m);
                        m &= m - 1;
                    }
                }
            }
            out += all;
            __syncthreads();  // marks and wave_sum are rewritten by the next range
        }
    }
}

// Scratch of the passage-level lists: n_long and counts [stripes][C] (the part that must be zero on entry), total [C],
// long_lists [C], rank [N], staged [N].
struct IvbScratch {
    int stripes;
    int32_t *n_long, *counts, *total, *long_lists, *rank, *staged;
    size_t zero_bytes, bytes;
};
static IvbScratch ivb_carve(void *scratch, int64_t N, int64_t C)
{
    auto a256 = [](size_t x) { return (x + 255) / 256 * 256; };
    IvbScratch x = {};
    x.stripes = 64;  // as many as keep the counter tables within 256 MiB
    while (x.stripes > 1 && (int64_t)x.stripes * C > (1ll << 26)) x.stripes >>= 1;
    const size_t n = (size_t)(N > 0 ? N : 1);
    char *p = (char *)scratch;
    x.n_long = (int32_t *)p;
    p += 256;
    x.counts = (int32_t *)p;
    p += a256((size_t)x.stripes * (size_t)C * 4);
    x.zero_bytes = (size_t)(p - (char *)scratch);
    x.total = (int32_t *)p;
    p += a256((size_t)C * 4);
    x.long_lists = (int32_t *)p;
    p += a256((size_t)C * 4);
    x.rank = (int32_t *)p;
    p += a256(n * 4);
    x.staged = (int32_t *)p;
    p += a256(n * 4);
    x.bytes = (size_t)(p - (char *)scratch);
    return x;
}
size_t plaid_ivf_lists_scratch_bytes(int64_t N, int64_t C) { return ivb_carve(nullptr, N, C).bytes; }
size_t plaid_ivf_lists_scratch_zero_bytes(int64_t N, int64_t C) { return ivb_carve(nullptr, N, C).zero_bytes; }

static unsigned ivb_passage_blocks(int64_t P)
{
    int64_t blocks = (P + 3) / 4;
    if (blocks > 16384) blocks = 16384;
    return (unsigned)(blocks < 1 ? 1 : blocks);
}
// scratch: plaid_ivf_lists_scratch_bytes(N, C) bytes, the first plaid_ivf_lists_scratch_zero_bytes(N, C) of them zero.
void plaid_launch_ivf_build_offsets(hipStream_t st, const int32_t *codes, const int64_t *doc_offsets, int64_t P, int64_t N,
                                    int64_t C, void *scratch, int64_t *ivf_offsets, int32_t *bad)
{
    const IvbScratch x = ivb_carve(scratch, N, C);
    hipLaunchKernelGGL(ivb_rank_kernel, dim3(ivb_passage_blocks(P)), dim3(256), 0, st, codes, doc_offsets, P, N, C, x.stripes,
                       x.counts, x.rank, bad);
    hipLaunchKernelGGL(ivb_stripe_totals_kernel, dim3((unsigned)((C + 255) / 256)), dim3(256), 0, st, x.counts, C, x.stripes,
                       x.total);
    hipLaunchKernelGGL(ivb_offsets_kernel, dim3(1), dim3(1024), 0, st, x.total, C, ivf_offsets, x.long_lists, x.n_long);
}
// After plaid_launch_ivf_build_offsets on the same scratch, and only when it reported no bad input.
void plaid_launch_ivf_build_fill(hipStream_t st, const int32_t *codes, const int64_t *doc_offsets, int64_t P, int64_t N,
                                 int64_t C, void *scratch, const int64_t *ivf_offsets, int32_t *ivf_pids, int64_t capacity)
{
    const IvbScratch x = ivb_carve(scratch, N, C);
    // (capacity >= the lists' total, which is at most N: every staged position is inside both buffers)
    hipLaunchKernelGGL(ivb_scatter_kernel, dim3(ivb_passage_blocks(P)), dim3(256), 0, st, codes, doc_offsets, P, N, C, x.stripes,
                       x.counts, ivf_offsets, x.rank, x.staged, capacity < N ? capacity : N);
    int64_t blocks = (C + 3) / 4;
    if (blocks > 32768) blocks = 32768;
    hipLaunchKernelGGL(ivb_sort_short_kernel, dim3((unsigned)blocks), dim3(256), 0, st, ivf_offsets, C, x.staged, ivf_pids);
    hipLaunchKernelGGL(ivb_sort_long_kernel, dim3(1024), dim3(1024), 0, st, ivf_offsets, x.long_lists, x.n_long, P, x.staged,
                       ivf_pids);
}

// ------------------------------------------------------------------ embedding-level inverted lists (vanilla ColBERTv2 retrieval)
// list c = the ascending indices of the tokens coded c (Section 4.1 describes vanilla's lists as centroid -> embedding
// ids).  Tokens are split into groups of consecutive indices.  Pass 1 counts per (group, centroid).  A scan over
// (centroid major, group minor) turns the counts into the position where each group starts writing inside each list.
// Pass 2 gives every group to one wave, which walks its tokens 64 at a time; a lane's position is the cursor of its code
// plus the number of earlier lanes of the chunk with the same code, so the list comes out in token order without a sort
// and without atomics.  (Built once per index for the baseline's retrieval; not on the search path.)
int64_t plaid_embedding_lists_groups(int64_t N)
{
    int64_t G = N < 2048 ? N : 2048;
    return G < 1 ? 1 : G;
}
size_t plaid_embedding_lists_scratch_bytes(int64_t N, int64_t C)
{
    return (size_t)plaid_embedding_lists_groups(N) * (size_t)C * 4 + (size_t)C * 8 + 256;
}
// One pass over the count table: counts[g][c] <- sum of counts[g'][c] over g' < g (the 32-bit position inside list c at
// which group g starts writing), total[c] = the sum over all groups (the list's length).
__global__ __launch_bounds__(256) void evb_totals_kernel(int32_t *__restrict__ counts, int64_t C, int64_t G,
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
__global__ __launch_bounds__(1024) void evb_scan_kernel(const int64_t *__restrict__ total, int64_t C,
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
// scratch: plaid_embedding_lists_scratch_bytes(N, C) bytes, zero on entry.  offsets [C+1], eids [N] (N < 2^31).
void plaid_launch_embedding_lists(hipStream_t st, const int32_t *codes, int64_t N, int64_t C, void *scratch, int64_t *offsets,
                                  int32_t *eids, int32_t *bad)
{
    const int64_t G = plaid_embedding_lists_groups(N), per = (N + G - 1) / G;
    int32_t *counts = (int32_t *)scratch;
    int64_t *total = (int64_t *)((char *)scratch + ((size_t)G * (size_t)C * 4 + 255) / 256 * 256);
    int64_t blocks = (N + 255) / 256;
    if (blocks > 16384) blocks = 16384;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(evb_count_kernel, dim3((unsigned)blocks), dim3(256), 0, st, codes, N, C, per > 0 ? per : 1, counts, bad);
    hipLaunchKernelGGL(evb_totals_kernel, dim3((unsigned)((C + 255) / 256)), dim3(256), 0, st, counts, C, G, total);
    hipLaunchKernelGGL(evb_scan_kernel, dim3(1), dim3(1024), 0, st, total, C, offsets);
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
