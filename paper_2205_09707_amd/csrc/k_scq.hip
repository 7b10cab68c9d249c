// Stage 1 in one kernel: query-centroid scores S_cq = C . Q^T (Eq. 2), the centroid pruning map of
// Eq. 5, the nprobe best centroids of every query token (Section 4.1) and the table of surviving
// centroids that stage 2 consumes.
//
// Every later decision of the pipeline (which centroids are probed, which survive t_cs, which
// passages make the ndocs and ndocs/4 cuts) is a comparison of S_cq values or of sums of them,
// so they are computed the way the definition reads: each S[c][i] is the dot product accumulated
// in double over the dimensions in index order, rounded once to fp32.  A product of two fp32
// values is exact in double, so a chain of fused multiply-adds in that order gives the same bits
// as "multiply, then add" on any machine -- the scores carry no accumulation-order freedom.
//
// Two kernels compute the same bits.
//
// Matrix form (scq_mfma_kernel): the double-precision matrix instruction D = A(16x4) B(4x16) + C adds its four
// products to C one after the other, rounding after each, i.e. it IS the chain of fused multiply-adds over four
// consecutive dimensions; 32 of them in a row walk the 128 dimensions in index order.  A workgroup of four waves
// owns 128 centroid rows and the 64 token columns of two queries; centroid rows are staged in LDS 32 dimensions at
// a time with coalesced loads, next to the same 32 dimensions of the queries in operand order, and a wave holds a
// 32 x 64 block of double accumulators.  That the instruction reproduces the chain is checked once per process on
// the device (plaid_scq_matrix_form_ok): if it ever did not, the vector form below is used instead.
//
// Vector form (scq_fused_kernel): a workgroup of eight waves owns 64 centroid rows, staged once in LDS with coalesced
// loads; wave g computes query tokens 4g..4g+3 for all 64 rows (lane = centroid, four double
// accumulators).  The query, pre-converted to double and laid out [token group][dim][4], is
// uniform across a wave and is fetched through the scalar unit, so the inner loop is one
// v_fma_f64 per (dimension, token) whose only per-lane operand is the LDS-resident centroid row.
//
// Either way the tile of results then yields the row maxima (pruning bits) and, per query token, the maximum of the
// tile's column.  The probes come from those maxima: with T the nprobe-th largest tile maximum of a token, each of
// the nprobe best tiles holds a score >= T, so the nprobe-th best score is >= T and every centroid among the nprobe
// best lies in a tile whose maximum is >= T -- normally just nprobe tiles.  A one-workgroup-per-query kernel finds T,
// ranks the rows of those tiles from S_cq, and builds the duplicate-free union of the probes and the survivor table.
// (Ranking inside the score kernel instead costs it a third of its running time: its waves' vector instructions
// queue behind other waves' matrix instructions.)
#include "plaid_internal.h"

#include <math.h>


#define SCQ_THREADS 512
#define SCQ_ROWS 64
#define SCQ_HALF 64      // dimensions staged at a time
#define SCQ_RSTRIDE 68   // floats per staged half row: 16-byte aligned, consecutive rows 4 banks apart
#define SCQ_SSTRIDE 33   // floats per row of the result tile (conflict-free column and row walks)
#define SCQ_GROUPS 8     // token groups = waves per workgroup
#define SCQ_TOK 4        // query tokens per wave
#define TAIL_THREADS 1024
#define TAIL_LANES 32     // lanes of the tail kernel that share one query token

// Vector form only (the matrix form does both inside its score kernel): clears the workspace region that must start
// at zero and lays out the queries, Qd[q][g][t][u] = (double) Q[q][4g + u][t].
__global__ __launch_bounds__(256) void stage1_prep_kernel(const float *__restrict__ Q, double *__restrict__ Qd, int nq,
                                                          uint32_t *__restrict__ zero, int64_t zero_words)
{
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < zero_words; i += (int64_t)gridDim.x * blockDim.x)
        zero[i] = 0u;
    for (int q = blockIdx.x; q < nq; q += gridDim.x)
        for (int e = threadIdx.x; e < QLEN * DIM; e += blockDim.x) {
            const int u = e & 3, t = (e >> 2) & (DIM - 1), g = e >> 9;
            Qd[(int64_t)q * QLEN * DIM + e] = (double)Q[(int64_t)q * QLEN * DIM + (4 * g + u) * DIM + t];
        }
}

template <int NP>
__device__ __forceinline__ void scq_insert_key(uint64_t (&best)[NP], uint64_t key)
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

// v into a descending list of NP values (the smallest drops out)
template <int NP>
__device__ __forceinline__ void scq_insert_desc(float (&top)[NP], float v)
{
    if (v > top[NP - 1]) {
#pragma unroll
        for (int j = NP - 1; j >= 0; --j)
            if (v > top[j]) {
                if (j + 1 < NP) top[j + 1] = top[j];
                top[j] = v;
            }
    }
}

struct Stage1Out {          // per-query outputs of the tail (device pointers, leading dimension = query)
    int32_t *probed;        // [nq][32][nprobe] best first
    int32_t *uniq;          // [nq][uniq_stride] ascending distinct probed centroids
    int32_t *n_uniq;        // [nq]
    int uniq_stride;
    S2Meta *meta;           // [nq]
    int32_t *kept_ids;      // [nq][S2_MAX_KEPT]
    float *T;               // [nq][S2_MAX_KEPT + 1][32]
    const int64_t *ivf_offsets;  // [C + 1] inverted-list offsets: slots are numbered by list length (null: by id)
    int32_t *qcount;        // [3] / [3][qlist_stride]: the queries by number of surviving centroids (none, 1..31, more),
    int32_t *qlist;         //   appended as their workgroups finish (null: not recorded).  Stage 2 runs one kernel per
    int qlist_stride;       //   class and takes its queries from these lists.
};

// One entry of S_cq as the definition reads: the products of the 128 dimensions accumulated in double in index order
// (a product of two fp32 values is exact in double, so the fused multiply-add chain is "multiply, then add"), rounded
// once to fp32.  Used where a decision must not rest on the split-fp16 kernel's approximate scores.
// crow: the centroid's row in global memory, fetched 32 dimensions at a time (eight 16-byte loads in flight); qrow: the
// query token's row, which the caller keeps in LDS.
__device__ __forceinline__ float scq_exact_entry(const float *__restrict__ crow, const float *qrow)
{
    double acc = 0.0;
#pragma unroll 1
    for (int d0 = 0; d0 < DIM; d0 += 32) {
        float4 c[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) c[u] = *reinterpret_cast<const float4 *>(crow + d0 + 4 * u);
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const float4 x = *reinterpret_cast<const float4 *>(qrow + d0 + 4 * u);
            acc = fma((double)c[u].x, (double)x.x, acc);
            acc = fma((double)c[u].y, (double)x.y, acc);
            acc = fma((double)c[u].z, (double)x.z, acc);
            acc = fma((double)c[u].w, (double)x.w, acc);
        }
    }
    return (float)acc;
}

// Survivor table of one query (runs in one workgroup, all of whose threads call it).  K = number of centroids
// passing Eq. 5; when K <= S2_MAX_KEPT their ids are listed ascending, their rows copied to T (slot s at T[s],
// s = 1..K), a collision-free hash shift is chosen for stage 2's table, and bin_hi / bin_scale are set from bounds
// of any non-empty passage's pruned score.  top1[i] = best centroid of token i (gives the bounds when K is large).
// APPROX (Sq comes from the split-fp16 kernel): the pruning bits were completed by this workgroup a moment ago with
// atomics, so they are read past the first-level cache, and the rows of T are re-evaluated in double from the centroids
// Cm and the query Qq, which makes every stage-2 score that is built from T the exact one.
template <bool APPROX>
__device__ __forceinline__ void stage1_survivor_table(const float *__restrict__ Sq, int64_t C, const uint32_t *__restrict__ kb,
                                      int64_t keep_words, const int32_t *top1, S2Meta *meta_q,
                                      int32_t *__restrict__ kept_ids_q, float *__restrict__ Tq, int32_t *scan /*[waves]*/,
                                      int32_t *ids /*[S2_MAX_KEPT + 1]*/, uint32_t *trial /*[S2_NHASH][S2_HASH / 32]*/,
                                      float *colmm /*[2][32]*/, int32_t *misc /*[2]*/, const float *__restrict__ Cm = nullptr,
                                      const float *Qq = nullptr /* the query's rows, in LDS */,
                                      const int64_t *__restrict__ ivf_offsets = nullptr, int q = 0,
                                      int32_t *qcount = nullptr, int32_t *qlist = nullptr, int qlist_stride = 0)
{
    auto keep_word = [&](int64_t w) -> uint32_t {
        if (APPROX) return __hip_atomic_load(kb + w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return kb[w];
    };
    const int tid = threadIdx.x, nthreads = blockDim.x;
    if (tid == 0) {
        misc[0] = 0;   // running count of survivors
        misc[1] = -1;  // chosen hash trial
    }
    for (int e = tid; e < S2_NHASH * (S2_HASH / 32); e += nthreads) trial[e] = 0u;
    __syncthreads();
    // survivors in ascending id order: thread t owns the contiguous words [t * per, (t + 1) * per); positions come from
    // a wave-level prefix sum of the per-thread counts plus the wave totals (scan[wave])
    {
        const int64_t per = (keep_words + nthreads - 1) / nthreads;
        const int64_t wa = (int64_t)tid * per, wb = wa + per < keep_words ? wa + per : keep_words;
        int cnt = 0;
        for (int64_t w = wa; w < wb; ++w) cnt += __popc(keep_word(w));
        int incl = cnt;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int t = __shfl_up(incl, d);
            if ((tid & 63) >= d) incl += t;
        }
        if ((tid & 63) == 63) scan[tid >> 6] = incl;
        __syncthreads();
        int start = incl - cnt;
        for (int wv = 0; wv < (tid >> 6); ++wv) start += scan[wv];
        int pos = start;
        for (int64_t w = wa; w < wb && pos < S2_MAX_KEPT; ++w) {
            uint32_t v = keep_word(w);
            while (v && pos < S2_MAX_KEPT) {
                const int b = __ffs(v) - 1;
                v &= v - 1;
                ids[pos++] = (int32_t)(w * 32 + b);
            }
        }
        if (tid == nthreads - 1) misc[0] = start + cnt;  // total number of survivors
        __syncthreads();
    }
    int K = misc[0];
    if (C > (1ll << 26) - 2 && K <= S2_MAX_KEPT) K = S2_MAX_KEPT + 1;  // ids must fit the 26-bit field of a table entry
    // Slots in the order of decreasing inverted-list length (ties: smaller id first): the centroids most passages hold
    // get the lowest slots, which stage 2 scores through a table of their subsets.
    if (ivf_offsets && K > 1 && K <= S2_MAX_KEPT) {
        int32_t my_id = 0;
        int rank = 0;
        uint32_t *lens = trial;  // the first K words serve as the list lengths here and are cleared again below
        if (tid < K) {
            my_id = ids[tid];
            lens[tid] = (uint32_t)(ivf_offsets[my_id + 1] - ivf_offsets[my_id]);  // at most P < 2^31 entries
        }
        __syncthreads();
        if (tid < K) {
            const uint32_t my_len = lens[tid];
            for (int u = 0; u < K; ++u) {
                const uint32_t len = lens[u];
                rank += (len > my_len || (len == my_len && u < tid)) ? 1 : 0;
            }
        }
        __syncthreads();
        if (tid < K) {
            ids[rank] = my_id;
            lens[tid] = 0u;
        }
        __syncthreads();
    }
    // a hash h(c) = (c ^ (c >> sh)) & (S2_HASH - 1) that maps the survivors to distinct entries makes a lookup one
    // probe; thread t tries shift S2_SHIFT0 + t on a private bitmap.  No such shift (very rare): gather kernel.
    if (K <= S2_MAX_KEPT) {
        bool ok = tid < S2_NHASH;
        if (ok) {
            const int sh = S2_SHIFT0 + tid;
            uint32_t *mine = trial + tid * (S2_HASH / 32);
            for (int s = 0; s < K; ++s) {
                const uint32_t c = (uint32_t)ids[s];
                const uint32_t h = (c ^ (c >> sh)) & (S2_HASH - 1);
                const uint32_t bit = 1u << (h & 31);
                if (mine[h >> 5] & bit) ok = false;
                mine[h >> 5] |= bit;
            }
        }
        if (ok) atomicMax(&misc[1], S2_NHASH - 1 - tid);  // smallest successful shift wins
        __syncthreads();
        if (misc[1] < 0) K = S2_MAX_KEPT + 1;
    }
    const int hash_shift = (K <= S2_MAX_KEPT) ? S2_SHIFT0 + (S2_NHASH - 1 - misc[1]) : 0;
    if (K <= S2_MAX_KEPT) {
        for (int e = tid; e < K * QLEN; e += nthreads)
            Tq[QLEN + e] = APPROX ? scq_exact_entry(Cm + (int64_t)ids[e >> 5] * DIM, Qq + (e & 31) * DIM)
                                  : Sq[(int64_t)ids[e >> 5] * QLEN + (e & 31)];
        if (tid < K) kept_ids_q[tid] = ids[tid];
        if (tid < QLEN) {
            float mx = -INFINITY, mn = INFINITY;
            for (int s0 = 0; s0 < K; s0 += 8) {  // eight rows in flight
                float v[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) v[u] = Sq[(int64_t)ids[s0 + u < K ? s0 + u : s0] * QLEN + tid];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    mx = fmaxf(mx, v[u]);
                    mn = fminf(mn, v[u]);
                }
            }
            colmm[tid] = mx;
            colmm[QLEN + tid] = mn;
        }
    } else if (tid < QLEN) {
        // many survivors: the best centroid of each token bounds every row from above
        const float mx = Sq[(int64_t)top1[tid] * QLEN + tid];
        colmm[tid] = mx;
        colmm[QLEN + tid] = -mx - 1.0f;
    }
    __syncthreads();
    if (tid == 0) {
        double u = 0.0, l = 0.0;
        for (int i = 0; i < QLEN; ++i) {
            u += (double)colmm[i];
            l += (double)colmm[QLEN + i];
        }
        S2Meta m;
        m.K = K;
        m.bin_hi = (float)u;
        const float range = (float)u - (float)l;
        m.bin_scale = (K > 0 && range > 0.f && range < INFINITY) ? (float)SEL_BINS / range : 0.f;
        m.hash_shift = hash_shift;
        *meta_q = m;
        if (qlist) {
            const int cls = K == 0 ? 0 : (K <= 31 ? 1 : 2);
            const int at = atomicAdd(&qcount[cls], 1);
            if (at < qlist_stride) qlist[(int64_t)cls * qlist_stride + at] = q;  // (always, when the counts start at zero)
        }
    }
}

// Standalone form for the general top-nprobe path (nprobe > 8), where the probes come from the generic selection.
__global__ __launch_bounds__(512) void stage1_survivor_kernel(const float *__restrict__ S, int64_t C,
                                                              const uint32_t *__restrict__ keepbits, int64_t keep_words,
                                                              const int32_t *__restrict__ probed, int nprobe, Stage1Out o)
{
    __shared__ int32_t scan[512];
    __shared__ int32_t ids[S2_MAX_KEPT + 1];
    __shared__ uint32_t trial[S2_NHASH * (S2_HASH / 32)];
    __shared__ float colmm[2 * QLEN];
    __shared__ int32_t misc[2];
    __shared__ int32_t top1[QLEN];
    const int q = blockIdx.x;
    if (threadIdx.x < QLEN) top1[threadIdx.x] = probed[((int64_t)q * QLEN + threadIdx.x) * nprobe];
    __syncthreads();
    stage1_survivor_table<false>(S + (int64_t)q * C * QLEN, C, keepbits + (int64_t)q * keep_words, keep_words, top1, o.meta + q,
                                 o.kept_ids + (int64_t)q * S2_MAX_KEPT, o.T + (int64_t)q * (S2_MAX_KEPT + 1) * QLEN, scan, ids,
                                 trial, colmm, misc, nullptr, nullptr, o.ivf_offsets, q, o.qcount, o.qlist, o.qlist_stride);
}

// tilemax: [q][tile][32] column maxima of each tile (null: scores and pruning bits only).
__global__ __launch_bounds__(SCQ_THREADS) void scq_fused_kernel(const float *__restrict__ Cm, int64_t C,
                                                                const double *__restrict__ Qd, float t_cs,
                                                                float *__restrict__ S, uint32_t *__restrict__ keepbits,
                                                                int64_t keep_words, float *__restrict__ tilemax)
{
    // one LDS arena: half of the centroid tile (64 dimensions) at a time during the contraction; afterwards the 64x32
    // result tile and the partial column maxima
    constexpr int ARENA_FLOATS = SCQ_ROWS * SCQ_RSTRIDE > SCQ_ROWS * SCQ_SSTRIDE + 8 * QLEN
                                     ? SCQ_ROWS * SCQ_RSTRIDE
                                     : SCQ_ROWS * SCQ_SSTRIDE + 8 * QLEN;
    __shared__ __align__(16) float arena[ARENA_FLOATS];
    float *tile = arena;                             // [64][SCQ_SSTRIDE]
    float *cm = arena + SCQ_ROWS * SCQ_SSTRIDE;      // [8][32]
    const int q = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63;
    const int g = __builtin_amdgcn_readfirstlane(tid >> 6);  // token group of this wave (uniform -> scalar loads of Qd)
    const int64_t c0 = (int64_t)blockIdx.x * SCQ_ROWS;
    const int nrows = (int)(C - c0 < SCQ_ROWS ? C - c0 : SCQ_ROWS);

    // staging: a half tile is 64 rows x 64 dims = 1024 float4, two per thread; 256-byte row halves read contiguously.
    // The second half is requested before the first is multiplied, so only the first load's latency is exposed.
    const int r0 = tid >> 4, c4 = tid & 15;  // this thread stages rows r0 and r0 + 32, float4 column c4
    float4 pre[2];
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        const int r = r0 + 32 * k;
        pre[k] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (r < nrows) pre[k] = *reinterpret_cast<const float4 *>(Cm + (c0 + r) * DIM + 4 * c4);
    }
    const double *__restrict__ qd = Qd + ((int64_t)q * SCQ_GROUPS + g) * DIM * SCQ_TOK;
    const float4 *row = reinterpret_cast<const float4 *>(arena + lane * SCQ_RSTRIDE);
    double acc[SCQ_TOK] = {0.0, 0.0, 0.0, 0.0};
#pragma unroll 1
    for (int half = 0; half < DIM / SCQ_HALF; ++half) {
#pragma unroll
        for (int k = 0; k < 2; ++k)
            *reinterpret_cast<float4 *>(arena + (r0 + 32 * k) * SCQ_RSTRIDE + 4 * c4) = pre[k];
        __syncthreads();
        if (half + 1 < DIM / SCQ_HALF) {
#pragma unroll
            for (int k = 0; k < 2; ++k) {
                const int r = r0 + 32 * k;
                if (r < nrows) pre[k] = *reinterpret_cast<const float4 *>(Cm + (c0 + r) * DIM + SCQ_HALF * (half + 1) + 4 * c4);
            }
        }
        // the query operands of the next four dimensions are requested (scalar loads) before the current four are used
        const double *__restrict__ qh = qd + half * SCQ_HALF * SCQ_TOK;
        double qa[4 * SCQ_TOK], qb[4 * SCQ_TOK];
#pragma unroll
        for (int e = 0; e < 4 * SCQ_TOK; ++e) qa[e] = qh[e];
#pragma unroll 1
        for (int t8 = 0; t8 < SCQ_HALF / 8; ++t8) {
            {
#pragma unroll
                for (int e = 0; e < 4 * SCQ_TOK; ++e) qb[e] = qh[(8 * t8 + 4) * SCQ_TOK + e];
                const float4 a4 = row[2 * t8];
                const double a[4] = {(double)a4.x, (double)a4.y, (double)a4.z, (double)a4.w};
#pragma unroll
                for (int u = 0; u < 4; ++u)
#pragma unroll
                    for (int i = 0; i < SCQ_TOK; ++i) acc[i] = fma(a[u], qa[u * SCQ_TOK + i], acc[i]);
            }
            {
                const int tn = t8 + 1 < SCQ_HALF / 8 ? 8 * t8 + 8 : 0;  // the last round re-reads the first operands (unused)
#pragma unroll
                for (int e = 0; e < 4 * SCQ_TOK; ++e) qa[e] = qh[tn * SCQ_TOK + e];
                const float4 a4 = row[2 * t8 + 1];
                const double a[4] = {(double)a4.x, (double)a4.y, (double)a4.z, (double)a4.w};
#pragma unroll
                for (int u = 0; u < 4; ++u)
#pragma unroll
                    for (int i = 0; i < SCQ_TOK; ++i) acc[i] = fma(a[u], qb[u * SCQ_TOK + i], acc[i]);
            }
        }
        __syncthreads();  // every wave is done with this half: the arena is rewritten next
    }
    const float4 s4 = make_float4((float)acc[0], (float)acc[1], (float)acc[2], (float)acc[3]);
    if (lane < nrows) *reinterpret_cast<float4 *>(S + ((int64_t)q * C + c0 + lane) * QLEN + SCQ_TOK * g) = s4;
    float *trow = tile + lane * SCQ_SSTRIDE + SCQ_TOK * g;
    trow[0] = s4.x;
    trow[1] = s4.y;
    trow[2] = s4.z;
    trow[3] = s4.w;
    __syncthreads();

    // Eq. 5: pruning bits of the 64 rows (wave 0)
    if (tid < 64) {
        float m = -INFINITY;
#pragma unroll
        for (int i = 0; i < QLEN; ++i) m = fmaxf(m, tile[tid * SCQ_SSTRIDE + i]);
        const unsigned long long b = __ballot(tid < nrows && m >= t_cs);
        if (tid == 0) {
            uint32_t *kb = keepbits + (int64_t)q * keep_words + (c0 >> 5);
            kb[0] = (uint32_t)b;
            if ((c0 >> 5) + 1 < keep_words) kb[1] = (uint32_t)(b >> 32);
        }
    }
    if (!tilemax) return;  // uniform

    // column maxima of the tile: thread (i, p) takes rows 8p .. 8p+7 of column i
    if (tid < 256) {
        const int i = tid & 31, p = tid >> 5;
        float m = -INFINITY;
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const int rr = 8 * p + r;
            if (rr < nrows) m = fmaxf(m, tile[rr * SCQ_SSTRIDE + i]);
        }
        cm[p * QLEN + i] = m;
    }
    __syncthreads();
    if (tid < QLEN) {
        float m = cm[tid];
#pragma unroll
        for (int p = 1; p < 8; ++p) m = fmaxf(m, cm[p * QLEN + tid]);
        tilemax[((int64_t)q * gridDim.x + blockIdx.x) * QLEN + tid] = m;
    }
}


// ------------------------------------------------------------------ matrix form
typedef double scq_double4 __attribute__((ext_vector_type(4)));
// Four waves of 32 rows measured best: eight waves of 16 rows (more waves per SIMD to fill the matrix pipe while
// others are in their epilogue) lose more to the per-wave epilogue instructions than they gain (5.2 vs 4.95 ms per 512
// queries on C = 65536), 64 rows per wave halve the occupancy.
#define SM_THREADS 256
#define SM_RT 2                      // 16-row tiles per wave
#define SM_WAVES (SM_THREADS / 64)
#define SM_WROWS (16 * SM_RT)        // centroid rows per wave
#define SM_ROWS (SM_WAVES * SM_WROWS)  // centroid rows per workgroup
static_assert(SM_WROWS == 16 || SM_WROWS == 32, "pruning bits are assembled from 16- or 32-row pieces");
static_assert(SM_ROWS % (SM_THREADS / 8) == 0 && SM_THREADS >= QLEN, "tile shape");
#define SM_KC 32                     // dimensions staged at a time
#define SM_ASTRIDE 36                // floats per staged row chunk: the 64 operand reads of a step hit 64 banks
#define SM_MIN_WAVES 4               // waves per SIMD the register allocation leaves room for

// Operand and result layout of v_mfma_f64_16x16x4_f64 for lane = 16 g + i: A operand = A[i][g], B operand = B[g][i],
// result register r = D[4 r + g][i].
__device__ __forceinline__ scq_double4 scq_mma(double a, double b, scq_double4 c)
{
    return __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, c, 0, 0, 0);
}

// Workgroup barrier that orders LDS accesses only.  __syncthreads() also waits for every outstanding global store, and
// this kernel has 16 KB of score stores in flight per query when it reaches the barriers that guard the LDS tile.
__device__ __forceinline__ void scq_lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// NQ = queries per workgroup (1 or 2).  Grid: x = query group, y = row block.
// tilemax: [q][32-row block][32] column maxima over the 32 rows a wave owns (null: scores and pruning bits only).
template <int NQ>
__global__ __launch_bounds__(SM_THREADS, SM_MIN_WAVES) void scq_mfma_kernel(const float *__restrict__ Cm, int64_t C,
                                                              const float *__restrict__ Q, int nq, float t_cs,
                                                              float *__restrict__ S, uint32_t *__restrict__ keepbits,
                                                              int64_t keep_words, float *__restrict__ tilemax,
                                                              uint32_t *__restrict__ zero, int64_t zero_words)
{
    constexpr int NT = 2 * NQ;  // 16-column tiles
    __shared__ __align__(16) float arena[SM_ROWS * SM_ASTRIDE];  // staged centroid chunk
    __shared__ __align__(16) float Bq[(SM_KC / 4) * NT * 64];    // the chunk's query operands: [step][column tile][lane]
    const int tid = threadIdx.x, lane = tid & 63, li = lane & 15, lg = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // Outside the matrix loop a wave runs at raised priority: its few vector instructions (set-up, staging, epilogue)
    // would otherwise wait their turn behind the matrix instructions of every other wave on the SIMD, and the sooner a
    // wave is through them, the sooner it feeds the matrix pipe again.
    __builtin_amdgcn_s_setprio(3);
    // the workspace words that later kernels expect to be zero are cleared here, by the whole grid (no kernel of this
    // search has touched them yet, and every kernel of the previous one has finished)
    for (int64_t i = ((int64_t)blockIdx.y * gridDim.x + blockIdx.x) * SM_THREADS + tid; i < zero_words;
         i += (int64_t)gridDim.x * gridDim.y * SM_THREADS)
        zero[i] = 0u;
    const int q0 = blockIdx.x * NQ;
    const int64_t c0 = (int64_t)blockIdx.y * SM_ROWS;
    const int nrows = (int)(C - c0 < SM_ROWS ? C - c0 : SM_ROWS);

    // staging: a chunk is SM_ROWS rows x 32 dims = 8 float4 per row; thread -> rows tid/8 + SM_RPP k, float4 column tid%8
    constexpr int SM_RPP = SM_THREADS / 8;  // rows per staging pass
    const int r0 = tid >> 3, c4 = tid & 7;
    float4 pre[SM_ROWS / SM_RPP];
#pragma unroll
    for (int k = 0; k < SM_ROWS / SM_RPP; ++k) {
        const int r = r0 + SM_RPP * k;
        pre[k] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (r < nrows) pre[k] = *reinterpret_cast<const float4 *>(Cm + (c0 + r) * DIM + 4 * c4);
    }
    // The queries' operands of a chunk, in operand order [step][column tile][lane]: 8 steps x 2 halves x 64 lanes per
    // query, four consecutive lanes per thread: 256 threads per query, thread bt of them (zeros for a query past the
    // end).  Lane 16 g + i of step s, half h holds Q[16 h + i][4 s + g], so a thread's four values are one column of
    // four consecutive query tokens.
    static_assert(SM_THREADS % 256 == 0, "query staging works in groups of 256 threads");
    constexpr int BQ_PASSES = (NQ * 256 + SM_THREADS - 1) / SM_THREADS;  // queries staged per thread
    const int bt = tid & 255;
    const int bdst = (((bt >> 5) * NT + ((bt >> 4) & 1)) * 64 + 4 * (bt & 15));  // + 2 qi column tiles
    const int bsrc = (16 * ((bt >> 4) & 1) + 4 * (bt & 3)) * DIM + 4 * (bt >> 5) + ((bt >> 2) & 3);  // + 32 ch
    float4 preb[BQ_PASSES];
#pragma unroll
    for (int k = 0; k < BQ_PASSES; ++k) {
        const int qi = (tid >> 8) + (SM_THREADS / 256) * k;
        preb[k] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (qi < NQ && q0 + qi < nq) {
            const float *src = Q + (int64_t)(q0 + qi) * QLEN * DIM + bsrc;
            preb[k] = make_float4(src[0], src[DIM], src[2 * DIM], src[3 * DIM]);
        }
    }
    scq_double4 acc[SM_RT][NT];
#pragma unroll
    for (int m = 0; m < SM_RT; ++m)
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[m][t] = scq_double4{0.0, 0.0, 0.0, 0.0};
    const float *arow = arena + (wave * SM_WROWS + li) * SM_ASTRIDE + lg;  // + 16 m rows, + 4 j floats
    const float *bcol = Bq + lane;
#pragma unroll 1
    for (int ch = 0; ch < DIM / SM_KC; ++ch) {
#pragma unroll
        for (int k = 0; k < SM_ROWS / SM_RPP; ++k)
            *reinterpret_cast<float4 *>(arena + (r0 + SM_RPP * k) * SM_ASTRIDE + 4 * c4) = pre[k];
#pragma unroll
        for (int k = 0; k < BQ_PASSES; ++k) {
            const int qi = (tid >> 8) + (SM_THREADS / 256) * k;
            if (qi < NQ) *reinterpret_cast<float4 *>(Bq + bdst + 2 * qi * 64) = preb[k];
        }
        scq_lds_barrier();
        if (ch + 1 < DIM / SM_KC) {
#pragma unroll
            for (int k = 0; k < SM_ROWS / SM_RPP; ++k) {
                const int r = r0 + SM_RPP * k;
                if (r < nrows) pre[k] = *reinterpret_cast<const float4 *>(Cm + (c0 + r) * DIM + SM_KC * (ch + 1) + 4 * c4);
            }
#pragma unroll
            for (int k = 0; k < BQ_PASSES; ++k) {
                const int qi = (tid >> 8) + (SM_THREADS / 256) * k;
                if (qi < NQ && q0 + qi < nq) {
                    const float *src = Q + (int64_t)(q0 + qi) * QLEN * DIM + bsrc + SM_KC * (ch + 1);
                    preb[k] = make_float4(src[0], src[DIM], src[2 * DIM], src[3 * DIM]);
                }
            }
        }
        __builtin_amdgcn_s_setprio(0);
#pragma unroll
        for (int j = 0; j < SM_KC / 4; ++j) {
            double a[SM_RT], b[NT];
#pragma unroll
            for (int m = 0; m < SM_RT; ++m) a[m] = (double)arow[16 * m * SM_ASTRIDE + 4 * j];
#pragma unroll
            for (int t = 0; t < NT; ++t) b[t] = (double)bcol[(j * NT + t) * 64];
#pragma unroll
            for (int m = 0; m < SM_RT; ++m)
#pragma unroll
                for (int t = 0; t < NT; ++t) acc[m][t] = scq_mma(a[m], b[t], acc[m][t]);
        }
        __builtin_amdgcn_s_setprio(3);
        if (ch + 1 < DIM / SM_KC) scq_lds_barrier();  // every wave is done with this chunk: the arena is rewritten next
    }

    // Epilogue, straight from the accumulators (no LDS, no barrier: every vector instruction here queues behind the
    // matrix instructions of the other waves on the SIMD, so the fewer the better).  Lane 16 g + i holds rows 4 r + g of
    // columns i and 16 + i of each 16-row tile: a store instruction writes four 64-byte row halves, the two halves of
    // a row back to back.  Eq. 5: the comparison's lane mask holds, in its 16-bit field g, the columns of row 4 r + g, so
    // a row passes when its field is not zero -- scalar work on the mask, none per lane.
    const bool ragged = nrows < SM_ROWS;  // rows past the end of the table hold zeros: not stored, not in a maximum
    const int wrow0 = wave * SM_WROWS;
    const int wrows = nrows - wrow0 < 0 ? 0 : (nrows - wrow0 < SM_WROWS ? nrows - wrow0 : SM_WROWS);  // this wave's rows
    static_assert(SM_WROWS == 32, "one word of the pruning bitmap per wave");
#pragma unroll
    for (int qi = 0; qi < NQ; ++qi) {
        const int q = q0 + qi;
        if (q >= nq) break;  // uniform
        uint32_t kbits = 0u;                     // uniform: bit = row within the wave's 32 rows
        float cm0 = -INFINITY, cm1 = -INFINITY;  // maxima of this lane's two columns (tokens li and 16 + li) over its rows
        float *srow = S + ((int64_t)q * C + c0 + wrow0 + lg) * QLEN + li;
#pragma unroll
        for (int m = 0; m < SM_RT; ++m)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int row = 16 * m + 4 * r;  // + lg
                const float v0 = (float)acc[m][2 * qi][r], v1 = (float)acc[m][2 * qi + 1][r];
                if (!ragged || row + lg < wrows) {
                    srow[row * QLEN] = v0;
                    srow[row * QLEN + 16] = v1;
                    // med3(a, b, +inf) = max(a, b) for ordered operands, without the canonicalising copies of fmaxf
                    cm0 = __builtin_amdgcn_fmed3f(cm0, v0, INFINITY);
                    cm1 = __builtin_amdgcn_fmed3f(cm1, v1, INFINITY);
                }
                const unsigned long long pass = __ballot(v0 >= t_cs || v1 >= t_cs);
                const uint32_t lo = (uint32_t)pass, hi = (uint32_t)(pass >> 32);
                const uint32_t nib = ((lo & 0xFFFFu) ? 1u : 0u) | ((lo >> 16) ? 2u : 0u) | ((hi & 0xFFFFu) ? 4u : 0u) |
                                     ((hi >> 16) ? 8u : 0u);
                kbits |= nib << row;
            }
        if (tilemax) {  // uniform
            cm0 = __builtin_amdgcn_fmed3f(cm0, __shfl_xor(cm0, 16), INFINITY);
            cm1 = __builtin_amdgcn_fmed3f(cm1, __shfl_xor(cm1, 16), INFINITY);
            cm0 = __builtin_amdgcn_fmed3f(cm0, __shfl_xor(cm0, 32), INFINITY);
            cm1 = __builtin_amdgcn_fmed3f(cm1, __shfl_xor(cm1, 32), INFINITY);
            const int64_t blk = (int64_t)blockIdx.y * SM_WAVES + wave, n_blk = (C + SM_WROWS - 1) / SM_WROWS;
            if (lg == 0 && blk < n_blk) {  // a block with a row in range; rows past the end were left out above
                float *tmx = tilemax + ((int64_t)q * n_blk + blk) * QLEN + li;
                tmx[0] = cm0;
                tmx[16] = cm1;
            }
        }
        // rows past the end of the centroid table (a ragged last block) never pass
        if (wrows < SM_WROWS) kbits &= (1u << wrows) - 1u;
        const int64_t w0 = (c0 >> 5) + wave;  // one 32-bit word of the pruning bitmap per 32 rows
        if (lane == 0 && w0 < keep_words) keepbits[(int64_t)q * keep_words + w0] = kbits;
    }
}

// One wave: the matrix instruction chained over 128 dimensions against the chain of fused multiply-adds, on
// pseudo-random fp32 operands; mismatch[0] counts results whose bits differ.
__global__ __launch_bounds__(64) void scq_matrix_form_check_kernel(uint32_t seed, int32_t *__restrict__ mismatch)
{
    __shared__ float A[16][DIM], B[DIM][16];
    const int lane = threadIdx.x, li = lane & 15, lg = lane >> 4;
    uint32_t x = seed * 2654435761u + (uint32_t)lane * 40503u + 12345u;
    for (int e = lane; e < 16 * DIM; e += 64) {
        x = x * 1664525u + 1013904223u;
        (&A[0][0])[e] = (float)(int32_t)(x >> 8) * (1.0f / 8388608.0f) - 1.0f;
        x = x * 1664525u + 1013904223u;
        (&B[0][0])[e] = (float)(int32_t)(x >> 8) * (1.0f / 8388608.0f) - 1.0f;
    }
    __syncthreads();
    scq_double4 acc = {0.0, 0.0, 0.0, 0.0};
    for (int s = 0; s < DIM / 4; ++s) acc = scq_mma((double)A[li][4 * s + lg], (double)B[4 * s + lg][li], acc);
    int bad = 0;
    for (int r = 0; r < 4; ++r) {
        const int row = 4 * r + lg;
        double c = 0.0;
        for (int k = 0; k < DIM; ++k) c = fma((double)A[row][k], (double)B[k][li], c);
        bad += __double_as_longlong(c) != __double_as_longlong(acc[r]) ? 1 : 0;
    }
    if (bad) atomicAdd(mismatch, bad);
}

int plaid_scq_matrix_form_ok(hipStream_t st, int *ok)
{
    *ok = 0;
    int32_t *d = nullptr;
    hipError_t e = hipMalloc((void **)&d, sizeof(int32_t));
    if (e != hipSuccess) return (int)e;
    int32_t h = -1;
    e = hipMemsetAsync(d, 0, sizeof(int32_t), st);
    for (uint32_t seed = 1; e == hipSuccess && seed <= 64; ++seed)
        hipLaunchKernelGGL(scq_matrix_form_check_kernel, dim3(1), dim3(64), 0, st, seed, d);
    if (e == hipSuccess) e = hipGetLastError();
    if (e == hipSuccess) e = hipMemcpyAsync(&h, d, sizeof(int32_t), hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    (void)hipFree(d);
    if (e != hipSuccess) return (int)e;
    *ok = h == 0 ? 1 : 0;
    return 0;
}

// One workgroup per query: the probes (rank order) from the tiles' column maxima, their ascending duplicate-free
// union, and the survivor table.  tilemax is [tile][token]: a thread reads four tokens of every 128th tile (16-byte
// loads, consecutive threads at consecutive addresses, eight loads in flight) and keeps each token's NP largest; the
// eight lanes of a wave that share tokens merge their lists by shuffles.  Then 32 consecutive lanes share a token:
// T = the nprobe-th largest of the token's tile maxima (nprobe rounds of "maximum over the 32 lanes, its first holder
// drops it").  A second pass over tilemax lists the tiles whose maximum is >= T in LDS (normally nprobe of them; a
// tie group too long for the list makes the lanes walk all tiles instead); their rows are ranked by (score
// descending, id ascending) from S_cq, four loads per lane in flight, and the 32 lists are merged by a shuffle tree.
// tile_rows = centroid rows per tile.
//
// APPROX: S, its tile maxima and the pruning bits come from the split-fp16 kernel, every entry within eps =
// PLAID_SCQ16_EPS of the exact one.  The decisions stay those of the exact scores:
//   probes   at least nprobe entries are >= T (approximately), hence >= T - eps exactly, so the nprobe-th best exact
//            score is >= T - eps and every centroid among the nprobe best has an approximate score >= T - 2 eps.  The
//            tiles with maximum >= T - 2 eps are listed, and each of their rows with a score >= T - 2 eps (normally
//            just the nprobe best) is re-evaluated in double and ranked by its exact score;
//   pruning  a row whose approximate maximum lies within eps of t_cs was left open by the score kernel (ambbits): its
//            entries >= t_cs - eps are re-evaluated and the row's bit is set when one of them reaches t_cs;
//   table    the rows of the surviving centroids that stage 2 scores with are re-evaluated (stage1_survivor_table).
#define TAIL_SEL 16  // listed tiles per token
#define TAIL_AMB 2048  // ambiguous rows decided per round
struct Stage1Exact {        // what the re-evaluations need (APPROX only)
    const float *Cm;        // [C][128] centroids
    const float *Q;         // [nq][32][128] queries
    const uint32_t *ambbits;  // [nq][keep_words]
    float t_cs, t_lo;       // threshold of Eq. 5 and the smallest approximate score that can still reach it
    float margin;           // 2 eps
};
template <int NP, bool APPROX>
__global__ __launch_bounds__(TAIL_THREADS) void stage1_tail_kernel(const float *__restrict__ S, int64_t C,
                                                                   uint32_t *__restrict__ keepbits, int64_t keep_words,
                                                                   const float *__restrict__ tilemax, int nblk, int tile_rows,
                                                                   int nprobe, Stage1Out o, Stage1Exact x)
{
    __shared__ int32_t idl[256];   // probed ids
    __shared__ int32_t top1[QLEN];
    __shared__ int32_t scan[TAIL_THREADS / 64 + 1];
    __shared__ int32_t ids[S2_MAX_KEPT + 1];
    __shared__ uint32_t trial[S2_NHASH * (S2_HASH / 32)];
    __shared__ float colmm[2 * QLEN];
    __shared__ int32_t misc[2];
    constexpr int TAIL_WAVES = TAIL_THREADS / 64;
    constexpr int TAIL_FLY = 8;                          // loads in flight per thread
    constexpr int TAIL_PARTS = TAIL_THREADS / (QLEN / 4);  // threads that share four tokens
    __shared__ float cand[QLEN][TAIL_WAVES * NP + 1];  // each wave's NP largest tile maxima of every token
    static_assert(TAIL_WAVES <= TAIL_LANES, "one lane per wave list");
    __shared__ float Tsh[QLEN];
    __shared__ int32_t sel_cnt[QLEN];
    __shared__ int32_t sel_tile[QLEN][TAIL_SEL];
    static_assert(TAIL_THREADS == QLEN * TAIL_LANES && TAIL_LANES == 32, "32 lanes per query token");
    const int q = blockIdx.x, tid = threadIdx.x;
    const float *__restrict__ Sq = S + (int64_t)q * C * QLEN;
    const float *__restrict__ tmq = tilemax + (int64_t)q * nblk * QLEN;
    const float margin = APPROX ? x.margin : 0.f;
    // APPROX: the query's rows in LDS for the re-evaluations, and per token the rows to re-evaluate
    constexpr int TAIL_XCAP = TAIL_LANES;  // listed rows per token: one per lane
    __shared__ __align__(16) float Qs[APPROX ? QLEN * DIM : 4];
    __shared__ int32_t xc_id[APPROX ? QLEN : 1][TAIL_XCAP];
    __shared__ int32_t xc_cnt[QLEN];
    const float *Qq = Qs;
    if (APPROX) {
        static_assert(TAIL_THREADS * 4 == QLEN * DIM, "one 16-byte load per thread stages the query");
        *reinterpret_cast<float4 *>(Qs + 4 * tid) = *reinterpret_cast<const float4 *>(x.Q + (int64_t)q * QLEN * DIM + 4 * tid);
    }
    {
        // pass 1: thread (tokens 4 tk4 .. 4 tk4 + 3, part) keeps the NP largest maxima of tiles part, part + 128, ...
        const int tk4 = tid % (QLEN / 4), part = tid / (QLEN / 4);
        float top[4][NP];
#pragma unroll
        for (int c = 0; c < 4; ++c)
#pragma unroll
            for (int j = 0; j < NP; ++j) top[c][j] = -INFINITY;
        for (int b0 = part; b0 < nblk; b0 += TAIL_PARTS * TAIL_FLY) {
            float4 v[TAIL_FLY];
#pragma unroll
            for (int u = 0; u < TAIL_FLY; ++u) {
                const int b = b0 + TAIL_PARTS * u;
                v[u] = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
                if (b < nblk) v[u] = *reinterpret_cast<const float4 *>(tmq + (int64_t)b * QLEN + 4 * tk4);
            }
#pragma unroll
            for (int u = 0; u < TAIL_FLY; ++u) {
                const float x[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
                for (int c = 0; c < 4; ++c) scq_insert_desc<NP>(top[c], x[c]);
            }
        }
        // the lanes of a wave with the same tk4 are 8 apart
#pragma unroll
        for (int d = QLEN / 4; d < 64; d <<= 1)
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                float other[NP];
#pragma unroll
                for (int j = 0; j < NP; ++j) other[j] = __shfl_xor(top[c][j], d);
#pragma unroll
                for (int j = 0; j < NP; ++j) scq_insert_desc<NP>(top[c], other[j]);
            }
        if ((tid & 63) < QLEN / 4) {
#pragma unroll
            for (int c = 0; c < 4; ++c)
#pragma unroll
                for (int j = 0; j < NP; ++j) cand[4 * tk4 + c][(tid >> 6) * NP + j] = top[c][j];
        }
    }
    __syncthreads();
    const int i = tid / TAIL_LANES, l = tid % TAIL_LANES;
    {
        float top[NP];  // descending
#pragma unroll
        for (int j = 0; j < NP; ++j) top[j] = l < TAIL_WAVES ? cand[i][l * NP + j] : -INFINITY;
        float T = -INFINITY;
#pragma unroll
        for (int r = 0; r < NP; ++r)
            if (r < nprobe) {  // uniform
                float m = top[0];
#pragma unroll
                for (int d = TAIL_LANES / 2; d > 0; d >>= 1) m = fmaxf(m, __shfl_xor(m, d));
                T = m;
                const unsigned long long who = __ballot(top[0] == m);
                const uint32_t mine = (tid & 32) ? (uint32_t)(who >> 32) : (uint32_t)who;  // this token's 32 lanes
                if (l == __ffs(mine) - 1) {
#pragma unroll
                    for (int j = 0; j + 1 < NP; ++j) top[j] = top[j + 1];
                    top[NP - 1] = -INFINITY;
                }
            }
        if (l == 0) {
            Tsh[i] = T;
            sel_cnt[i] = 0;
            xc_cnt[i] = 0;
        }
    }
    __syncthreads();
    {
        // pass 2, same thread -> (tokens, tiles) map: list the tiles that can hold one of the nprobe best
        const int tk4 = tid % (QLEN / 4), part = tid / (QLEN / 4);
        const float T4[4] = {Tsh[4 * tk4] - margin, Tsh[4 * tk4 + 1] - margin, Tsh[4 * tk4 + 2] - margin,
                             Tsh[4 * tk4 + 3] - margin};
        for (int b0 = part; b0 < nblk; b0 += TAIL_PARTS * TAIL_FLY) {
            float4 v[TAIL_FLY];
#pragma unroll
            for (int u = 0; u < TAIL_FLY; ++u) {
                const int b = b0 + TAIL_PARTS * u;
                v[u] = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
                if (b < nblk) v[u] = *reinterpret_cast<const float4 *>(tmq + (int64_t)b * QLEN + 4 * tk4);
            }
#pragma unroll
            for (int u = 0; u < TAIL_FLY; ++u) {
                const int b = b0 + TAIL_PARTS * u;
                const float x[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    if (b < nblk && x[c] >= T4[c]) {
                        const int pos = atomicAdd(&sel_cnt[4 * tk4 + c], 1);
                        if (pos < TAIL_SEL) sel_tile[4 * tk4 + c][pos] = b;
                    }
            }
        }
    }
    __syncthreads();
    {
        uint64_t best[NP];
#pragma unroll
        for (int j = 0; j < NP; ++j) best[j] = PLAID_KEY_MAX;
        const float T = Tsh[i] - margin;
        const int n_sel = sel_cnt[i];
        const bool listed = n_sel <= TAIL_SEL;
        const int chunks = (tile_rows + TAIL_LANES - 1) / TAIL_LANES;  // 32-row pieces of a tile
        const int n_items = (listed ? n_sel : nblk) * chunks;
        // walk: every listed row with its score; what happens to a row is up to `visit`
        auto walk = [&](auto visit) {
            for (int it0 = 0; it0 < n_items; it0 += 4) {
                float sv[4];
                int64_t cc[4];
                bool ok[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int it = it0 + u;
                    ok[u] = it < n_items;
                    const int k = ok[u] ? it / chunks : 0, r = (it % chunks) * TAIL_LANES + l;
                    const int t = listed ? sel_tile[i][k] : k;
                    if (!listed && ok[u]) ok[u] = tmq[(int64_t)t * QLEN + i] >= T;
                    cc[u] = (int64_t)t * tile_rows + r;
                    ok[u] = ok[u] && r < tile_rows && cc[u] < C;
                    // (no stored scores: nearest-centroid assignment keeps only the tile maxima, and every row of a listed
                    // tile counts as a row that may be among the best)
                    sv[u] = ok[u] ? (S ? Sq[cc[u] * QLEN + i] : INFINITY) : 0.f;
                }
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    if (ok[u]) visit(sv[u], cc[u]);
            }
        };
        if (!APPROX) {
            walk([&](float sv, int64_t cc) { scq_insert_key<NP>(best, plaid_make_key(sv, (uint32_t)cc)); });
        } else {
            // Only a row that can be among the nprobe best (score >= T - 2 eps) is ranked, and by its exact score.  The
            // rows are listed first and re-evaluated one per lane, all at once; a token with more such rows than lanes
            // (many equal scores) re-evaluates them as it meets them.
            walk([&](float sv, int64_t cc) {
                if (sv >= T) {
                    const int pos = atomicAdd(&xc_cnt[i], 1);
                    if (pos < TAIL_XCAP) xc_id[i][pos] = (int32_t)cc;
                }
            });
            __syncthreads();
            const int n_x = xc_cnt[i];
            if (n_x <= TAIL_XCAP) {
                if (l < n_x) {
                    const int32_t c = xc_id[i][l];
                    best[0] = plaid_make_key(scq_exact_entry(x.Cm + (int64_t)c * DIM, Qq + i * DIM), (uint32_t)c);
                }
            } else {
                walk([&](float sv, int64_t cc) {
                    if (sv >= T) scq_insert_key<NP>(best, plaid_make_key(scq_exact_entry(x.Cm + cc * DIM, Qq + i * DIM), (uint32_t)cc));
                });
            }
        }
        // shuffle tree over the 32 lanes of this token (lanes l and l ^ d exchange lists; both keep the merged list)
#pragma unroll
        for (int d = 1; d < TAIL_LANES; d <<= 1) {
            uint64_t other[NP];
#pragma unroll
            for (int j = 0; j < NP; ++j) other[j] = __shfl_xor(best[j], d);
#pragma unroll
            for (int j = 0; j < NP; ++j) scq_insert_key<NP>(best, other[j]);
        }
        if (l == 0) {
#pragma unroll
            for (int j = 0; j < NP; ++j)
                if (j < nprobe) {
                    // A list entry can only be missing when the scores are not numbers (a query holding NaN compares
                    // false against every threshold): later kernels index the inverted lists with these ids, so such a
                    // slot gets centroid j (nprobe <= C), never an id out of range.
                    const int32_t id = best[j] == PLAID_KEY_MAX ? j : (int32_t)(best[j] & 0xFFFFFFFFu);
                    o.probed[((int64_t)q * QLEN + i) * nprobe + j] = id;
                    idl[i * nprobe + j] = id;
                }
            top1[i] = best[0] == PLAID_KEY_MAX ? 0 : (int32_t)(best[0] & 0xFFFFFFFFu);
        }
    }
    __syncthreads();
    // ascending duplicate-free union of the n = 32 * nprobe (<= 256) probed ids by counting: an id is kept at its first
    // occurrence, at position = number of distinct smaller ids.  Four lanes share the n comparisons of one id.
    {
        const int n = QLEN * nprobe;
        const int t = tid >> 2, part = tid & 3;
        const int32_t id = t < n ? idl[t] : 0x7FFFFFFF;
        int earlier_same = 0;
        for (int u = part; u < n; u += 4) earlier_same += (idl[u] == id && u < t) ? 1 : 0;
        earlier_same += __shfl_xor(earlier_same, 1);
        earlier_same += __shfl_xor(earlier_same, 2);
        const bool fo = t < n && earlier_same == 0;
        // position = number of first occurrences with a smaller id
        __shared__ int32_t first[256];
        if (part == 0 && t < n) first[t] = fo ? 1 : 0;
        __syncthreads();
        int pos = 0;
        for (int u = part; u < n; u += 4) pos += (first[u] && idl[u] < id) ? 1 : 0;
        pos += __shfl_xor(pos, 1);
        pos += __shfl_xor(pos, 2);
        if (fo && part == 0) o.uniq[(int64_t)q * o.uniq_stride + pos] = id;
        const int total = __syncthreads_count(fo && part == 0);
        if (tid == 0) o.n_uniq[q] = total;
    }
    if (APPROX) {
        // Eq. 5 for the rows the score kernel left open.  Rounds of at most TAIL_AMB rows: the rows of a range of bitmap
        // words are listed in LDS, then their 32 entries each are spread over the workgroup.  (One round, a handful of
        // rows, unless the threshold sits where many row maxima do.)
        __shared__ int32_t amb_rows[TAIL_AMB];
        __shared__ int32_t amb_n, amb_total;
        uint32_t *kbq = keepbits + (int64_t)q * keep_words;
        const uint32_t *abq = x.ambbits + (int64_t)q * keep_words;
        if (tid == 0) amb_total = 0;
        __syncthreads();
        {
            int cnt = 0;
            for (int64_t w = tid; w < keep_words; w += TAIL_THREADS) cnt += __popc(abq[w]);
            if (cnt) atomicAdd(&amb_total, cnt);
        }
        __syncthreads();
        const int total = amb_total;  // uniform
        // words taken per round: all of them when every open row fits the list (the usual case: one round), else as
        // many as always fit
        const int64_t round_words = total <= TAIL_AMB ? keep_words : TAIL_AMB / 32;
        for (int64_t w0 = 0; total > 0 && w0 < keep_words; w0 += round_words) {
            __syncthreads();
            if (tid == 0) amb_n = 0;
            __syncthreads();
            const int64_t w1 = w0 + round_words < keep_words ? w0 + round_words : keep_words;
            for (int64_t w = w0 + tid; w < w1; w += TAIL_THREADS) {
                uint32_t v = abq[w];
                while (v) {
                    const int b = __ffs(v) - 1;
                    v &= v - 1;
                    amb_rows[atomicAdd(&amb_n, 1)] = (int32_t)(w * 32 + b);
                }
            }
            __syncthreads();
            const int n_amb = amb_n;
            for (int p = tid; p < n_amb * QLEN; p += TAIL_THREADS) {
                const int64_t c = amb_rows[p >> 5];
                const int tok = p & 31;
                if ((!S || Sq[c * QLEN + tok] >= x.t_lo) && scq_exact_entry(x.Cm + c * DIM, Qq + tok * DIM) >= x.t_cs)
                    atomicOr(&kbq[c >> 5], 1u << (c & 31));
            }
        }
        // The updates of the pruning words above are atomics, performed in the second-level cache, and the table below
        // reads the words there too (atomic loads): the barrier's wait for this wave's outstanding memory operations is
        // all the ordering the two need.
        __syncthreads();
    }
    stage1_survivor_table<APPROX>(S + (int64_t)q * C * QLEN, C, keepbits + (int64_t)q * keep_words, keep_words, top1,
                                  o.meta + q, o.kept_ids + (int64_t)q * S2_MAX_KEPT,
                                  o.T + (int64_t)q * (S2_MAX_KEPT + 1) * QLEN, scan, ids, trial, colmm, misc, x.Cm, Qq,
                                  o.ivf_offsets, q, o.qcount, o.qlist, o.qlist_stride);
}

// np = capacity of the tail's lists (1, 2, 4 or 8 >= nprobe); np = 0: scores and pruning bits only (large nprobe).
static void launch_fused(hipStream_t st, int phases, int np, const float *centroids, int64_t C, const float *Q, const void *Qx,
                         int form, const void *A16, int nq, float t_cs, float *S, uint32_t *keepbits, uint32_t *ambbits,
                         int64_t keep_words, float *tilemax, int nprobe, const Stage1Out &o, uint32_t *zero, int64_t zero_words,
                         unsigned long long *score_clocks)
{
    const bool matrix_form = form == PLAID_SCQ_MATRIX;
    const int tile_rows = form == PLAID_SCQ_VECTOR ? SCQ_ROWS : SM_WROWS;  // rows per tile of column maxima
    const int grid_rows = matrix_form ? SM_ROWS : SCQ_ROWS;   // rows per workgroup (the two double-precision forms)
    const unsigned nblk = (unsigned)((C + grid_rows - 1) / grid_rows);
    const int n_tiles = (int)((C + tile_rows - 1) / tile_rows);
    float *tmx = np > 0 ? tilemax : nullptr;
    static_assert(SM_WROWS == 32, "the split-fp16 kernel emits column maxima per 32 rows, like the matrix form");
    if (!(phases & PLAID_STAGE1_SCORES)) {
    } else if (form == PLAID_SCQ_SPLIT16) {
        plaid_launch_scq16(st, A16, C, Qx, nq, t_cs, S, keepbits, ambbits, keep_words, tmx, score_clocks);
    } else if (matrix_form) {
        if (nq == 1)
            hipLaunchKernelGGL(scq_mfma_kernel<1>, dim3(1, nblk), dim3(SM_THREADS), 0, st, centroids, C, Q, nq, t_cs, S, keepbits,
                               keep_words, tmx, zero, zero_words);
        else
            hipLaunchKernelGGL(scq_mfma_kernel<2>, dim3((unsigned)((nq + 1) / 2), nblk), dim3(SM_THREADS), 0, st, centroids, C, Q,
                               nq, t_cs, S, keepbits, keep_words, tmx, zero, zero_words);
    } else {
        hipLaunchKernelGGL(scq_fused_kernel, dim3(nblk, nq), dim3(SCQ_THREADS), 0, st, centroids, C, (const double *)Qx, t_cs, S,
                           keepbits, keep_words, tmx);
    }
    if (np > 0 && (phases & PLAID_STAGE1_PROBES)) {
        Stage1Exact x;
        x.Cm = centroids;
        x.Q = Q;
        x.ambbits = ambbits;
        x.t_cs = t_cs;
        x.t_lo = (t_cs > -INFINITY && t_cs < INFINITY) ? nextafterf(t_cs - PLAID_SCQ16_EPS, -INFINITY) : t_cs;
        x.margin = 2.0f * PLAID_SCQ16_EPS;
#define TAIL(NP_, AP_)                                                                                                     \
    hipLaunchKernelGGL((stage1_tail_kernel<NP_, AP_>), dim3(nq), dim3(TAIL_THREADS), 0, st, S, C, keepbits, keep_words,     \
                       tilemax, n_tiles, tile_rows, nprobe, o, x)
        if (form == PLAID_SCQ_SPLIT16) {
            if (np == 1) TAIL(1, true);
            else if (np == 2) TAIL(2, true);
            else if (np == 4) TAIL(4, true);
            else TAIL(8, true);
        } else {
            if (np == 1) TAIL(1, false);
            else if (np == 2) TAIL(2, false);
            else if (np == 4) TAIL(4, false);
            else TAIL(8, false);
        }
#undef TAIL
    }
}

size_t plaid_stage1_tilemax_bytes(int64_t C, int nq, int nprobe)
{
    if (nprobe > PLAID_PROBE_FAST_MAX) return 256;
    const int rows = SM_WROWS < SCQ_ROWS ? SM_WROWS : SCQ_ROWS;  // sized for the smaller of the two tile heights
    return (size_t)nq * ((C + rows - 1) / rows) * QLEN * 4;
}

void plaid_launch_stage1(hipStream_t st, int phases, const float *centroids, int64_t C, const float *Q, void *Qd, int form,
                         const void *A16, int nq, float t_cs, int nprobe, float *S, uint32_t *keepbits, uint32_t *ambbits,
                         int64_t keep_words, float *tilemax, uint32_t *zero, int64_t zero_words, int32_t *probed,
                         int32_t *uniq, int uniq_stride, int32_t *n_uniq, const Stage2Buffers &s2, void *probe_scratch,
                         size_t probe_scratch_bytes, unsigned long long *score_clocks)
{
    if ((phases & PLAID_STAGE1_PREP) && form == PLAID_SCQ_SPLIT16) plaid_launch_scq16_split_queries(st, Q, nq, Qd, zero, zero_words);
    if ((phases & PLAID_STAGE1_PREP) && form == PLAID_SCQ_VECTOR) {
        int64_t gz = (zero_words + 256 * 8 - 1) / (256 * 8);
        if (gz < nq) gz = nq;
        if (gz > 1024) gz = 1024;
        hipLaunchKernelGGL(stage1_prep_kernel, dim3((unsigned)gz), dim3(256), 0, st, Q, (double *)Qd, nq, zero, zero_words);
    }
    if (!(phases & (PLAID_STAGE1_SCORES | PLAID_STAGE1_PROBES))) return;
    Stage1Out o;
    o.probed = probed;
    o.uniq = uniq;
    o.n_uniq = n_uniq;
    o.uniq_stride = uniq_stride;
    o.meta = s2.meta;
    o.kept_ids = s2.kept_ids;
    o.T = s2.T;
    o.ivf_offsets = s2.ivf_offsets;
    o.qcount = s2.qcount;
    o.qlist = s2.qlist;
    o.qlist_stride = s2.qlist_stride;
    const int np = nprobe == 1 ? 1 : (nprobe == 2 ? 2 : (nprobe <= 4 ? 4 : (nprobe <= PLAID_PROBE_FAST_MAX ? 8 : 0)));
    if (np > 0)
        launch_fused(st, phases, np, centroids, C, Q, Qd, form, A16, nq, t_cs, S, keepbits, ambbits, keep_words, tilemax, nprobe,
                     o, zero, zero_words, score_clocks);
    else {
        // large nprobe: scores and pruning bits here, probes through the generic selection, survivor table after it
        launch_fused(st, phases, 0, centroids, C, Q, Qd, form, A16, nq, t_cs, S, keepbits, ambbits, keep_words, tilemax, nprobe,
                     o, zero, zero_words, score_clocks);
        if (phases & PLAID_STAGE1_PROBES) {
            plaid_launch_top_nprobe_general(st, S, C, nq, nprobe, probed, uniq, uniq_stride, n_uniq, probe_scratch,
                                            probe_scratch_bytes);
            hipLaunchKernelGGL(stage1_survivor_kernel, dim3(nq), dim3(512), 0, st, S, C, keepbits, keep_words, probed, nprobe, o);
        }
    }
}
