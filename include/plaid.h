/*
 * plaid.h -- C ABI of the MI355X (gfx950) PLAID search library.
 *
 * The library runs the search pipeline of "PLAID: An Efficient Engine for Late Interaction
 * Retrieval" (Figure 4, Sections 4.1-4.5) for one or more queries on ONE GPU:
 *
 *   stage 1  S_cq = C . Q^T (Eq. 2); per query token the nprobe best centroids; candidate
 *            passages = union of the probed centroids' inverted lists (Section 4.1, no size cap);
 *   stage 2  centroid interaction (Eq. 3-4) over all candidates using only tokens whose centroid
 *            passes the pruning test max_i S_cq[c][i] >= t_cs (Eq. 5); keep the best ndocs;
 *   stage 3  centroid interaction without pruning over those; keep the best max(1, ndocs/4)
 *            (Figure 4, Section 4.3);
 *   stage 4  decompress the residuals of those passages through the byte lookup table
 *            (Section 4.5), exact MaxSim (Eq. 1), best k (Section 4.4).
 *
 * Readings where the paper is silent: rankings are by (score descending, id ascending); a passage
 * with no surviving token in stage 2 scores -infinity and still fills the ndocs slots in pid
 * order; reconstructed vectors are centroid + bucket weight with no renormalisation; packed
 * bucket indices are stored most-significant first (dimension order preserved inside a byte).
 *
 * Conventions: every function returns PLAID_OK (0) or a negative plaid_status and never throws
 * or aborts; plaid_last_error() returns a thread-local description of the last failure.
 * Pointers marked DEVICE are HIP device pointers valid on the index's device; pointers marked
 * HOST are ordinary host pointers.  The caller owns every buffer it passes; the library owns the
 * index handle and a per-index workspace that grows on demand and is released by
 * plaid_index_free.  Searches on one index must not run concurrently.  Kernels are enqueued on
 * the caller's stream; plaid_search returns without waiting for them unless stated otherwise.
 */
#ifndef PLAID_H
#define PLAID_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PLAID_QLEN 32 /* query tokens per query   */
#define PLAID_DIM 128 /* embedding dimension      */

typedef enum {
    PLAID_OK = 0,
    PLAID_EINVAL = -1,  /* null pointer, size out of range, malformed view */
    PLAID_ENOMEM = -2,  /* host or device allocation failed                */
    PLAID_EHIP = -3,    /* a HIP runtime call failed (text in last_error)  */
    PLAID_EIO = -4,     /* file could not be opened or read                */
    PLAID_EFORMAT = -5  /* file is not a PLAID index file                  */
} plaid_status;

typedef struct plaid_index plaid_index; /* opaque */

/* Borrowed description of an index (storage format of Section 3.1: a 4-byte centroid id and a
 * 16*nbits-byte packed residual per token; inverted lists of unique passage ids, Section 4.1).
 * All arrays live on the host (on_device = 0) or all on the device (on_device = 1). */
typedef struct {
    int32_t dim;                 /* must be PLAID_DIM */
    int32_t nbits;               /* 1 or 2 bits per residual dimension */
    int64_t num_centroids;       /* C, 1 <= C < 2^31 */
    int64_t num_passages;        /* P, 1 <= P < 2^31 */
    int64_t num_embeddings;      /* N = doc_offsets[P] */
    const float *centroids;      /* [C][128] row-major fp32 */
    const int64_t *doc_offsets;  /* [P+1], doc_offsets[0] = 0, non-decreasing; tokens of passage p are
                                    doc_offsets[p] .. doc_offsets[p+1]-1 */
    const int32_t *codes;        /* [N], centroid id of each token, in [0, C) */
    const uint8_t *residuals;    /* [N][16*nbits] packed bucket indices */
    const float *bucket_weights; /* [2^nbits] */
    const int64_t *ivf_offsets;  /* [C+1], ivf_offsets[0] = 0 */
    const int32_t *ivf_pids;     /* [ivf_offsets[C]], ascending unique pids per centroid */
    int32_t on_device;
} plaid_index_view;

/* Optional per-stage outputs of plaid_search_debug.  Every pointer is DEVICE, caller-owned, and may be
 * NULL (that output is skipped).  nq is the number of queries of the call. */
typedef struct {
    float *S_cq;          /* [nq][C][32]  Eq. 2 scores, row c = centroid c (the score kernel's values: see
                             plaid_get_score_kernel for how close to the definition's they are) */
    int32_t *probed;      /* [nq][32][nprobe]  per query token, best first (Section 4.1) */
    int32_t *cand;        /* [nq][P]  ascending candidate pids, first n_cand[q] valid */
    int32_t *n_cand;      /* [nq] */
    int32_t *sel2_ids;    /* [nq][ndocs]  stage-2 survivors, unspecified order, first n2[q] valid */
    float *sel2_scores;   /* [nq][ndocs]  their pruned centroid-interaction scores (Eq. 3-5) */
    int32_t *n2;          /* [nq]  = min(ndocs, n_cand) */
    int32_t *sel3_ids;    /* [nq][max(1,ndocs/4)]  stage-3 survivors, unspecified order */
    float *sel3_scores;   /* [nq][max(1,ndocs/4)]  their unpruned centroid-interaction scores (Eq. 3-4) */
    int32_t *n3;          /* [nq]  = min(max(1,ndocs/4), n2) */
    uint32_t *keep;       /* [nq][ceil(C/32)]  pruning map of Eq. 5: bit c%32 of word c/32 = centroid c is kept */
} plaid_debug_buffers;

/* Read an index file and upload it to `device` (a HIP device ordinal).  File layout, little-endian:
 * bytes 0-7 "PLAIDIX1"; int32 dim, int32 nbits, int64 C, P, N, ivf_len; zero padding to byte 64; then
 * centroids, doc_offsets, codes, residuals, bucket_weights, ivf_offsets, ivf_pids in the types of
 * plaid_index_view, each section starting at a multiple of 64 bytes.  On success *out is a new handle.
 * Errors: PLAID_EINVAL, PLAID_EIO, PLAID_EFORMAT, PLAID_ENOMEM, PLAID_EHIP. */
int plaid_index_load(const char *path, int device, plaid_index **out);

/* Build a handle from caller memory.  copy = 1: the arrays (host or device) are copied into
 * library-owned device memory.  copy = 0: requires on_device = 1; the library keeps the caller's device
 * pointers (centroids, codes and residuals must then be aligned to 16 bytes, else PLAID_EINVAL) and the caller
 * must keep them alive and unchanged until plaid_index_free.  The arrays are validated either way (offsets monotone
 * from 0 to their end, codes in [0, C), passage ids in [0, P) and strictly ascending within each list): on the host for
 * host arrays, by one kernel for device arrays; a violation is PLAID_EINVAL and nothing is searched. */
int plaid_index_from_view(const plaid_index_view *view, int device, int copy, plaid_index **out);

/* Release the handle, its workspace and any memory the library allocated for it.  NULL is allowed. */
void plaid_index_free(plaid_index *idx);

/* Search nq queries (Figure 4 pipeline, stages as listed at the top of this file).
 *   Q           DEVICE  [nq][32][128] fp32 query token embeddings (unit norm expected, not checked), 16-byte aligned
 *   nprobe      centroids probed per query token, 1 <= nprobe <= C
 *   t_cs        pruning threshold of Eq. 5; -INFINITY disables pruning, +INFINITY prunes everything
 *   ndocs       passages kept by stage 2 (>= 1); stage 3 keeps max(1, ndocs/4)
 *   k           results per query (>= 1)
 *   out_ids     DEVICE  [nq][k] passage ids, best first; unused slots -1
 *   out_scores  DEVICE  [nq][k] MaxSim scores (Eq. 1) of the reconstructed passages; unused slots -INFINITY
 *   hip_stream  a hipStream_t (NULL = the default stream); the call is asynchronous on it
 * Errors: PLAID_EINVAL for null pointers or out-of-range sizes, PLAID_ENOMEM when the workspace cannot be
 * allocated, PLAID_EHIP for launch failures. */
int plaid_search(plaid_index *idx, const float *Q, int32_t nq, int32_t nprobe, float t_cs, int32_t ndocs,
                 int32_t k, int32_t *out_ids, float *out_scores, void *hip_stream);

/* plaid_search that also copies the intermediates named in *dbg out of the workspace (same kernels, same
 * results).  dbg = NULL behaves like plaid_search. */
int plaid_search_debug(plaid_index *idx, const float *Q, int32_t nq, int32_t nprobe, float t_cs, int32_t ndocs,
                       int32_t k, int32_t *out_ids, float *out_scores, void *hip_stream,
                       const plaid_debug_buffers *dbg);

/* plaid_search for callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): same arguments, same kernels and bit-identical results, but the workspace is a
 * 64 MiB array inside the library (one copy per device, held until the process ends) instead of memory the library
 * allocates, so the call performs no hipMalloc / hipFree and no other allocating call.  Batches are processed in
 * chunks that fit the array; PLAID_EINVAL when even one query does not fit (plaid_workspace_bytes with nq = 1 tells:
 * about 132 C + 16 P bytes).  Every call on a device uses that device's one array, which keeps the previous call's
 * contents (what must start at zero is cleared by the first kernel of each chunk): calls that overlap on one device
 * race, whichever index they use.  Stage timing and debug outputs are not available through this entry point. */
int plaid_search_static(plaid_index *idx, const float *Q, int32_t nq, int32_t nprobe, float t_cs, int32_t ndocs,
                        int32_t k, int32_t *out_ids, float *out_scores, void *hip_stream);

/* Vanilla ColBERTv2 retrieval, the baseline the paper measures PLAID against (Sections 3.1-3.2, 4.1), on the same index
 * and with the same kernels for Eq. 2, decompression and MaxSim:
 *   1. S_cq and the nprobe best centroids of every query token, as in plaid_search;
 *   2. the inverted list of a centroid holds the ids of the EMBEDDINGS assigned to it; the candidates are the passages
 *      owning an embedding of a probed list (the library builds these lists and a token -> passage map on the first
 *      call: 8 bytes per embedding, kept until plaid_index_free; fewer than 2^31 embeddings);
 *   3. when a query has more than ncandidates candidates they are pruned by scoring the embeddings of the probed lists
 *      -- only those -- with full residual decompression: score = sum over the query tokens of the maximum over the
 *      passage's embeddings among them, the best ncandidates by (score descending, pid ascending) stay;
 *   4. every token of every remaining candidate is decompressed and scored exactly (Eq. 1); the best k are returned
 *      like plaid_search returns them.
 * dbg may be NULL; its pointers are DEVICE, caller-owned and may each be NULL:
 *   cand [nq][P] ascending candidate pids, n_cand [nq];  kept_ids / kept_scores [nq][ncandidates] the candidates after
 *   step 3 in unspecified order with their pruning scores (0 for a query that needed no pruning), n_kept [nq].
 * The first call synchronises the device.  Errors as plaid_search. */
typedef struct {
    int32_t *cand;
    int32_t *n_cand;
    int32_t *kept_ids;
    float *kept_scores;
    int32_t *n_kept;
} plaid_vanilla_debug;
int plaid_search_vanilla(plaid_index *idx, const float *Q, int32_t nq, int32_t nprobe, int32_t ncandidates, int32_t k,
                         int32_t *out_ids, float *out_scores, void *hip_stream, const plaid_vanilla_debug *dbg);

/* Decompress the tokens of n listed passages (Section 4.5: packed byte -> bucket indices through the
 * 256-entry table, value = centroid + bucket weight, one fp32 addition per element).
 *   pids         DEVICE [n] passage ids
 *   out_offsets  DEVICE [n+1] receives the exclusive prefix sum of the passages' token counts (may be NULL)
 *   out_vectors  DEVICE [total][128] fp32 reconstructed vectors, passages concatenated in list order (may be NULL)
 *   out_indices  DEVICE [total][128] uint8 unpacked bucket indices (may be NULL)
 *   capacity     rows available in out_vectors / out_indices; PLAID_EINVAL if total exceeds it
 * Synchronises the stream once (the total is read back to check the capacity). */
int plaid_decompress_passages(plaid_index *idx, const int32_t *pids, int32_t n, int64_t *out_offsets,
                              float *out_vectors, uint8_t *out_indices, int64_t capacity, void *hip_stream);

/* Sizes of a loaded index: any pointer may be NULL. */
int plaid_index_info(const plaid_index *idx, int64_t *num_centroids, int64_t *num_passages,
                     int64_t *num_embeddings, int32_t *nbits, int64_t *ivf_len);

/* Which kernel computes S_cq (Eq. 2) for this index: HOST *form =
 *   2  the half-precision matrix instruction on operands split into two fp16 terms each (the default).  Scores are
 *      within 2^-15 of the exact dot products for vectors of norm <= 1 whose components lie in fp16's range (observed:
 *      a few 1e-7); every decision taken on them -- probed centroids (Section 4.1), the pruning map (Eq. 5) -- is
 *      completed in double wherever that bound leaves it open, and the rows of the surviving centroids that stage 2
 *      scores with are re-evaluated in double, so probes, candidates, the pruning map and the stage-2 scores of
 *      queries with at most 63 surviving centroids are those of forms 0 and 1; stage-3 and final scores inherit the
 *      bound (32 entries per score).  Serves nprobe <= 8; a search with a larger nprobe runs form 1 (or 0).  Needs
 *      centroid components below 32 in magnitude: an index whose table exceeds that is given form 1 (or 0) instead.
 *   1  the double-precision matrix instruction, 0  a vector fused-multiply-add chain: both accumulate each score in
 *      double over the dimensions in index order and round once, the definition's bits.  Form 1 is used only when a
 *      check run on the device at the first index creation of the process confirms that the instruction adds its
 *      products in that order.
 * The environment variable PLAID_SCQ_FORM=vector|matrix|split16 (read at index creation) overrides the choice (matrix is
 * an error when the check fails). */
int plaid_get_score_kernel(const plaid_index *idx, int32_t *form);

/* How candidates and their pruned scores (Section 4.1, Eq. 3-5) are computed for this index: HOST *form = 1 or 2 for
 * the inverted form (a passage holds centroid c exactly when c's inverted list holds the passage, so the candidate set
 * and every pruned bag follow from the lists of the probed and the surviving centroids), 0 for the union of the probed
 * lists followed by a stream over the candidates' token codes.  Same results either way.  The inverted form needs a
 * table of num_centroids x (num_passages / R + 1) 32-bit positions, R = 2048 passages per workgroup (form 1) or 8192
 * (form 2), built at index creation with the smaller R whose table is at most 32 MiB or at most four times the size of
 * the inverted lists (device memory of the library's own, beside the index);
 * PLAID_STAGE2_FORM=stream|inverted|inverted11|inverted13 (read at index creation) overrides. */
int plaid_get_stage2_kernel(const plaid_index *idx, int32_t *form);

/* Per-stage GPU time of the most recent plaid_search on this index when stage timing is on
 * (plaid_set_stage_timing(idx, 1)): HOST out_ms[PLAID_NUM_STAGES], summed over the call's query chunks.
 * Turning timing on makes every search synchronise at its end. */
#define PLAID_NUM_STAGES 10
/* stage order: 0 workspace clearing + query layout, 1 S_cq + pruning map (Eq. 2, 5), 2 top-nprobe, probe union and
 * table of surviving centroids, 3 candidate union (Section 4.1), 4 stage-2 interaction (Eq. 3-5), 5 select ndocs,
 * 6 stage-3 interaction (Eq. 3-4), 7 select ndocs/4, 8 stage-4 decompress + MaxSim (Section 4.5, Eq. 1), 9 top-k */
int plaid_set_stage_timing(plaid_index *idx, int32_t on);
int plaid_get_stage_ms(const plaid_index *idx, float *out_ms);

/* The clock the chip held while the S_cq kernel (Eq. 2; score kernel 2 of plaid_get_score_kernel only) of the most
 * recent plaid_search with stage timing on was running: HOST out_ticks[2] = how far the shader-clock counter
 * (out_ticks[0]) and the fixed-rate 100 MHz timer (out_ticks[1]) moved, each summed over the kernel's workgroups;
 * 100 * out_ticks[0] / out_ticks[1] is the shader clock in MHz.  Both are 0 when nothing was measured.  Synchronises
 * the device.  A diagnostic, like the stage times: the published peak rates assume the chip's top clock. */
int plaid_get_score_kernel_clocks(const plaid_index *idx, uint64_t *out_ticks);

/* Storage variant (Section 4.5 reconstructs the stored embedding and is silent on its length; the embeddings that were
 * stored have unit length, Section 3.1, the reconstruction centroid + residual does not): on != 0 makes every later
 * plaid_search / plaid_search_debug / plaid_search_static on this index score, and plaid_decompress_passages return,
 * reconstructed vectors scaled back to unit length: each token's vector is multiplied by
 * fl32(1 / sqrt(sum of the squares of its fp32 components, added in double in index order)) (0 for a zero vector).
 * The first call with on != 0 computes that factor for every token (num_embeddings floats of device memory owned by the
 * index; the call synchronises the device's default stream); on = 0 switches back.  Stages 1-3 use centroids only and
 * do not change.  Not to be called while a search on this index is in flight.  plaid_search_vanilla returns
 * PLAID_EINVAL while the variant is on.  Errors: PLAID_EINVAL (null index), PLAID_ENOMEM, PLAID_EHIP. */
int plaid_index_set_renormalize(plaid_index *idx, int32_t on);

/* Limit on queries processed per internal chunk (0 = library default).  Affects workspace size only. */
int plaid_set_max_chunk(plaid_index *idx, int32_t max_queries_per_chunk);

/* Bytes of device workspace a plaid_search with these parameters allocates (once, grown on demand, kept until
 * plaid_index_free) on an index with C centroids and P passages, and the number of queries the call processes per
 * internal chunk.  Host arithmetic only: no device is touched.  max_queries_per_chunk as for plaid_set_max_chunk
 * (0 = the library's default: up to 512 queries within about 24 GiB).  bytes: HOST, required; queries_per_chunk: HOST,
 * may be NULL.  Errors: PLAID_EINVAL. */
int plaid_workspace_bytes(int64_t C, int64_t P, int32_t nq, int32_t nprobe, int32_t ndocs, int32_t k,
                          int32_t max_queries_per_chunk, int64_t *bytes, int32_t *queries_per_chunk);

/* ---- Index construction: the step before the search path.  Every array is DEVICE memory of `device`; the calls
 * synchronise `hip_stream` before they return (sizes and error flags are read back) and allocate temporary device
 * memory, which they release. ---- */

/* Nearest centroid of each vector (Section 3.1: a token is stored with the id of its closest centroid):
 * codes[j] = the centroid with the largest dot product centroids[c] . x[j], the dot products accumulated in double over
 * the dimensions in index order and rounded once to fp32, exactly as S_cq of Eq. 2 is (the same kernel computes them,
 * 32 vectors at a time); among equal scores the smaller id wins.
 *   centroids  [C][128] fp32, 16-byte aligned     x  [n][128] fp32, 16-byte aligned     codes  [n] int32 (output)
 * Errors: PLAID_EINVAL (null or misaligned pointers, sizes out of range), PLAID_ENOMEM, PLAID_EHIP. */
int plaid_assign_centroids(const float *centroids, int64_t C, const float *x, int64_t n, int32_t *codes, int device,
                           void *hip_stream);

/* Residual encoding (Section 3.1; the inverse of the byte table of Section 4.5): per dimension r = x - centroid (one
 * fp32 subtraction), bucket = the number of cut-offs strictly below r, and 8 / nbits bucket indices per byte, the first
 * dimension in the most significant bits.
 *   cutoffs    [2^nbits - 1] fp32 ascending        codes  [n] in [0, C)
 *   residuals  [n][16 * nbits] uint8 (output), 4-byte aligned
 * Errors: PLAID_EINVAL (also when a code is outside [0, C): nothing is read out of bounds), PLAID_ENOMEM, PLAID_EHIP. */
int plaid_encode_residuals(const float *centroids, int64_t C, const float *x, const int32_t *codes, int64_t n,
                           const float *cutoffs, int32_t nbits, uint8_t *residuals, int device, void *hip_stream);

/* Passage-level inverted lists (Section 4.1): list c = the ascending unique ids of the passages with a token coded c.
 *   codes        [N] in [0, C)            doc_offsets  [P+1], from 0 to N, non-decreasing
 *   ivf_offsets  [C+1] int64 (output)     ivf_pids     [capacity] int32 (output; NULL: offsets and length only)
 *   ivf_len      HOST, receives ivf_offsets[C] (may be NULL)
 * Errors: PLAID_EINVAL (malformed offsets, a code out of range, capacity below the length), PLAID_ENOMEM, PLAID_EHIP. */
int plaid_build_ivf(const int32_t *codes, const int64_t *doc_offsets, int64_t P, int64_t N, int64_t C, int64_t *ivf_offsets,
                    int32_t *ivf_pids, int64_t capacity, int64_t *ivf_len, int device, void *hip_stream);

/* Thread-local message describing the most recent error on the calling thread ("" if none). */
const char *plaid_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* PLAID_H */
