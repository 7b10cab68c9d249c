// Internal declarations shared by the HIP translation units of libplaid (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "plaid.h"

#define QLEN PLAID_QLEN
#define DIM PLAID_DIM

// ---------------------------------------------------------------------------------------------
// Ranking keys.  Every top-n of the pipeline ranks by (score descending, id ascending).  A 64-bit
// key whose ASCENDING order is that ranking: high word = bitwise complement of the usual
// order-preserving map of the fp32 score, low word = id.  Keys are unique because ids are.
// ---------------------------------------------------------------------------------------------
__host__ __device__ __forceinline__ uint32_t plaid_score_to_ord(float s)
{
    s += 0.0f;  // -0 -> +0 so that the two zeros tie
    union { float f; uint32_t u; } c;
    c.f = s;
    uint32_t u = c.u;
    u ^= (u >> 31) ? 0xFFFFFFFFu : 0x80000000u;  // larger score -> larger u
    return ~u;                                   // larger score -> smaller key
}
__host__ __device__ __forceinline__ float plaid_ord_to_score(uint32_t k)
{
    uint32_t u = ~k;
    u ^= (u >> 31) ? 0x80000000u : 0xFFFFFFFFu;
    union { float f; uint32_t u; } c;
    c.u = u;
    return c.f;
}
__host__ __device__ __forceinline__ uint64_t plaid_make_key(float score, uint32_t id)
{
    return ((uint64_t)plaid_score_to_ord(score) << 32) | id;
}
#define PLAID_KEY_MAX 0xFFFFFFFFFFFFFFFFull

// Sum over the 32 query tokens of Eq. 4: lane i (0..31) of the wave holds the column maximum of query token i; the
// values are added in double in index order, as the definition's sum reads, and rounded once.  The result is the same
// in every lane.
__device__ __forceinline__ float plaid_sum32_in_order(float m)
{
    double d = 0.0;
#pragma unroll
    for (int i = 0; i < 32; ++i) d += (double)__int_as_float(__builtin_amdgcn_readlane(__float_as_int(m), i));
    return (float)d;
}

// ---------------------------------------------------------------------------------------------
// Selection (k_select.hip): first m keys in ascending order out of per-segment lists.
// ---------------------------------------------------------------------------------------------
#define SEL_RADIX_BITS 11
#define SEL_BINS (1 << SEL_RADIX_BITS)
#define SEL_SORT_CAP 8192  // keys one block can sort in LDS

// Per-segment state of a multi-level selection (device memory, 64 bytes, zeroed before each use).
struct SelState {
    unsigned long long key_or;   // OR over the input keys   (accumulated by the producer or by sel_andor_kernel)
    unsigned long long key_nor;  // OR over their complements (AND of the keys = ~key_nor)
    int32_t n_in;       // number of input keys
    int32_t m_rem[3];   // keys still to take before level 0 / level 1 / the finishing step
    int32_t n_sure;     // keys already known to be selected
    int32_t n_list[2];  // sizes of the boundary lists after level 0 and level 1
    int32_t shift[2];   // bit position of the digit examined at level 0 / level 1
    int32_t width[2];   // its width in bits
    int32_t pad;
};
static_assert(sizeof(SelState) == 64, "SelState is a 64-byte record");

struct SelScratch {         // all device pointers, per segment strides in elements
    SelState *state;        // [nseg]                 } zeroed together before each use:
    int32_t *hist;          // [nseg][2][SEL_BINS]    } plaid_select_zero_bytes(nseg) bytes from `state`
    uint64_t *sure;         // [nseg][sure_stride]
    uint64_t *list0;        // [nseg][list_stride]   boundary list after level 0
    uint64_t *list1;        // [nseg][list_stride]   boundary list after level 1
    uint64_t *sortbuf;      // [nseg][pow2(m)] only when more than SEL_SORT_CAP sorted results are requested
    int64_t sure_stride, list_stride;
};

// keys: [nseg][key_stride]; counts[seg] valid entries (device).  n_upper / m: host upper bounds.
// out: [nseg][out_stride] receives min(m, count) keys (ascending if sorted != 0, else unspecified
// order), out_counts[seg] their number.  When state_ready != 0 the producer has already filled
// SelState::key_and / key_or / n_in for every segment.
void plaid_launch_select(hipStream_t st, const uint64_t *keys, int64_t key_stride, const int32_t *counts, int nseg,
                         int64_t n_upper, int32_t m, uint64_t *out, int64_t out_stride, int32_t *out_counts,
                         int sorted, const SelScratch &sc, int state_ready);
size_t plaid_select_scratch_bytes(int nseg, int64_t n_upper, int32_t m);
// Final ranking of short lists (n_upper <= SEL_SORT_CAP) written straight to the caller's [nseg][k] buffers.
void plaid_launch_rank_output(hipStream_t st, const uint64_t *keys, int64_t key_stride, const int32_t *counts, int nseg,
                              int64_t n_upper, int32_t k, int32_t *out_ids, float *out_scores);
size_t plaid_select_zero_bytes(int nseg);
size_t plaid_select_body_bytes(int nseg, int64_t n_upper, int32_t m);
SelScratch plaid_select_scratch_carve(void *base, int nseg, int64_t n_upper, int32_t m);
SelScratch plaid_select_scratch_carve2(void *zero_base, void *body_base, int nseg, int64_t n_upper, int32_t m);

// ---------------------------------------------------------------------------------------------
// Stage kernels
// ---------------------------------------------------------------------------------------------
// Stage 1 (k_scq.hip): clears the zero region, then S[q][c][i] (Eq. 2), the keep bitmap (Eq. 5; bit c of
// keepbits[q] = max_i S[q][c][i] >= t_cs), per query token the nprobe best centroids in rank order and their
// ascending duplicate-free union (Section 4.1), and stage 2's survivor table (s2.meta / kept_ids / T).
#define PLAID_PROBE_FAST_MAX 8  // nprobe handled by the tile-maxima kernel (stage1_tail_kernel); larger values go through the selection
// Qx: 32 KB of scratch per query for the re-laid-out queries.  matrix_form selects the score kernel built on the
// double-precision matrix instruction; plaid_scq_matrix_form_ok tells (once per process) whether that instruction
// adds its four products in index order with a rounding after each, which is what makes the two forms bit-identical.
int plaid_scq_matrix_form_ok(hipStream_t st, int *ok);  // returns a hipError_t value
// phases: which of the three steps to enqueue (the caller may time them apart): PREP = clear + query layout,
// SCORES = the score kernel (S, keep bits, column maxima of its tiles), PROBES = probes, their union and the survivor table.
#define PLAID_STAGE1_PREP 1
#define PLAID_STAGE1_SCORES 2
#define PLAID_STAGE1_PROBES 4
// form: which kernel computes the scores.  The two double-precision forms give the definition's bits; the split-fp16
// form (A16 = operand form of the centroids, ambbits = [nq][keep_words] scratch) gives scores within PLAID_SCQ16_EPS and
// the same probes, pruning bits and survivor table, completed in double where the bound leaves a decision open; it
// serves nprobe <= PLAID_PROBE_FAST_MAX only (the caller falls back to a double-precision form beyond).
#define PLAID_SCQ_VECTOR 0
#define PLAID_SCQ_MATRIX 1
#define PLAID_SCQ_SPLIT16 2
void plaid_launch_stage1(hipStream_t st, int phases, const float *centroids, int64_t C, const float *Q, void *Qx, int form,
                         const void *A16, int nq, float t_cs, int nprobe, float *S, uint32_t *keepbits, uint32_t *ambbits,
                         int64_t keep_words, float *tilemax, uint32_t *zero, int64_t zero_words, int32_t *probed,
                         int32_t *uniq, int uniq_stride, int32_t *n_uniq, const struct Stage2Buffers &s2, void *probe_scratch,
                         size_t probe_scratch_bytes, unsigned long long *score_clocks = nullptr);
size_t plaid_stage1_tilemax_bytes(int64_t C, int nq, int nprobe);

// Split-fp16 form of Eq. 2 (k_scq16.hip).  S differs from the exact dot products by at most PLAID_SCQ16_EPS for
// vectors of norm <= 1 (components within fp16's range); keepbits holds the rows that pass Eq. 5 even if every entry
// were that much lower, ambbits the rows whose test the bound leaves open (decided in double by the probe kernel).
#define PLAID_SCQ16_EPS 3.0517578125e-05f  // 2^-15
// The kernel forms 2^11 a1 in fp16 on the centroid side: components must stay below this magnitude.
#define PLAID_SCQ16_CENTROID_MAX 31.0f
// max_bits[0] (zero on entry) = bit pattern of the largest |x[i]|, infinity's when a value is not a number.
void plaid_launch_scq16_max_abs(hipStream_t st, const float *x, int64_t n, uint32_t *max_bits);
size_t plaid_scq16_centroid_bytes(int64_t C);  // operand form of the centroid table, built once per index
size_t plaid_scq16_query_bytes(int nq);        // operand form of nq queries
void plaid_launch_scq16_split_centroids(hipStream_t st, const float *centroids, int64_t C, void *A16);
void plaid_launch_scq16_split_queries(hipStream_t st, const float *Q, int nq, void *B16, uint32_t *zero, int64_t zero_words);
// clocks (may be null): [0] += shader-clock ticks, [1] += 100 MHz timer ticks, both summed over the workgroups.
void plaid_launch_scq16(hipStream_t st, const void *A16, int64_t C, const void *B16, int nq, float t_cs, float *S,
                        uint32_t *keepbits, uint32_t *ambbits, int64_t keep_words, float *tilemax,
                        unsigned long long *clocks = nullptr);

// General top-nprobe (nprobe > PLAID_PROBE_FAST_MAX): ranking keys of every S column through the generic selection.
void plaid_launch_top_nprobe_general(hipStream_t st, const float *S, int64_t C, int nq, int nprobe, int32_t *probed,
                                     int32_t *uniq, int uniq_stride, int32_t *n_uniq, void *scratch, size_t scratch_bytes);
size_t plaid_top_nprobe_scratch_bytes(int64_t C, int nq, int nprobe);

// Section 4.1: candidate bitmap = union of the inverted lists of the unique probed centroids.
void plaid_launch_ivf_union(hipStream_t st, const int32_t *uniq, const int32_t *n_uniq, int uniq_stride,
                            const int64_t *ivf_offsets, const int32_t *ivf_pids, int nq, uint32_t *candbits,
                            int64_t cand_words);

// ---------------------------------------------------------------------------------------------
// Stage 2 (k_stage2.hip) and its selection (k_select.hip)
// ---------------------------------------------------------------------------------------------
#define S2_MAX_KEPT 63  // surviving centroids the streaming kernel handles (slots 1..63 of a 64-bit set)
#define S2_HASH 1024    // entries of the survivor table: direct-mapped, collision-free by choice of hash
#define S2_NHASH 24     // hash functions tried per query: h(c) = (c ^ (c >> (S2_SHIFT0 + t))) & (S2_HASH - 1)
#define S2_SHIFT0 5

struct S2Meta {        // per query
    int32_t K;         // number of centroids passing Eq. 5
    float bin_hi;      // upper bound of any non-empty passage's pruned score
    float bin_scale;   // SEL_BINS / (upper bound - lower bound), 0 when every key falls into bin 0
    int32_t hash_shift;  // hash of the streaming kernel's survivor table
};

// Per-query state of the stage-2 selection (device memory, 64 bytes, zeroed before each use).
struct Sel2State {
    unsigned long long b_or, b_nor;    // OR over the boundary keys / over their complements
    unsigned long long b_or1, b_nor1;  // the same over the list the first digit filter leaves
    int32_t n_sure;                    // keys already written to the output
    int32_t n_b;                       // boundary list after the bin filter
    int32_t m_rem;                     // keys still to take from it
    int32_t n_b1;                      // boundary list after the first digit filter (only when n_b > SEL2_DIGIT_MIN)
    int32_t m_rem1;
    int32_t shift1, width1;            // digit examined by the first digit filter
    int32_t n_b2;                      // ... after the second one (only when it is launched and n_b1 > SEL2_DIGIT_MIN)
    int32_t m_rem2;
    int32_t shift2, width2;
    int32_t pad[13];
};
static_assert(sizeof(Sel2State) == 128, "Sel2State is a 128-byte record");

// Bin of a finite pruned score: 0 for the best scores, SEL_BINS-1 for the worst.  Monotone in the score, so bins
// never contradict the ranking; producer and selection call this same function on the same inputs.
__device__ __forceinline__ int plaid_s2_bin(float score, float bin_hi, float bin_scale)
{
    float x = (bin_hi - score) * bin_scale;
    x = fminf(fmaxf(x, 0.f), (float)(SEL_BINS - 1));
    return (int)x;
}

struct Stage2Buffers {   // all device pointers, leading dimension = query of the chunk
    // zeroed before each chunk
    int32_t *hist;       // [nq][SEL_BINS]  bin histogram of the valid keys
    int32_t *hist1;      // [nq][SEL_BINS]  digit histogram of an over-long boundary list
    int32_t *hist2;      // [nq][SEL_BINS]  ... of the list the first digit filter leaves, when that is over-long too
    Sel2State *state;    // [nq]
    int32_t *qcount;     // [3] queries of the chunk with no / 1..31 / more surviving centroids (null: not recorded)
    // no initialisation needed
    int32_t *qlist;      // [3][qlist_stride] those queries, in the order their probe workgroups finished
    int qlist_stride;
    S2Meta *meta;        // [nq]
    int32_t *kept_ids;   // [nq][S2_MAX_KEPT]
    float *T;            // [nq][S2_MAX_KEPT+1][32] rows of the surviving centroids (slot 0 unused)
    uint32_t *emptybits; // [nq][cand_words] candidates whose bag is empty
    uint64_t *blist;     // [nq][P] boundary list after the bin filter
    // of the index (null when there is none: nearest-centroid assignment)
    const int64_t *ivf_offsets;  // [C + 1]: the probe kernel numbers the surviving centroids by list length
};

// Eq. 3-5 over every candidate.  The passage id of a stage-2 key is its position, so only the score half is stored:
// the 32-bit word p of query q's region of keys2 (region = key_stride 64-bit words) is the score word of candidate p
// (plaid_score_to_ord), PLAID_S2_NO_SCORE when its bag is empty; words of 32-passage groups without candidates are left
// untouched.  Also produced: the bin histogram of the scores and the bitmap of the candidates with an empty bag.
#define PLAID_S2_NO_SCORE 0xFFFFFFFFu  // (the score word of one NaN bit pattern: scores are numbers)
void plaid_launch_stage2(hipStream_t st, const float *S, int64_t C, const uint32_t *keepbits, int64_t keep_words,
                         const int32_t *probed, int nprobe, const uint32_t *candbits, int64_t cand_words, int64_t P,
                         int64_t N, const int64_t *doc_offsets, const int32_t *codes, int nq, const Stage2Buffers &b,
                         uint64_t *keys2, int64_t key_stride);

// Inverted form of candidate generation + stage 2 (k_stage2.hip): the same outputs as plaid_launch_ivf_union followed by
// plaid_launch_stage2 (candbits included, which need not be cleared beforehand), computed from the inverted lists of
// the probed and the surviving centroids.  table: plaid_ivf_range_table_bytes(C, P, shift) bytes filled once per index
// by plaid_launch_ivf_range_table.
// shift: log2 of the passages per table column = per workgroup of the inverted kernel, 11 or 13.
size_t plaid_ivf_range_table_bytes(int64_t C, int64_t P, int shift);
void plaid_launch_ivf_range_table(hipStream_t st, const int64_t *ivf_offsets, const int32_t *ivf_pids, int64_t C, int64_t P,
                                  int shift, uint32_t *table);
void plaid_launch_stage2_inverted(hipStream_t st, const int32_t *uniq, const int32_t *n_uniq, int uniq_stride,
                                  const int64_t *ivf_offsets, const int32_t *ivf_pids, const uint32_t *table, const float *S,
                                  int64_t C, const uint32_t *keepbits, int64_t keep_words, const int32_t *codes,
                                  const int64_t *doc_offsets, int64_t P, int nq, const Stage2Buffers &b, uint32_t *candbits,
                                  int64_t cand_words, uint64_t *keys2, int64_t key_stride, const int32_t *dense_id,
                                  const uint32_t *dense_bits, int shift);
// Bitmaps over the passages for the longest inverted lists (built once per index, next to the range table):
// dense_id[c] = bitmap row of centroid c or -1 (counter[0], zero before the call, returns the number of rows);
// bits: rows x words, zero before the call, words = ceil(P / 32).
void plaid_launch_ivf_dense_mark(hipStream_t st, const int64_t *ivf_offsets, int64_t C, int64_t P, int32_t *dense_id,
                                 int32_t *counter);
void plaid_launch_ivf_dense_fill(hipStream_t st, const int64_t *ivf_offsets, const int32_t *ivf_pids, int64_t C, int64_t P,
                                 const int32_t *dense_id, uint32_t *bits, int64_t words);

// ---------------------------------------------------------------------------------------------
// Index construction (k_build.hip)
// ---------------------------------------------------------------------------------------------
// residuals[j] = packed bucket indices of x[j] - centroids[codes[j]]; bad[0] is set when a code is out of range.
void plaid_launch_encode_residuals(hipStream_t st, const float *centroids, int64_t C, const float *x, const int32_t *codes,
                                   int64_t n, const float *cutoffs, int nbits, uint8_t *residuals, int32_t *bad);
// Inverted lists in two steps sharing a scratch area of plaid_ivf_lists_scratch_bytes(N, C) bytes, whose first
// plaid_ivf_lists_scratch_zero_bytes(N, C) bytes are zero on entry: offsets first (bad[0] is set when a code or an
// offset is out of range), then -- only if nothing was bad -- the passage ids.
size_t plaid_ivf_lists_scratch_bytes(int64_t N, int64_t C);
size_t plaid_ivf_lists_scratch_zero_bytes(int64_t N, int64_t C);
void plaid_launch_ivf_build_offsets(hipStream_t st, const int32_t *codes, const int64_t *doc_offsets, int64_t P, int64_t N,
                                    int64_t C, void *scratch, int64_t *ivf_offsets, int32_t *bad);
void plaid_launch_ivf_build_fill(hipStream_t st, const int32_t *codes, const int64_t *doc_offsets, int64_t P, int64_t N,
                                 int64_t C, void *scratch, const int64_t *ivf_offsets, int32_t *ivf_pids, int64_t capacity);

// Best min(m, #candidates) candidates by (score desc, pid asc): from the keys by bin filter (+ digit filter when the
// boundary bin is over-long), then from the empty candidates in pid order.  keys2 is overwritten (scratch).
void plaid_launch_select2(hipStream_t st, uint64_t *keys2, int64_t key_stride, const uint32_t *candbits, int nq, int64_t P,
                          int64_t cand_words, int32_t m, const Stage2Buffers &b, uint64_t *out, int64_t out_stride,
                          int32_t *out_counts);

// Eq. 3-4 over a key list (stage 3): out_keys[q][j] is the key of the passage of in_keys[q][j].
void plaid_launch_ci_list(hipStream_t st, const float *S, int64_t C, const int64_t *doc_offsets, const int32_t *codes,
                          int nq, const uint64_t *in_keys, int64_t in_stride, const int32_t *in_counts, int n_upper,
                          uint64_t *out_keys, int64_t out_stride);

// Section 4.5 + Eq. 1 over a key list (stage 4); S = this chunk's S_cq, whose rows supply the centroids' share.
void plaid_launch_decompress_maxsim(hipStream_t st, const float *Q, const float *S, int64_t C, const int64_t *doc_offsets,
                                    const int32_t *codes, const uint8_t *residuals, const float *bucket_weights,
                                    int nbits, int nq, const uint64_t *in_keys, int64_t in_stride,
                                    const int32_t *in_counts, int n_upper, uint64_t *out_keys, int64_t out_stride,
                                    const float *inv_norm = nullptr /* [N]: reconstructed vectors scaled to unit length */);

// Section 4.5 alone: reconstructed vectors / bucket indices of listed passages.
void plaid_launch_decompress_dump(hipStream_t st, const float *centroids, const int64_t *doc_offsets,
                                  const int32_t *codes, const uint8_t *residuals, const float *bucket_weights,
                                  int nbits, const int32_t *pids, int n, const int64_t *out_offsets, float *out_vectors,
                                  uint8_t *out_indices, const float *inv_norm = nullptr);
// inv_norm[t] = 1 / |centroid[code_t] + residual_t| (fp32, from a double-precision sum of squares), 0 for a zero vector.
void plaid_launch_token_inv_norm(hipStream_t st, const float *centroids, const int32_t *codes, const uint8_t *residuals,
                                 const float *bucket_weights, int nbits, int64_t N, float *inv_norm);
void plaid_launch_passage_offsets(hipStream_t st, const int64_t *doc_offsets, const int32_t *pids, int n,
                                  int64_t *out_offsets);

// Structural check of device-resident index arrays (k_util.hip); bad[0] (zero before the call) receives a bit per kind
// of violation: 1 doc_offsets, 2 codes, 4 ivf_offsets, 8 passage id out of range, 16 inverted list not strictly ascending.
void plaid_launch_index_validate(hipStream_t st, const int64_t *doc_offsets, int64_t P, int64_t N, const int32_t *codes,
                                 int64_t C, const int64_t *ivf_offsets, const int32_t *ivf_pids, int64_t ivf_len, int32_t *bad);

// ---------------------------------------------------------------------------------------------
// Vanilla ColBERTv2 retrieval, the paper's baseline (k_build.hip, k_vanilla.hip, k_stage4.hip)
// ---------------------------------------------------------------------------------------------
// Embedding-level inverted lists: offsets [C+1], eids [N] = ascending token indices per centroid (N < 2^31);
// scratch: plaid_embedding_lists_scratch_bytes(N, C) bytes, zero on entry; bad[0] is set when a code is out of range.
size_t plaid_embedding_lists_scratch_bytes(int64_t N, int64_t C);
void plaid_launch_embedding_lists(hipStream_t st, const int32_t *codes, int64_t N, int64_t C, void *scratch, int64_t *offsets,
                                  int32_t *eids, int32_t *bad);
void plaid_launch_tok2pid(hipStream_t st, const int64_t *doc_offsets, int64_t P, int64_t N, int32_t *tok2pid);
// probebits (zero on entry) = bitmap of each query's probed centroids; candbits (zero on entry) |= the passages that own
// an embedding of those centroids' embedding lists.
void plaid_launch_vanilla_candidates(hipStream_t st, const int32_t *uniq, const int32_t *n_uniq, int uniq_stride,
                                     const int64_t *eoff, const int32_t *eids, const int32_t *tok2pid, int nq, int64_t keep_words,
                                     uint32_t *probebits, uint32_t *candbits, int64_t cand_words);
// out_keys[q][j] = key of candidate cand[q][j] scored on the embeddings of the probed lists alone (score 0 for every
// candidate of a query with at most ncandidates of them).
void plaid_launch_vanilla_prune(hipStream_t st, const float *Q, const float *S, int64_t C, const int64_t *doc_offsets,
                                const int32_t *codes, const uint8_t *residuals, const float *bucket_weights, int nbits,
                                const uint32_t *probebits, int64_t keep_words, int nq, const int32_t *cand, int64_t cand_stride,
                                const int32_t *n_cand, int64_t n_upper, int32_t ncandidates, uint64_t *out_keys,
                                int64_t out_stride);

// Small utilities
void plaid_launch_fill_u32(hipStream_t st, uint32_t *p, int64_t n, uint32_t v);
void plaid_launch_keys_to_output(hipStream_t st, const uint64_t *keys, int64_t key_stride, const int32_t *counts, int nq,
                                 int32_t k, int32_t *out_ids, float *out_scores);
void plaid_launch_keys_to_pairs(hipStream_t st, const uint64_t *keys, int64_t key_stride, const int32_t *counts, int nq,
                                int32_t cap, int32_t *out_ids, float *out_scores, int32_t *out_counts);
void plaid_launch_bitmap_to_list(hipStream_t st, const uint32_t *bits, int64_t words, int64_t nbits_valid, int nq,
                                 int32_t *out, int64_t out_stride, int32_t *out_counts);
