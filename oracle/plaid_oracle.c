/*
 * PLAID search path -- reference oracle (TEST INFRASTRUCTURE, not the product).
 *
 * A plain, slow, scalar CPU implementation of what the search path computes, written from the
 * paper's definitions: Eq. 1 (MaxSim), Eq. 2 (query-centroid scores), Eq. 3-4 (centroid
 * interaction), Eq. 5 (centroid pruning), Figure 4 / Section 4.3 (stage cut-offs ndocs and
 * ndocs/4), Section 4.5 (byte lookup-table decompression) and Section 3.1 (storage format).
 * Only tests, the smoke check and the benchmark's CPU-baseline leg may call it.  It shares no
 * code with the HIP library.  No blocking, fusion or reordering: every function is the
 * definition written out.
 *
 * Arithmetic: inputs are fp32.  Every dot product is accumulated in double in index order and
 * rounded once to fp32; maxima are taken on those fp32 values; every sum over the query tokens
 * is accumulated in double and rounded once to fp32.
 *
 * Orderings (the paper does not state tie rules; these are the readings used throughout):
 * centroids are ranked by (score descending, id ascending); passages by (score descending,
 * pid ascending); a passage none of whose tokens survives pruning scores -infinity.
 *
 * Parity pins (tests/test_oracle_*.py): numpy fp64 matmul for Eq. 2; full stable sorts for every
 * top-n; brute-force membership for inverted lists and candidates; "centroid interaction ==
 * MaxSim over an index whose bucket weights are all zero"; stage-2 monotonicity invariants;
 * numpy unpackbits for the byte table; encode/decode bucket-resolution bounds; a hand-computed
 * 3-centroid index; and "nprobe = C, t_cs = -inf, ndocs >= 4P  ==>  pipeline == exhaustive".
 * The vanilla ColBERTv2 routines (the paper's baseline): embedding lists against a stable argsort of the codes; the
 * candidate set against the passage-level candidates of the same probes; "nprobe = C, ncandidates >= P  ==>  vanilla ==
 * exhaustive"; pruning scores against numpy on the decompressed embeddings of E, bounded above by exact MaxSim.
 * Every function here has such a pin.  What has none: the paper prints no worked example and no per-stage values, and
 * its quality tables need collections and checkpoints that are not available, so retrieval quality against the paper
 * is parity unpinned.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_QLEN_MAX 64

typedef struct {
    int32_t dim;    /* embedding dimension d */
    int32_t nbits;  /* b: 1, 2, 4 or 8 bits per dimension */
    int64_t C, P, N;
    const float *centroids;      /* [C][dim] */
    const int64_t *doc_offsets;  /* [P+1]: tokens of passage p are doc_offsets[p] .. doc_offsets[p+1]-1 */
    const int32_t *codes;        /* [N] centroid id per token */
    const uint8_t *residuals;    /* [N][dim*nbits/8] */
    const float *bucket_weights; /* [2^nbits] */
    const int64_t *ivf_offsets;  /* [C+1] */
    const int32_t *ivf_pids;     /* ascending unique pids per centroid */
    int32_t renormalize;         /* 0: reconstructed vectors as they come (the reading used by default);
                                    1: scaled to unit length, see orc_decompress */
} orc_index;

/* ------------------------------------------------------------------ Eq. 2: S_cq = C . Q^T */
void orc_scq(const float *centroids, int64_t C, const float *Q, int32_t qlen, int32_t dim, float *S /* [C][qlen] */)
{
    for (int64_t c = 0; c < C; ++c)
        for (int32_t i = 0; i < qlen; ++i) {
            double acc = 0.0;
            for (int32_t t = 0; t < dim; ++t)
                acc += (double)centroids[c * dim + t] * (double)Q[i * dim + t];
            S[c * qlen + i] = (float)acc;
        }
}

/* ------------------------------------------------------------------ generic ranking */
typedef struct {
    float score;
    int32_t id;
} orc_pair;

static int orc_pair_cmp(const void *a, const void *b)
{
    const orc_pair *x = (const orc_pair *)a, *y = (const orc_pair *)b;
    if (x->score > y->score) return -1;
    if (x->score < y->score) return 1;
    if (x->id < y->id) return -1;
    if (x->id > y->id) return 1;
    return 0;
}

/* First min(m, n) of the n (id, score) items ordered by (score desc, id asc).  Returns the count written. */
int64_t orc_select(const int32_t *ids, const float *scores, int64_t n, int64_t m, int32_t *out_ids, float *out_scores)
{
    orc_pair *v = (orc_pair *)malloc((size_t)(n > 0 ? n : 1) * sizeof(orc_pair));
    for (int64_t j = 0; j < n; ++j) {
        v[j].score = scores[j];
        v[j].id = ids[j];
    }
    qsort(v, (size_t)n, sizeof(orc_pair), orc_pair_cmp);
    int64_t r = m < n ? m : n;
    if (r < 0) r = 0;
    for (int64_t j = 0; j < r; ++j) {
        out_ids[j] = v[j].id;
        if (out_scores) out_scores[j] = v[j].score;
    }
    free(v);
    return r;
}

/* ------------------------------------------------------------------ Section 4.1: top-nprobe centroids per query token */
void orc_top_nprobe(const float *S, int64_t C, int32_t qlen, int32_t nprobe, int32_t *out /* [qlen][nprobe] */)
{
    int32_t *ids = (int32_t *)malloc((size_t)C * sizeof(int32_t));
    float *col = (float *)malloc((size_t)C * sizeof(float));
    for (int32_t i = 0; i < qlen; ++i) {
        for (int64_t c = 0; c < C; ++c) {
            ids[c] = (int32_t)c;
            col[c] = S[c * qlen + i];
        }
        orc_select(ids, col, C, nprobe, out + (int64_t)i * nprobe, NULL);
    }
    free(ids);
    free(col);
}

static int orc_i32_cmp(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/* Section 4.1: candidate passages = union of the inverted lists of the probed centroids,
 * returned ascending and duplicate-free.  No cap on the size.  `cand` must hold P entries. */
int64_t orc_candidates(const int32_t *probed, int64_t nprobed, const int64_t *ivf_offsets, const int32_t *ivf_pids,
                       int64_t P, int32_t *cand)
{
    uint8_t *seen = (uint8_t *)calloc((size_t)(P > 0 ? P : 1), 1);
    for (int64_t j = 0; j < nprobed; ++j) {
        int32_t c = probed[j];
        for (int64_t e = ivf_offsets[c]; e < ivf_offsets[c + 1]; ++e)
            seen[ivf_pids[e]] = 1;
    }
    int64_t n = 0;
    for (int64_t p = 0; p < P; ++p)
        if (seen[p]) cand[n++] = (int32_t)p;
    free(seen);
    return n;
}

/* Eq. 5: centroid c is kept iff max_i S[c][i] >= t_cs. */
void orc_keep(const float *S, int64_t C, int32_t qlen, float t_cs, uint8_t *keep)
{
    for (int64_t c = 0; c < C; ++c) {
        float m = S[c * qlen];
        for (int32_t i = 1; i < qlen; ++i)
            if (S[c * qlen + i] > m) m = S[c * qlen + i];
        keep[c] = (m >= t_cs) ? 1 : 0;
    }
}

/* Eq. 3-4: centroid interaction of each listed passage.  D~ has one row S[code_j] per token of the
 * passage (only tokens whose centroid is kept, when keep != NULL); the score is the sum over query
 * tokens of the column maxima of D~.  An empty D~ scores -infinity. */
void orc_centroid_interaction(const float *S, int32_t qlen, const int32_t *pids, int64_t n, const int64_t *doc_offsets,
                              const int32_t *codes, const uint8_t *keep, float *scores)
{
    for (int64_t a = 0; a < n; ++a) {
        int64_t p = pids[a];
        float mx[ORC_QLEN_MAX];
        int any = 0;
        for (int32_t i = 0; i < qlen; ++i) mx[i] = -INFINITY;
        for (int64_t j = doc_offsets[p]; j < doc_offsets[p + 1]; ++j) {
            int32_t c = codes[j];
            if (keep && !keep[c]) continue;
            any = 1;
            for (int32_t i = 0; i < qlen; ++i)
                if (S[(int64_t)c * qlen + i] > mx[i]) mx[i] = S[(int64_t)c * qlen + i];
        }
        if (!any) {
            scores[a] = -INFINITY;
            continue;
        }
        double acc = 0.0;
        for (int32_t i = 0; i < qlen; ++i) acc += (double)mx[i];
        scores[a] = (float)acc;
    }
}

/* ------------------------------------------------------------------ Section 4.5: residual codec */
/* All 2^8 possible lists of bucket indices a packed byte can hold: table[v][t], t = 0 .. 8/nbits-1.
 * Indices are stored most-significant first, so dimension order is preserved within the byte. */
void orc_build_byte_table(int32_t nbits, uint8_t *table /* [256][8/nbits] */)
{
    int32_t per = 8 / nbits;
    for (int32_t v = 0; v < 256; ++v)
        for (int32_t t = 0; t < per; ++t)
            table[v * per + t] = (uint8_t)((v >> (nbits * (per - 1 - t))) & ((1 << nbits) - 1));
}

/* Decompress tokens [t0, t1): D[j][x] = fl32(centroid[code_j][x] + weight[index(j, x)]), the bucket index
 * read through the byte table.  idx_out (optional) receives the unpacked bucket indices.
 *
 * Section 4.5 says the reconstruction recovers the stored embedding and is silent on its length; the embeddings that
 * were stored had unit length (Section 3.1 scores by cosine similarity), the reconstruction does not.  The storage
 * variant ix->renormalize = 1 takes the other reading: the reconstructed vector is scaled back to unit length,
 *     n2 = sum_x D[j][x]^2 (double, index order),  inv = fl32(1 / sqrt(n2))  (0 when n2 = 0),  D[j][x] <- fl32(D[j][x] * inv),
 * and every score built on reconstructed vectors (Eq. 1, the vanilla pruning scores) uses the scaled ones. */
void orc_decompress(const orc_index *ix, int64_t t0, int64_t t1, float *D /* [(t1-t0)][dim] */, uint8_t *idx_out)
{
    int32_t per = 8 / ix->nbits, dim = ix->dim, rb = dim * ix->nbits / 8;
    uint8_t table[256 * 8];
    orc_build_byte_table(ix->nbits, table);
    for (int64_t j = t0; j < t1; ++j) {
        const float *cen = ix->centroids + (int64_t)ix->codes[j] * dim;
        const uint8_t *r = ix->residuals + j * rb;
        for (int32_t m = 0; m < rb; ++m)
            for (int32_t t = 0; t < per; ++t) {
                uint8_t b = table[(int32_t)r[m] * per + t];
                int32_t x = m * per + t;
                D[(j - t0) * dim + x] = cen[x] + ix->bucket_weights[b];
                if (idx_out) idx_out[(j - t0) * dim + x] = b;
            }
        if (ix->renormalize) {
            float *v = D + (j - t0) * dim;
            double n2 = 0.0;
            for (int32_t x = 0; x < dim; ++x) n2 += (double)v[x] * (double)v[x];
            float inv = n2 > 0.0 ? (float)(1.0 / sqrt(n2)) : 0.0f;
            for (int32_t x = 0; x < dim; ++x) v[x] = v[x] * inv;
        }
    }
}

/* Index-time encoding of one set of vectors against given centroid ids (Section 3.1): residual
 * r = fl32(x - centroid) per dimension, bucket = number of cut-offs strictly below r, packed
 * most-significant first. */
void orc_encode(const float *x, const int32_t *codes, int64_t n, const float *centroids, int32_t dim, int32_t nbits,
                const float *cutoffs /* [2^nbits - 1] */, uint8_t *packed /* [n][dim*nbits/8] */)
{
    int32_t per = 8 / nbits, rb = dim * nbits / 8, ncut = (1 << nbits) - 1;
    for (int64_t j = 0; j < n; ++j) {
        const float *cen = centroids + (int64_t)codes[j] * dim;
        for (int32_t m = 0; m < rb; ++m) {
            uint32_t byte = 0;
            for (int32_t t = 0; t < per; ++t) {
                float r = x[j * dim + m * per + t] - cen[m * per + t];
                uint32_t b = 0;
                for (int32_t q = 0; q < ncut; ++q)
                    if (cutoffs[q] < r) ++b;
                byte = (byte << nbits) | b;
            }
            packed[j * rb + m] = (uint8_t)byte;
        }
    }
}

/* Inverted lists from the token codes: list c = ascending unique pids having a token coded c.
 * Call with ivf_pids == NULL to obtain the offsets (and the total length) first. */
int64_t orc_build_ivf(const int32_t *codes, const int64_t *doc_offsets, int64_t P, int64_t C, int64_t *ivf_offsets,
                      int32_t *ivf_pids)
{
    int64_t *count = (int64_t *)calloc((size_t)C + 1, sizeof(int64_t));
    int64_t *last = (int64_t *)malloc((size_t)C * sizeof(int64_t));
    for (int64_t c = 0; c < C; ++c) last[c] = -1;
    for (int64_t p = 0; p < P; ++p)
        for (int64_t j = doc_offsets[p]; j < doc_offsets[p + 1]; ++j) {
            int32_t c = codes[j];
            if (last[c] != p) {
                last[c] = p;
                ++count[c];
            }
        }
    ivf_offsets[0] = 0;
    for (int64_t c = 0; c < C; ++c) ivf_offsets[c + 1] = ivf_offsets[c] + count[c];
    int64_t total = ivf_offsets[C];
    if (ivf_pids) {
        for (int64_t c = 0; c < C; ++c) {
            last[c] = -1;
            count[c] = 0;
        }
        for (int64_t p = 0; p < P; ++p) /* ascending p  =>  each list comes out ascending */
            for (int64_t j = doc_offsets[p]; j < doc_offsets[p + 1]; ++j) {
                int32_t c = codes[j];
                if (last[c] != p) {
                    last[c] = p;
                    ivf_pids[ivf_offsets[c] + count[c]++] = (int32_t)p;
                }
            }
    }
    free(count);
    free(last);
    return total;
}

/* ------------------------------------------------------------------ Eq. 1: exact MaxSim on reconstructed passages */
void orc_maxsim(const orc_index *ix, const float *Q, int32_t qlen, const int32_t *pids, int64_t n, float *scores)
{
    int32_t dim = ix->dim;
    for (int64_t a = 0; a < n; ++a) {
        int64_t p = pids[a], t0 = ix->doc_offsets[p], t1 = ix->doc_offsets[p + 1];
        if (t1 == t0) {
            scores[a] = -INFINITY;
            continue;
        }
        float *D = (float *)malloc((size_t)(t1 - t0) * dim * sizeof(float));
        orc_decompress(ix, t0, t1, D, NULL);
        double acc = 0.0;
        for (int32_t i = 0; i < qlen; ++i) {
            float best = -INFINITY;
            for (int64_t j = 0; j < t1 - t0; ++j) {
                double dot = 0.0;
                for (int32_t t = 0; t < dim; ++t) dot += (double)Q[i * dim + t] * (double)D[j * dim + t];
                float f = (float)dot;
                if (f > best) best = f;
            }
            acc += (double)best;
        }
        scores[a] = (float)acc;
        free(D);
    }
}

/* Exhaustive search: Eq. 1 over every passage, first k by (score desc, pid asc); unused slots (-1, -inf). */
void orc_exhaustive(const orc_index *ix, const float *Q, int32_t qlen, int32_t k, int32_t *out_ids, float *out_scores)
{
    int64_t P = ix->P;
    int32_t *pids = (int32_t *)malloc((size_t)(P > 0 ? P : 1) * sizeof(int32_t));
    float *sc = (float *)malloc((size_t)(P > 0 ? P : 1) * sizeof(float));
    for (int64_t p = 0; p < P; ++p) pids[p] = (int32_t)p;
    orc_maxsim(ix, Q, qlen, pids, P, sc);
    for (int32_t j = 0; j < k; ++j) {
        out_ids[j] = -1;
        out_scores[j] = -INFINITY;
    }
    orc_select(pids, sc, P, k, out_ids, out_scores);
    free(pids);
    free(sc);
}

/* ------------------------------------------------------------------ vanilla ColBERTv2 retrieval (Sections 3.1-3.2, 4.1)
 * What PLAID is measured against.  As far as this paper states it: the inverted list of a centroid holds the ids of the
 * EMBEDDINGS assigned to it (Section 4.1); the embeddings in the lists of the probed centroids make up E, and the
 * candidate passages are the passages those embeddings belong to; when there are more than ncandidates of them they are
 * pruned by scoring the embeddings of E -- only those -- with full residual decompression (Section 4.1), after which
 * every token of every remaining candidate is decompressed and scored exactly (Section 3.2: index lookup,
 * decompression, MaxSim).  Readings where the text is silent: a candidate's pruning score is
 * sum_i max_{j in E, j in the passage} Q_i . D_j (the late-interaction form of Eq. 1 restricted to E; every candidate
 * owns at least one embedding of E); ranking by (score descending, pid ascending); pruning only when the candidate
 * count exceeds ncandidates. */

/* Embedding-level inverted lists: list c = the ascending indices of the tokens whose code is c.
 * eids may be NULL (offsets only).  Returns N. */
int64_t orc_build_ivf_embeddings(const int32_t *codes, int64_t N, int64_t C, int64_t *offsets /* [C+1] */, int64_t *eids /* [N] */)
{
    for (int64_t c = 0; c <= C; ++c) offsets[c] = 0;
    for (int64_t j = 0; j < N; ++j) offsets[codes[j] + 1] += 1;
    for (int64_t c = 0; c < C; ++c) offsets[c + 1] += offsets[c];
    if (eids) {
        int64_t *fill = (int64_t *)malloc((size_t)(C > 0 ? C : 1) * sizeof(int64_t));
        for (int64_t c = 0; c < C; ++c) fill[c] = offsets[c];
        for (int64_t j = 0; j < N; ++j) eids[fill[codes[j]]++] = j;
        free(fill);
    }
    return N;
}

/* Pruning score of each listed candidate (Section 4.1): sum over the query tokens of the maximum, over the passage's
 * embeddings in E (inE[j] != 0), of Q_i . D_j with D_j decompressed in full; -inf for a passage with no embedding in E. */
void orc_vanilla_prune_scores(const orc_index *ix, const float *Q, int32_t qlen, const uint8_t *inE, const int32_t *pids,
                              int64_t n, float *scores)
{
    int32_t dim = ix->dim;
    float *D = (float *)malloc((size_t)dim * sizeof(float));
    for (int64_t a = 0; a < n; ++a) {
        int64_t p = pids[a];
        float best[ORC_QLEN_MAX];
        int any = 0;
        for (int32_t i = 0; i < qlen; ++i) best[i] = -INFINITY;
        for (int64_t j = ix->doc_offsets[p]; j < ix->doc_offsets[p + 1]; ++j) {
            if (!inE[j]) continue;
            any = 1;
            orc_decompress(ix, j, j + 1, D, NULL);
            for (int32_t i = 0; i < qlen; ++i) {
                double dot = 0.0;
                for (int32_t t = 0; t < dim; ++t) dot += (double)Q[i * dim + t] * (double)D[t];
                float f = (float)dot;
                if (f > best[i]) best[i] = f;
            }
        }
        double acc = 0.0;
        for (int32_t i = 0; i < qlen; ++i) acc += (double)best[i];
        scores[a] = any ? (float)acc : -INFINITY;
    }
    free(D);
}

typedef struct {  /* optional dumps of orc_vanilla_search; any pointer may be NULL */
    int32_t *cand;        /* [P] ascending candidate passages */
    int64_t *n_cand;
    int64_t *n_embeddings; /* |E| */
    int32_t *kept;        /* [min(ncandidates, P)] candidates after pruning, ascending pid */
    float *kept_scores;   /* their pruning scores (only when pruning happened, else untouched) */
    int64_t *n_kept;
    int32_t *pruned;      /* 1 when the candidate count exceeded ncandidates */
} orc_vanilla_dumps;

/* One query.  eoff / eids: embedding-level lists (orc_build_ivf_embeddings).  Unused output slots get (-1, -inf). */
int32_t orc_vanilla_search(const orc_index *ix, const int64_t *eoff, const int64_t *eids, const float *Q, int32_t qlen,
                           int32_t nprobe, int64_t ncandidates, int32_t k, int32_t *out_ids, float *out_scores,
                           const orc_vanilla_dumps *dump)
{
    int64_t C = ix->C, P = ix->P, N = ix->N;
    int32_t dim = ix->dim;
    if (qlen > ORC_QLEN_MAX || nprobe < 1 || nprobe > C || ncandidates < 1 || k < 1) return -1;
    float *S = (float *)malloc((size_t)C * qlen * sizeof(float));
    int32_t *probed = (int32_t *)malloc((size_t)qlen * nprobe * sizeof(int32_t));
    orc_scq(ix->centroids, C, Q, qlen, dim, S);
    orc_top_nprobe(S, C, qlen, nprobe, probed);
    /* E: a flag per embedding; which passage owns an embedding: by walking the passage offsets */
    uint8_t *probed_c = (uint8_t *)calloc((size_t)C, 1), *inE = (uint8_t *)calloc((size_t)(N > 0 ? N : 1), 1);
    for (int64_t a = 0; a < (int64_t)qlen * nprobe; ++a) probed_c[probed[a]] = 1;
    int64_t nE = 0;
    for (int64_t c = 0; c < C; ++c)
        if (probed_c[c])
            for (int64_t e = eoff[c]; e < eoff[c + 1]; ++e) {
                inE[eids[e]] = 1;
                nE += 1;
            }
    int32_t *cand = (int32_t *)malloc((size_t)(P > 0 ? P : 1) * sizeof(int32_t));
    int64_t n_cand = 0;
    for (int64_t p = 0; p < P; ++p) {
        int any = 0;
        for (int64_t j = ix->doc_offsets[p]; j < ix->doc_offsets[p + 1]; ++j) any |= inE[j];
        if (any) cand[n_cand++] = (int32_t)p;
    }
    if (dump && dump->cand) memcpy(dump->cand, cand, (size_t)n_cand * sizeof(int32_t));
    if (dump && dump->n_cand) *dump->n_cand = n_cand;
    if (dump && dump->n_embeddings) *dump->n_embeddings = nE;
    /* pruning of an over-large candidate set by the embeddings of E alone */
    int64_t n_kept = n_cand;
    int32_t *kept = cand;
    int32_t *kbuf = NULL;
    int32_t pruned = n_cand > ncandidates;
    if (pruned) {
        float *ps = (float *)malloc((size_t)n_cand * sizeof(float));
        orc_vanilla_prune_scores(ix, Q, qlen, inE, cand, n_cand, ps);
        kbuf = (int32_t *)malloc((size_t)ncandidates * sizeof(int32_t));
        float *ks = (float *)malloc((size_t)ncandidates * sizeof(float));
        n_kept = orc_select(cand, ps, n_cand, ncandidates, kbuf, ks);
        /* report the kept set in ascending pid order, scores alongside */
        for (int64_t a = 1; a < n_kept; ++a) {
            int32_t id = kbuf[a];
            float sc = ks[a];
            int64_t b = a - 1;
            while (b >= 0 && kbuf[b] > id) {
                kbuf[b + 1] = kbuf[b];
                ks[b + 1] = ks[b];
                --b;
            }
            kbuf[b + 1] = id;
            ks[b + 1] = sc;
        }
        if (dump && dump->kept_scores) memcpy(dump->kept_scores, ks, (size_t)n_kept * sizeof(float));
        kept = kbuf;
        free(ps);
        free(ks);
    }
    if (dump && dump->kept) memcpy(dump->kept, kept, (size_t)n_kept * sizeof(int32_t));
    if (dump && dump->n_kept) *dump->n_kept = n_kept;
    if (dump && dump->pruned) *dump->pruned = pruned;
    /* every token of every remaining candidate: exact MaxSim (Eq. 1), best k */
    float *sc = (float *)malloc((size_t)(n_kept > 0 ? n_kept : 1) * sizeof(float));
    orc_maxsim(ix, Q, qlen, kept, n_kept, sc);
    for (int32_t j = 0; j < k; ++j) {
        out_ids[j] = -1;
        out_scores[j] = -INFINITY;
    }
    orc_select(kept, sc, n_kept, k, out_ids, out_scores);
    free(sc);
    free(kbuf);
    free(cand);
    free(inE);
    free(probed_c);
    free(probed);
    free(S);
    return 0;
}

/* ------------------------------------------------------------------ the four-stage pipeline (Figure 4, Sections 4.1-4.4) */
typedef struct {  /* optional per-stage dumps; any pointer may be NULL */
    float *S;             /* [C][qlen] */
    int32_t *probed;      /* [qlen][nprobe] */
    int32_t *cand;        /* [P] */
    int64_t *n_cand;
    int32_t *sel2_ids;    /* [ndocs] */
    float *sel2_scores;
    int64_t *n2;
    int32_t *sel3_ids;    /* [max(1, ndocs/4)] */
    float *sel3_scores;
    int64_t *n3;
} orc_dumps;

int32_t orc_search(const orc_index *ix, const float *Q, int32_t qlen, int32_t nprobe, float t_cs, int32_t ndocs, int32_t k,
                   int32_t *out_ids, float *out_scores, const orc_dumps *dump)
{
    int64_t C = ix->C, P = ix->P;
    if (qlen > ORC_QLEN_MAX || nprobe < 1 || nprobe > C || ndocs < 1 || k < 1) return -1;

    /* Stage 1: centroid scores, probes, candidates */
    float *S = (float *)malloc((size_t)C * qlen * sizeof(float));
    orc_scq(ix->centroids, C, Q, qlen, ix->dim, S);
    int32_t *probed = (int32_t *)malloc((size_t)qlen * nprobe * sizeof(int32_t));
    orc_top_nprobe(S, C, qlen, nprobe, probed);
    int32_t *cand = (int32_t *)malloc((size_t)(P > 0 ? P : 1) * sizeof(int32_t));
    int64_t n_cand = orc_candidates(probed, (int64_t)qlen * nprobe, ix->ivf_offsets, ix->ivf_pids, P, cand);

    /* Stage 2: centroid interaction with pruning, keep ndocs */
    uint8_t *keep = (uint8_t *)malloc((size_t)C);
    orc_keep(S, C, qlen, t_cs, keep);
    float *s2 = (float *)malloc((size_t)(n_cand > 0 ? n_cand : 1) * sizeof(float));
    orc_centroid_interaction(S, qlen, cand, n_cand, ix->doc_offsets, ix->codes, keep, s2);
    int32_t *sel2 = (int32_t *)malloc((size_t)ndocs * sizeof(int32_t));
    float *sel2s = (float *)malloc((size_t)ndocs * sizeof(float));
    int64_t n2 = orc_select(cand, s2, n_cand, ndocs, sel2, sel2s);

    /* Stage 3: centroid interaction without pruning, keep ndocs/4 */
    int64_t m3 = ndocs / 4 > 1 ? ndocs / 4 : 1;
    float *s3 = (float *)malloc((size_t)(n2 > 0 ? n2 : 1) * sizeof(float));
    orc_centroid_interaction(S, qlen, sel2, n2, ix->doc_offsets, ix->codes, NULL, s3);
    int32_t *sel3 = (int32_t *)malloc((size_t)m3 * sizeof(int32_t));
    float *sel3s = (float *)malloc((size_t)m3 * sizeof(float));
    int64_t n3 = orc_select(sel2, s3, n2, m3, sel3, sel3s);

    /* Stage 4: decompress, exact MaxSim, top-k */
    float *s4 = (float *)malloc((size_t)(n3 > 0 ? n3 : 1) * sizeof(float));
    orc_maxsim(ix, Q, qlen, sel3, n3, s4);
    for (int32_t j = 0; j < k; ++j) {
        out_ids[j] = -1;
        out_scores[j] = -INFINITY;
    }
    orc_select(sel3, s4, n3, k, out_ids, out_scores);

    if (dump) {
        if (dump->S) memcpy(dump->S, S, (size_t)C * qlen * sizeof(float));
        if (dump->probed) memcpy(dump->probed, probed, (size_t)qlen * nprobe * sizeof(int32_t));
        if (dump->cand) memcpy(dump->cand, cand, (size_t)n_cand * sizeof(int32_t));
        if (dump->n_cand) *dump->n_cand = n_cand;
        if (dump->sel2_ids) memcpy(dump->sel2_ids, sel2, (size_t)n2 * sizeof(int32_t));
        if (dump->sel2_scores) memcpy(dump->sel2_scores, sel2s, (size_t)n2 * sizeof(float));
        if (dump->n2) *dump->n2 = n2;
        if (dump->sel3_ids) memcpy(dump->sel3_ids, sel3, (size_t)n3 * sizeof(int32_t));
        if (dump->sel3_scores) memcpy(dump->sel3_scores, sel3s, (size_t)n3 * sizeof(float));
        if (dump->n3) *dump->n3 = n3;
    }
    free(S); free(probed); free(cand); free(keep); free(s2); free(sel2); free(sel2s);
    free(s3); free(sel3); free(sel3s); free(s4);
    return 0;
}

/* A batch of independent queries; OpenMP (when compiled in) parallelises across queries only --
 * each query still runs the scalar code above on one thread.  Returns the number of threads used. */
int32_t orc_search_batch(const orc_index *ix, const float *Q, int32_t nq, int32_t qlen, int32_t nprobe, float t_cs,
                         int32_t ndocs, int32_t k, int32_t *out_ids, float *out_scores, int32_t nthreads)
{
    int32_t used = 1;
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    if (nthreads < 1) nthreads = omp_get_max_threads();
    used = nthreads < nq ? nthreads : nq;
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads)
#endif
    for (int32_t q = 0; q < nq; ++q)
        orc_search(ix, Q + (int64_t)q * qlen * ix->dim, qlen, nprobe, t_cs, ndocs, k, out_ids + (int64_t)q * k,
                   out_scores + (int64_t)q * k, NULL);
    return used;
}
