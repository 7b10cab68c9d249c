// C ABI of libplaid: index handles, the per-index workspace, and the host side of the search
// pipeline (Figure 4): it only enqueues kernels on the caller's stream and never reads a result
// back, so a search costs no host-device round trip.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <mutex>
#include <string>
#include <vector>

#include "plaid_internal.h"

// ------------------------------------------------------------------ errors
static thread_local char g_err[512] = "";

static int fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}
extern "C" const char *plaid_last_error(void) { return g_err; }

#define HIP_TRY(expr)                                                                                         \
    do {                                                                                                      \
        hipError_t e_ = (expr);                                                                               \
        if (e_ != hipSuccess) return fail(PLAID_EHIP, "%s: %s (%s:%d)", #expr, hipGetErrorString(e_), __FILE__, __LINE__); \
    } while (0)

// ------------------------------------------------------------------ workspace of the entry point that allocates nothing
// plaid_search_static carves its workspace out of this array instead of library-allocated memory.  The name below is a
// host-side stand-in, not a device address: each device holds its own copy, whose address hipGetSymbolAddress returns
// with that device current; host code only ever uses the addresses kept in g_scratch_addr.
#define PLAID_STATIC_WORKSPACE_BYTES ((size_t)64 << 20)
static __device__ __align__(256) unsigned char scratch[PLAID_STATIC_WORKSPACE_BYTES];
static void *g_scratch_addr[64] = {nullptr};  // per device ordinal
static std::mutex g_scratch_guard;

// ------------------------------------------------------------------ handle
#define N_EVENTS (PLAID_NUM_STAGES + 1)

struct plaid_index {
    int device = 0;
    int32_t nbits = 0;
    int64_t C = 0, P = 0, N = 0, ivf_len = 0;
    const float *centroids = nullptr;
    const int64_t *doc_offsets = nullptr;
    const int32_t *codes = nullptr;
    const uint8_t *residuals = nullptr;
    const float *weights = nullptr;
    const int64_t *ivf_offsets = nullptr;
    const int32_t *ivf_pids = nullptr;
    std::vector<void *> owned;  // device allocations released by plaid_index_free
    void *ws = nullptr;         // workspace, grown on demand
    char *static_ws = nullptr;  // this device's copy of the static workspace array (plaid_search_static)
    size_t ws_bytes = 0;
    int32_t max_chunk = 0;
    int32_t timing = 0;
    unsigned long long *score_clocks = nullptr;  // device [2] (owned): tick sums of the score kernel while timing is on
    int32_t scq_matrix_form = 0;  // double-precision score kernel: 1 = matrix instruction, 0 = vector FMA chain
    int32_t scq_form = 0;         // score kernel of a search: PLAID_SCQ_VECTOR / _MATRIX / _SPLIT16
    void *A16 = nullptr;          // split-fp16 operand form of the centroids (owned), when scq_form is PLAID_SCQ_SPLIT16
    float *inv_norm = nullptr;    // [N] 1 / |reconstructed vector| (owned; built by plaid_index_set_renormalize)
    bool renormalize = false;     // stage 4 and plaid_decompress_passages scale reconstructed vectors to unit length
    bool no_scores = false;       // nearest-centroid assignment with the split-fp16 kernel: S_cq itself is not stored
    uint32_t *ivr_table = nullptr;  // range table of the inverted lists (owned); null: union + code stream are used
    int32_t ivr_shift = 11;         // log2 of the passages per table column (11 or 13)
    int32_t *dense_id = nullptr;    // with the range table: bitmap row of each centroid's list, -1 for all but the longest
    uint32_t *dense_bits = nullptr; // [rows][ceil(P / 32)]
    // vanilla ColBERTv2 retrieval (built on its first use): embedding-level inverted lists and the passage of each token
    int64_t *emb_offsets = nullptr;  // [C + 1]
    int32_t *emb_ids = nullptr;      // [N] ascending token indices per centroid
    int32_t *tok2pid = nullptr;      // [N]
    float stage_ms[PLAID_NUM_STAGES] = {0};
    hipEvent_t ev[N_EVENTS] = {nullptr};
};

struct DeviceGuard {
    int prev = -1;
    bool ok = false;
    explicit DeviceGuard(int dev)
    {
        if (hipGetDevice(&prev) == hipSuccess && hipSetDevice(dev) == hipSuccess) ok = true;
    }
    ~DeviceGuard()
    {
        if (prev >= 0) (void)hipSetDevice(prev);
    }
};

// Address of the static workspace array on `device`, which must be the current device (looked up once per device).
static int static_workspace_address(int device, char **out)
{
    if (device < 0 || device >= 64) return fail(PLAID_EINVAL, "device ordinal %d out of range", device);
    const std::lock_guard<std::mutex> lock(g_scratch_guard);
    if (!g_scratch_addr[device]) {
        void *p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) {
            (void)hipGetLastError();
            return fail(PLAID_EHIP, "hipGetSymbolAddress(static workspace): %s", hipGetErrorString(e));
        }
        g_scratch_addr[device] = p;
    }
    *out = (char *)g_scratch_addr[device];
    return PLAID_OK;
}

// Which score kernel this handle uses.  Default: the split-fp16 matrix kernel, with the double-precision matrix kernel
// (or, should the device check of that instruction fail, the vector chain) behind it for nprobe values the fast probe
// kernel does not serve.  PLAID_SCQ_FORM=vector|matrix|split16 overrides the choice (matrix is refused when the device
// check fails); the check itself runs once per process and device.
static int choose_scq_form(plaid_index *ix)
{
    static int checked[64] = {0};  // 0 = not yet, 1 = matrix form verified, 2 = not usable
    static std::mutex guard;       // indexes may be created from several host threads
    const std::lock_guard<std::mutex> lock(guard);
    const char *env = getenv("PLAID_SCQ_FORM");
    if (env && strcmp(env, "vector") && strcmp(env, "matrix") && strcmp(env, "split16"))
        return fail(PLAID_EINVAL, "PLAID_SCQ_FORM must be 'vector', 'matrix' or 'split16'");
    if (env && !strcmp(env, "vector")) {
        ix->scq_matrix_form = 0;
        ix->scq_form = PLAID_SCQ_VECTOR;
        return PLAID_OK;
    }
    const int slot = ix->device < 64 ? ix->device : 63;
    if (!checked[slot] || ix->device >= 64) {
        int ok = 0;
        const int e = plaid_scq_matrix_form_ok(nullptr, &ok);
        if (e) return fail(PLAID_EHIP, "score-kernel self check failed: %s", hipGetErrorString((hipError_t)e));
        checked[slot] = ok ? 1 : 2;
    }
    const bool want_matrix = env && !strcmp(env, "matrix");
    if (want_matrix && checked[slot] != 1)
        return fail(PLAID_EHIP, "PLAID_SCQ_FORM=matrix, but the matrix instruction does not reproduce the FMA chain here");
    ix->scq_matrix_form = checked[slot] == 1;
    ix->scq_form = want_matrix ? PLAID_SCQ_MATRIX : PLAID_SCQ_SPLIT16;
    return PLAID_OK;
}

struct TempAlloc {  // device memory released when the call returns
    void *p = nullptr;
    ~TempAlloc()
    {
        if (p) (void)hipFree(p);
    }
};

// The split kernel scales the centroids' leading fp16 terms by 2^11: a table with a component of 32 or more (or one that
// is not a number) cannot use it.  Such an index (ix->scq_form is PLAID_SCQ_SPLIT16 on entry) gets a double-precision
// form instead, unless the caller insisted on the split form, which is then an error.  Synchronises the stream.
static int scq16_check_centroids(plaid_index *ix, const float *centroids, int64_t C, hipStream_t st)
{
    TempAlloc mb;
    if (hipMalloc(&mb.p, 256) != hipSuccess) {
        (void)hipGetLastError();
        return fail(PLAID_ENOMEM, "hipMalloc(256) failed");
    }
    HIP_TRY(hipMemsetAsync(mb.p, 0, 256, st));
    plaid_launch_scq16_max_abs(st, centroids, C * DIM, (uint32_t *)mb.p);
    HIP_TRY(hipGetLastError());
    float largest = 0.f;
    HIP_TRY(hipMemcpyAsync(&largest, mb.p, 4, hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    if (largest <= PLAID_SCQ16_CENTROID_MAX) return PLAID_OK;
    const char *env = getenv("PLAID_SCQ_FORM");
    if (env && !strcmp(env, "split16"))
        return fail(PLAID_EINVAL, "PLAID_SCQ_FORM=split16 needs centroid components within %g (largest: %g)",
                    (double)PLAID_SCQ16_CENTROID_MAX, (double)largest);
    ix->scq_form = ix->scq_matrix_form ? PLAID_SCQ_MATRIX : PLAID_SCQ_VECTOR;
    return PLAID_OK;
}

// Operand form of the centroid table for the split-fp16 score kernel (512 bytes per centroid, built once).
static int build_scq16_operands(plaid_index *ix)
{
    if (ix->scq_form != PLAID_SCQ_SPLIT16) return PLAID_OK;
    int rc = scq16_check_centroids(ix, ix->centroids, ix->C, nullptr);
    if (rc || ix->scq_form != PLAID_SCQ_SPLIT16) return rc;
    const size_t bytes = plaid_scq16_centroid_bytes(ix->C);
    void *d = nullptr;
    if (hipMalloc(&d, bytes) != hipSuccess) {
        (void)hipGetLastError();
        return fail(PLAID_ENOMEM, "hipMalloc(%zu) for the centroids' matrix operands failed", bytes);
    }
    ix->owned.push_back(d);
    plaid_launch_scq16_split_centroids(nullptr, ix->centroids, ix->C, d);
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipStreamSynchronize(nullptr));
    ix->A16 = d;
    return PLAID_OK;
}

// The inverted form of candidate generation + stage 2 needs a table of C x (P / 2^shift + 1) positions, shift = 11 or
// 13 (2048 or 8192 passages per workgroup).  The finer one is faster at every index size measured (three or four
// workgroups share a compute unit instead of one or two); it is built when its table is at most four times the size of
// the inverted lists (or tiny in absolute terms), the coarser one under the same rule or when the finer table cannot
// be allocated.  PLAID_STAGE2_FORM=stream|inverted|inverted11|inverted13 (read at index creation) overrides that.
static int build_range_table(plaid_index *ix)
{
    const char *env = getenv("PLAID_STAGE2_FORM");
    if (env && strcmp(env, "stream") && strcmp(env, "inverted") && strcmp(env, "inverted11") && strcmp(env, "inverted13"))
        return fail(PLAID_EINVAL, "PLAID_STAGE2_FORM must be 'stream', 'inverted', 'inverted11' or 'inverted13'");
    const size_t list_bytes = (size_t)ix->ivf_len * 4;
    auto fits = [&](int shift) {
        const size_t b = plaid_ivf_range_table_bytes(ix->C, ix->P, shift);
        return b <= (size_t)32 << 20 || b <= 4 * list_bytes;
    };
    int shift = fits(11) ? 11 : (fits(13) ? 13 : 0);
    if (env && !strcmp(env, "stream")) shift = 0;
    if (env && !strcmp(env, "inverted") && !shift) shift = 13;
    if (env && !strcmp(env, "inverted11")) shift = 11;
    if (env && !strcmp(env, "inverted13")) shift = 13;
    if (!shift || ix->P == 0) return PLAID_OK;
    const bool forced = env != nullptr && strcmp(env, "inverted") != 0;  // else an allocation failure falls back
    void *d = nullptr;
    size_t bytes = plaid_ivf_range_table_bytes(ix->C, ix->P, shift);
    hipError_t e = hipMalloc(&d, bytes ? bytes : 4);
    if (e != hipSuccess && !forced && shift == 11) {  // the coarser table is a quarter of the size
        (void)hipGetLastError();
        shift = 13;
        bytes = plaid_ivf_range_table_bytes(ix->C, ix->P, shift);
        e = hipMalloc(&d, bytes ? bytes : 4);
    }
    if (e != hipSuccess) {
        (void)hipGetLastError();
        if (forced) return fail(PLAID_ENOMEM, "hipMalloc(%zu) for the inverted-list range table failed", bytes);
        return PLAID_OK;  // not essential: the streaming form is used
    }
    ix->ivr_shift = shift;
    ix->owned.push_back(d);
    plaid_launch_ivf_range_table(nullptr, ix->ivf_offsets, ix->ivf_pids, ix->C, ix->P, shift, (uint32_t *)d);
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipStreamSynchronize(nullptr));
    // bitmaps of the longest lists
    const int64_t words = (ix->P + 31) / 32;
    int32_t *did = nullptr, *counter = nullptr;
    if (hipMalloc((void **)&did, (size_t)ix->C * 4) != hipSuccess || hipMalloc((void **)&counter, 4) != hipSuccess) {
        (void)hipGetLastError();
        if (did) (void)hipFree(did);
        return fail(PLAID_ENOMEM, "hipMalloc for the dense-list index failed");
    }
    ix->owned.push_back(did);
    ix->owned.push_back(counter);
    HIP_TRY(hipMemset(counter, 0, 4));
    plaid_launch_ivf_dense_mark(nullptr, ix->ivf_offsets, ix->C, ix->P, did, counter);
    int32_t rows = 0;
    HIP_TRY(hipMemcpy(&rows, counter, 4, hipMemcpyDeviceToHost));
    void *db = nullptr;
    const size_t dbytes = (size_t)(rows > 0 ? rows : 1) * (size_t)words * 4;
    if (hipMalloc(&db, dbytes) != hipSuccess) {
        (void)hipGetLastError();
        return fail(PLAID_ENOMEM, "hipMalloc(%zu) for the dense-list bitmaps failed", dbytes);
    }
    ix->owned.push_back(db);
    HIP_TRY(hipMemset(db, 0, dbytes));
    if (rows > 0) plaid_launch_ivf_dense_fill(nullptr, ix->ivf_offsets, ix->ivf_pids, ix->C, ix->P, did, (uint32_t *)db, words);
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipStreamSynchronize(nullptr));
    ix->dense_id = did;
    ix->dense_bits = (uint32_t *)db;
    ix->ivr_table = (uint32_t *)d;
    return PLAID_OK;
}

static inline size_t a256(size_t x) { return (x + 255) & ~(size_t)255; }

static int check_sizes(int32_t dim, int32_t nbits, int64_t C, int64_t P, int64_t N, int64_t ivf_len)
{
    if (dim != PLAID_DIM) return fail(PLAID_EINVAL, "dim must be %d (got %d)", PLAID_DIM, dim);
    if (nbits != 1 && nbits != 2) return fail(PLAID_EINVAL, "nbits must be 1 or 2 (got %d)", nbits);
    if (C < 1 || C >= (1ll << 31)) return fail(PLAID_EINVAL, "num_centroids out of range (%lld)", (long long)C);
    if (P < 1 || P >= (1ll << 31)) return fail(PLAID_EINVAL, "num_passages out of range (%lld)", (long long)P);
    if (N < 0) return fail(PLAID_EINVAL, "num_embeddings negative");
    if (ivf_len < 0) return fail(PLAID_EINVAL, "inverted-list length negative");
    return PLAID_OK;
}

// Host-side structural validation of an index whose arrays are in host memory.
static int validate_host(const plaid_index_view *v, int64_t ivf_len)
{
    const int64_t C = v->num_centroids, P = v->num_passages, N = v->num_embeddings;
    if (v->doc_offsets[0] != 0) return fail(PLAID_EINVAL, "doc_offsets[0] must be 0");
    for (int64_t p = 0; p < P; ++p)
        if (v->doc_offsets[p + 1] < v->doc_offsets[p]) return fail(PLAID_EINVAL, "doc_offsets decreases at passage %lld", (long long)p);
    if (v->doc_offsets[P] != N) return fail(PLAID_EINVAL, "doc_offsets[P] (%lld) != num_embeddings (%lld)", (long long)v->doc_offsets[P], (long long)N);
    for (int64_t j = 0; j < N; ++j)
        if (v->codes[j] < 0 || v->codes[j] >= C) return fail(PLAID_EINVAL, "codes[%lld] = %d out of range", (long long)j, v->codes[j]);
    if (v->ivf_offsets[0] != 0) return fail(PLAID_EINVAL, "ivf_offsets[0] must be 0");
    for (int64_t c = 0; c < C; ++c) {
        const int64_t a = v->ivf_offsets[c], b = v->ivf_offsets[c + 1];
        if (b < a || b > ivf_len) return fail(PLAID_EINVAL, "ivf_offsets malformed at centroid %lld", (long long)c);
        for (int64_t e = a; e < b; ++e) {
            if (v->ivf_pids[e] < 0 || v->ivf_pids[e] >= P) return fail(PLAID_EINVAL, "ivf_pids[%lld] out of range", (long long)e);
            if (e > a && v->ivf_pids[e] <= v->ivf_pids[e - 1]) return fail(PLAID_EINVAL, "inverted list %lld not ascending/unique", (long long)c);
        }
    }
    return PLAID_OK;
}

static int dev_alloc_copy(plaid_index *ix, const void *src, size_t bytes, hipMemcpyKind kind, const void **out)
{
    void *d = nullptr;
    const size_t alloc = bytes ? bytes : 256;
    hipError_t e = hipMalloc(&d, alloc);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return fail(PLAID_ENOMEM, "hipMalloc(%zu) failed: %s", alloc, hipGetErrorString(e));
    }
    ix->owned.push_back(d);
    if (bytes) HIP_TRY(hipMemcpy(d, src, bytes, kind));
    *out = d;
    return PLAID_OK;
}

extern "C" void plaid_index_free(plaid_index *idx)
{
    if (!idx) return;
    DeviceGuard g(idx->device);
    (void)hipDeviceSynchronize();
    for (void *p : idx->owned) (void)hipFree(p);
    if (idx->ws) (void)hipFree(idx->ws);
    for (int i = 0; i < N_EVENTS; ++i)
        if (idx->ev[i]) (void)hipEventDestroy(idx->ev[i]);
    delete idx;
}

extern "C" int plaid_index_from_view(const plaid_index_view *v, int device, int copy, plaid_index **out)
{
    if (!v || !out) return fail(PLAID_EINVAL, "null argument");
    *out = nullptr;
    if (!v->centroids || !v->doc_offsets || !v->bucket_weights || !v->ivf_offsets)
        return fail(PLAID_EINVAL, "null array in view");
    if (v->num_embeddings > 0 && (!v->codes || !v->residuals)) return fail(PLAID_EINVAL, "null codes/residuals");
    if (!copy && !v->on_device) return fail(PLAID_EINVAL, "copy = 0 requires device arrays");
    if (!copy && ((((uintptr_t)v->centroids) | ((uintptr_t)v->codes) | ((uintptr_t)v->residuals)) & 15))
        return fail(PLAID_EINVAL, "copy = 0 requires centroids, codes and residuals aligned to 16 bytes");
    int rc = check_sizes(v->dim, v->nbits, v->num_centroids, v->num_passages, v->num_embeddings, 0);
    if (rc) return rc;
    const int64_t C = v->num_centroids, P = v->num_passages, N = v->num_embeddings;
    int64_t ivf_len = 0;
    if (!v->on_device) {
        // host arrays are checked in full before any device is touched
        ivf_len = v->ivf_offsets[C];
        if (ivf_len < 0 || (ivf_len > 0 && !v->ivf_pids)) return fail(PLAID_EINVAL, "bad inverted lists");
        rc = validate_host(v, ivf_len);
        if (rc) return rc;
    }
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || device < 0 || device >= ndev) {
        (void)hipGetLastError();
        return fail(PLAID_EHIP, "no HIP device %d (found %d)", device, ndev);
    }
    DeviceGuard g(device);
    if (!g.ok) return fail(PLAID_EHIP, "hipSetDevice(%d) failed", device);
    if (v->on_device) {
        HIP_TRY(hipMemcpy(&ivf_len, v->ivf_offsets + C, sizeof(int64_t), hipMemcpyDeviceToHost));
        int64_t n_chk = 0;
        HIP_TRY(hipMemcpy(&n_chk, v->doc_offsets + P, sizeof(int64_t), hipMemcpyDeviceToHost));
        if (n_chk != N) return fail(PLAID_EINVAL, "doc_offsets[P] (%lld) != num_embeddings (%lld)", (long long)n_chk, (long long)N);
        if (ivf_len < 0 || (ivf_len > 0 && !v->ivf_pids)) return fail(PLAID_EINVAL, "bad inverted lists");
        // device arrays get the same structural checks as host arrays, in one kernel: the search kernels index memory
        // with these offsets, codes and passage ids
        int32_t *flag = nullptr;
        if (hipMalloc((void **)&flag, 4) != hipSuccess) {
            (void)hipGetLastError();
            return fail(PLAID_ENOMEM, "hipMalloc failed");
        }
        int32_t bad = 0;
        hipError_t e = hipMemset(flag, 0, 4);
        if (e == hipSuccess) {
            plaid_launch_index_validate(nullptr, v->doc_offsets, P, N, v->codes, C, v->ivf_offsets, v->ivf_pids, ivf_len, flag);
            e = hipGetLastError();
        }
        if (e == hipSuccess) e = hipMemcpy(&bad, flag, 4, hipMemcpyDeviceToHost);
        (void)hipFree(flag);
        if (e != hipSuccess) return fail(PLAID_EHIP, "index validation: %s", hipGetErrorString(e));
        if (bad)
            return fail(PLAID_EINVAL, "malformed index arrays:%s%s%s%s%s", (bad & 1) ? " doc_offsets not monotone from 0 to N;" : "",
                        (bad & 2) ? " a code outside [0, C);" : "", (bad & 4) ? " ivf_offsets not monotone from 0 to their end;" : "",
                        (bad & 8) ? " a passage id outside [0, P);" : "", (bad & 16) ? " an inverted list not strictly ascending;" : "");
    }

    plaid_index *ix = new (std::nothrow) plaid_index();
    if (!ix) return fail(PLAID_ENOMEM, "host allocation failed");
    ix->device = device;
    ix->nbits = v->nbits;
    ix->C = C;
    ix->P = P;
    ix->N = N;
    ix->ivf_len = ivf_len;
    if (copy) {
        const hipMemcpyKind kind = v->on_device ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice;
        const size_t rb = (size_t)16 * v->nbits;
        rc = dev_alloc_copy(ix, v->centroids, (size_t)C * PLAID_DIM * 4, kind, (const void **)&ix->centroids);
        if (!rc) rc = dev_alloc_copy(ix, v->doc_offsets, (size_t)(P + 1) * 8, kind, (const void **)&ix->doc_offsets);
        if (!rc) rc = dev_alloc_copy(ix, v->codes, (size_t)N * 4, kind, (const void **)&ix->codes);
        if (!rc) rc = dev_alloc_copy(ix, v->residuals, (size_t)N * rb, kind, (const void **)&ix->residuals);
        if (!rc) rc = dev_alloc_copy(ix, v->bucket_weights, (size_t)(1 << v->nbits) * 4, kind, (const void **)&ix->weights);
        if (!rc) rc = dev_alloc_copy(ix, v->ivf_offsets, (size_t)(C + 1) * 8, kind, (const void **)&ix->ivf_offsets);
        if (!rc) rc = dev_alloc_copy(ix, v->ivf_pids, (size_t)ivf_len * 4, kind, (const void **)&ix->ivf_pids);
        if (rc) {
            plaid_index_free(ix);
            return rc;
        }
    } else {
        ix->centroids = v->centroids;
        ix->doc_offsets = v->doc_offsets;
        ix->codes = v->codes;
        ix->residuals = v->residuals;
        ix->weights = v->bucket_weights;
        ix->ivf_offsets = v->ivf_offsets;
        ix->ivf_pids = v->ivf_pids;
    }
    rc = choose_scq_form(ix);
    if (!rc) rc = build_scq16_operands(ix);
    if (!rc) rc = build_range_table(ix);
    if (!rc) rc = static_workspace_address(ix->device, &ix->static_ws);  // (the index's device is current here)
    if (rc) {
        plaid_index_free(ix);
        return rc;
    }
    *out = ix;
    return PLAID_OK;
}

// ------------------------------------------------------------------ index file
static const char kMagic[8] = {'P', 'L', 'A', 'I', 'D', 'I', 'X', '1'};

struct FileHeader {
    char magic[8];
    int32_t dim, nbits;
    int64_t C, P, N, ivf_len;
    char pad[16];
};
static_assert(sizeof(FileHeader) == 64, "index file header is 64 bytes");

static int read_section(FILE *f, std::vector<char> &buf, size_t bytes)
{
    const size_t padded = (bytes + 63) & ~(size_t)63;
    try {
        buf.resize(padded ? padded : 1);
    } catch (...) {
        return fail(PLAID_ENOMEM, "host allocation of %zu bytes failed", padded);
    }
    if (padded && fread(buf.data(), 1, padded, f) != padded) return fail(PLAID_EFORMAT, "index file truncated");
    return PLAID_OK;
}

extern "C" int plaid_index_load(const char *path, int device, plaid_index **out)
{
    if (!path || !out) return fail(PLAID_EINVAL, "null argument");
    *out = nullptr;
    FILE *f = fopen(path, "rb");
    if (!f) return fail(PLAID_EIO, "cannot open %s", path);
    FileHeader h;
    if (fread(&h, 1, sizeof(h), f) != sizeof(h) || memcmp(h.magic, kMagic, 8) != 0) {
        fclose(f);
        return fail(PLAID_EFORMAT, "%s is not a PLAID index file", path);
    }
    int rc = check_sizes(h.dim, h.nbits, h.C, h.P, h.N, h.ivf_len);
    if (rc) {
        fclose(f);
        return rc == PLAID_EINVAL ? fail(PLAID_EFORMAT, "bad header in %s: %s", path, std::string(g_err).c_str()) : rc;
    }
    const size_t rb = (size_t)16 * h.nbits;
    if (h.N >= (1ll << 56) || h.ivf_len >= (1ll << 56)) {
        fclose(f);
        return fail(PLAID_EFORMAT, "bad header in %s: counts out of range", path);
    }
    const size_t sizes[7] = {(size_t)h.C * PLAID_DIM * 4, (size_t)(h.P + 1) * 8, (size_t)h.N * 4, (size_t)h.N * rb,
                             (size_t)(1 << h.nbits) * 4, (size_t)(h.C + 1) * 8, (size_t)h.ivf_len * 4};
    // the sections the header announces must fit the file: checked before anything is allocated for them
    {
        unsigned long long need = sizeof(FileHeader);
        for (int s = 0; s < 7; ++s) need += (sizes[s] + 63) & ~(size_t)63;
        long long have = -1;
        if (fseek(f, 0, SEEK_END) == 0) have = ftell(f);
        if (have < 0 || fseek(f, (long)sizeof(FileHeader), SEEK_SET) != 0) {
            fclose(f);
            return fail(PLAID_EIO, "cannot determine the size of %s", path);
        }
        if ((unsigned long long)have < need) {
            fclose(f);
            return fail(PLAID_EFORMAT, "index file truncated: header announces %llu bytes, %s holds %lld", need, path, have);
        }
    }
    std::vector<char> sec[7];
    for (int s = 0; s < 7; ++s) {
        rc = read_section(f, sec[s], sizes[s]);
        if (rc) {
            fclose(f);
            return rc;
        }
    }
    fclose(f);
    plaid_index_view v;
    memset(&v, 0, sizeof(v));
    v.dim = h.dim;
    v.nbits = h.nbits;
    v.num_centroids = h.C;
    v.num_passages = h.P;
    v.num_embeddings = h.N;
    v.centroids = (const float *)sec[0].data();
    v.doc_offsets = (const int64_t *)sec[1].data();
    v.codes = (const int32_t *)sec[2].data();
    v.residuals = (const uint8_t *)sec[3].data();
    v.bucket_weights = (const float *)sec[4].data();
    v.ivf_offsets = (const int64_t *)sec[5].data();
    v.ivf_pids = (const int32_t *)sec[6].data();
    v.on_device = 0;
    if (v.ivf_offsets[h.C] != h.ivf_len) return fail(PLAID_EFORMAT, "inverted-list length in header does not match offsets");
    rc = plaid_index_from_view(&v, device, 1, out);
    if (rc == PLAID_EINVAL) return fail(PLAID_EFORMAT, "malformed index in %s: %s", path, std::string(g_err).c_str());
    return rc;
}

extern "C" int plaid_index_info(const plaid_index *idx, int64_t *num_centroids, int64_t *num_passages,
                                int64_t *num_embeddings, int32_t *nbits, int64_t *ivf_len)
{
    if (!idx) return fail(PLAID_EINVAL, "null index");
    if (num_centroids) *num_centroids = idx->C;
    if (num_passages) *num_passages = idx->P;
    if (num_embeddings) *num_embeddings = idx->N;
    if (nbits) *nbits = idx->nbits;
    if (ivf_len) *ivf_len = idx->ivf_len;
    return PLAID_OK;
}

extern "C" int plaid_get_score_kernel(const plaid_index *idx, int32_t *form)
{
    if (!idx || !form) return fail(PLAID_EINVAL, "null argument");
    *form = idx->scq_form;
    return PLAID_OK;
}

extern "C" int plaid_get_stage2_kernel(const plaid_index *idx, int32_t *form)
{
    if (!idx || !form) return fail(PLAID_EINVAL, "null argument");
    *form = idx->ivr_table ? (idx->ivr_shift == 11 ? 1 : 2) : 0;
    return PLAID_OK;
}

extern "C" int plaid_set_stage_timing(plaid_index *idx, int32_t on)
{
    if (!idx) return fail(PLAID_EINVAL, "null index");
    if (on && !idx->ev[0]) {
        DeviceGuard g(idx->device);
        for (int i = 0; i < N_EVENTS; ++i) HIP_TRY(hipEventCreate(&idx->ev[i]));
    }
    if (on && !idx->score_clocks) {
        DeviceGuard g(idx->device);
        void *d = nullptr;
        if (hipMalloc(&d, 256) != hipSuccess) {
            (void)hipGetLastError();
            return fail(PLAID_ENOMEM, "hipMalloc(256) failed");
        }
        idx->owned.push_back(d);
        HIP_TRY(hipMemset(d, 0, 256));
        idx->score_clocks = (unsigned long long *)d;
    }
    idx->timing = on ? 1 : 0;
    return PLAID_OK;
}
extern "C" int plaid_get_score_kernel_clocks(const plaid_index *idx, uint64_t *out_ticks)
{
    if (!idx || !out_ticks) return fail(PLAID_EINVAL, "null argument");
    out_ticks[0] = out_ticks[1] = 0;
    if (!idx->score_clocks) return PLAID_OK;
    DeviceGuard g(idx->device);
    if (!g.ok) return fail(PLAID_EHIP, "hipSetDevice(%d) failed", idx->device);
    unsigned long long h[2] = {0, 0};
    HIP_TRY(hipMemcpy(h, idx->score_clocks, sizeof(h), hipMemcpyDeviceToHost));
    out_ticks[0] = h[0];
    out_ticks[1] = h[1];
    return PLAID_OK;
}
extern "C" int plaid_get_stage_ms(const plaid_index *idx, float *out_ms)
{
    if (!idx || !out_ms) return fail(PLAID_EINVAL, "null argument");
    for (int i = 0; i < PLAID_NUM_STAGES; ++i) out_ms[i] = idx->stage_ms[i];
    return PLAID_OK;
}
extern "C" int plaid_index_set_renormalize(plaid_index *idx, int32_t on)
{
    if (!idx) return fail(PLAID_EINVAL, "null index");
    if (on && !idx->inv_norm && idx->N > 0) {
        DeviceGuard g(idx->device);
        if (!g.ok) return fail(PLAID_EHIP, "hipSetDevice(%d) failed", idx->device);
        void *d = nullptr;
        if (hipMalloc(&d, (size_t)idx->N * sizeof(float)) != hipSuccess) {
            (void)hipGetLastError();
            return fail(PLAID_ENOMEM, "hipMalloc(%zu) for the tokens' scaling factors failed", (size_t)idx->N * sizeof(float));
        }
        idx->owned.push_back(d);
        plaid_launch_token_inv_norm(nullptr, idx->centroids, idx->codes, idx->residuals, idx->weights, idx->nbits, idx->N,
                                    (float *)d);
        HIP_TRY(hipGetLastError());
        HIP_TRY(hipStreamSynchronize(nullptr));
        idx->inv_norm = (float *)d;
    }
    idx->renormalize = on != 0 && idx->N > 0;
    return PLAID_OK;
}
extern "C" int plaid_set_max_chunk(plaid_index *idx, int32_t max_queries_per_chunk)
{
    if (!idx || max_queries_per_chunk < 0) return fail(PLAID_EINVAL, "bad argument");
    idx->max_chunk = max_queries_per_chunk;
    return PLAID_OK;
}

// ------------------------------------------------------------------ workspace of one query chunk
struct Workspace {
    // region that must be zero before each chunk
    char *zero_base;
    size_t zero_bytes;
    uint32_t *candbits;  // [qc][cand_words]
    Stage2Buffers s2;    // n_ne, hist, hist1, hist2, state live in the zeroed region
    void *sel3_zero, *sel4_zero;
    // everything else
    double *Qd;          // [qc][128][32]
    float *S;            // [qc][C][32]
    uint32_t *keepbits;  // [qc][keep_words]
    uint32_t *ambbits;   // [qc][keep_words] rows whose pruning test the split-fp16 scores leave open
    int32_t *probed;     // [qc][32][nprobe]
    int32_t *uniq;       // [qc][uniq_stride]
    int32_t *n_uniq;     // [qc]
    void *probe_scratch;
    size_t probe_scratch_bytes;
    float *tilemax;      // [qc][tiles][32] column maxima of the score kernel's tiles
    uint64_t *keys2;  // [qc][P]
    uint64_t *sel2;   // [qc][nd]
    int32_t *n2;      // [qc]
    uint64_t *keys3;  // [qc][nd]
    uint64_t *sel3;   // [qc][m3]
    int32_t *n3;      // [qc]
    uint64_t *keys4;  // [qc][m3]
    uint64_t *topk;   // [qc][kk]
    int32_t *n_out;   // [qc]
    void *sel3_body, *sel4_body;
    int64_t keep_words, cand_words;
    int uniq_stride;
    size_t total;
};

struct Plan {
    int32_t nprobe, nd, m3, kk;  // effective sizes: nd = min(ndocs, P), m3 = min(max(1, ndocs/4), nd), kk = min(k, m3)
};

static Plan make_plan(int64_t P, int32_t nprobe, int32_t ndocs, int32_t k)
{
    Plan pl;
    pl.nprobe = nprobe;
    pl.nd = (int32_t)(ndocs < P ? ndocs : P);
    const int32_t m3 = ndocs / 4 > 1 ? ndocs / 4 : 1;
    pl.m3 = m3 < pl.nd ? m3 : pl.nd;
    pl.kk = k < pl.m3 ? k : pl.m3;
    return pl;
}

static Workspace carve(char *base, const plaid_index *ix, int qc, const Plan &pl)
{
    Workspace w;
    memset(&w, 0, sizeof(w));
    const int64_t C = ix->C, P = ix->P;
    w.keep_words = (C + 31) / 32;
    w.cand_words = (P + 31) / 32;
    const int64_t up = (int64_t)QLEN * pl.nprobe;
    w.uniq_stride = (int)(up < C ? up : C);
    size_t off = 0;
    auto take = [&](size_t bytes) {
        char *p = base ? base + off : nullptr;
        off += a256(bytes);
        return p;
    };
    w.zero_base = take(0);
    w.candbits = (uint32_t *)take((size_t)qc * w.cand_words * 4);
    w.s2.hist = (int32_t *)take((size_t)qc * SEL_BINS * 4);
    w.s2.hist1 = (int32_t *)take((size_t)qc * SEL_BINS * 4);
    w.s2.hist2 = (int32_t *)take((size_t)qc * SEL_BINS * 4);
    w.s2.state = (Sel2State *)take((size_t)qc * sizeof(Sel2State));
    w.s2.qcount = (int32_t *)take(4 * sizeof(int32_t));
    w.sel3_zero = take(plaid_select_zero_bytes(qc));
    w.sel4_zero = take(plaid_select_zero_bytes(qc));
    w.zero_bytes = off;
    w.Qd = (double *)take((size_t)qc * QLEN * DIM * 8);
    w.S = ix->no_scores ? nullptr : (float *)take((size_t)qc * C * QLEN * 4);
    w.keepbits = (uint32_t *)take((size_t)qc * w.keep_words * 4);
    w.ambbits = (uint32_t *)take((size_t)qc * w.keep_words * 4);
    w.probed = (int32_t *)take((size_t)qc * QLEN * pl.nprobe * 4);
    w.uniq = (int32_t *)take((size_t)qc * w.uniq_stride * 4);
    w.n_uniq = (int32_t *)take((size_t)qc * 4);
    w.probe_scratch_bytes = plaid_top_nprobe_scratch_bytes(C, qc, pl.nprobe);
    w.probe_scratch = take(w.probe_scratch_bytes);
    w.tilemax = (float *)take(plaid_stage1_tilemax_bytes(C, qc, pl.nprobe));
    w.keys2 = (uint64_t *)take((size_t)qc * P * 8);
    w.s2.blist = (uint64_t *)take((size_t)qc * P * 8);
    w.s2.meta = (S2Meta *)take((size_t)qc * sizeof(S2Meta));
    w.s2.kept_ids = (int32_t *)take((size_t)qc * S2_MAX_KEPT * 4);
    w.s2.T = (float *)take((size_t)qc * (S2_MAX_KEPT + 1) * QLEN * 4);
    w.s2.emptybits = (uint32_t *)take((size_t)qc * w.cand_words * 4);
    w.s2.qlist = (int32_t *)take((size_t)3 * qc * 4);
    w.s2.qlist_stride = qc;
    w.s2.ivf_offsets = ix->ivf_offsets;
    w.sel2 = (uint64_t *)take((size_t)qc * pl.nd * 8);
    w.n2 = (int32_t *)take((size_t)qc * 4);
    w.keys3 = (uint64_t *)take((size_t)qc * pl.nd * 8);
    w.sel3 = (uint64_t *)take((size_t)qc * pl.m3 * 8);
    w.n3 = (int32_t *)take((size_t)qc * 4);
    w.keys4 = (uint64_t *)take((size_t)qc * pl.m3 * 8);
    w.topk = (uint64_t *)take((size_t)qc * pl.kk * 8);
    w.n_out = (int32_t *)take((size_t)qc * 4);
    w.sel3_body = take(plaid_select_body_bytes(qc, pl.nd, pl.m3));
    w.sel4_body = take(plaid_select_body_bytes(qc, pl.m3, pl.kk));
    w.total = off;
    return w;
}

// Queries per chunk: bounded by the caller's limit, else 512 (the kernels that run one workgroup per query only fill
// the chip from a few hundred queries on) within a workspace budget of about 24 GiB.
static int choose_chunk(const plaid_index *ix, int32_t nq, const Plan &pl)
{
    const Workspace one = carve(nullptr, ix, 1, pl);
    int qc = ix->max_chunk > 0 ? ix->max_chunk : 512;
    if (ix->max_chunk <= 0) {
        const size_t budget = (size_t)24 << 30;
        const size_t fit = budget / (one.total ? one.total : 1);
        if ((size_t)qc > fit) qc = fit < 1 ? 1 : (int)fit;
    }
    if (qc > nq) qc = nq;
    if ((int64_t)qc * QLEN > 32768) qc = 32768 / QLEN;  // grid.y / segment limits of the per-token selections
    return qc;
}

static int ensure_workspace(plaid_index *ix, size_t bytes)
{
    if (ix->ws_bytes >= bytes) return PLAID_OK;
    if (ix->ws) {
        HIP_TRY(hipDeviceSynchronize());
        (void)hipFree(ix->ws);
        ix->ws = nullptr;
        ix->ws_bytes = 0;
    }
    void *p = nullptr;
    hipError_t e = hipMalloc(&p, bytes);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return fail(PLAID_ENOMEM, "workspace of %zu bytes: %s", bytes, hipGetErrorString(e));
    }
    ix->ws = p;
    ix->ws_bytes = bytes;
    return PLAID_OK;
}

// ------------------------------------------------------------------ search
// fixed_ws: null = the per-index workspace (allocated and grown here); otherwise the static array of fixed_bytes bytes:
// nothing is allocated, and the chunk shrinks until its workspace fits.
static int search_impl(plaid_index *ix, const float *Q, int32_t nq, int32_t nprobe, float t_cs, int32_t ndocs, int32_t k,
                       int32_t *out_ids, float *out_scores, void *hip_stream, const plaid_debug_buffers *dbg,
                       char *fixed_ws = nullptr, size_t fixed_bytes = 0)
{
    if (!ix) return fail(PLAID_EINVAL, "null index");
    if (!Q || !out_ids || !out_scores) return fail(PLAID_EINVAL, "null buffer");
    if ((uintptr_t)Q & 15) return fail(PLAID_EINVAL, "Q must be aligned to 16 bytes");
    if (nq < 1) return fail(PLAID_EINVAL, "nq must be >= 1 (got %d)", nq);
    if (nprobe < 1 || nprobe > ix->C) return fail(PLAID_EINVAL, "nprobe must be in [1, C] (got %d, C = %lld)", nprobe, (long long)ix->C);
    if (ndocs < 1) return fail(PLAID_EINVAL, "ndocs must be >= 1 (got %d)", ndocs);
    if (k < 1) return fail(PLAID_EINVAL, "k must be >= 1 (got %d)", k);
    if (t_cs != t_cs) return fail(PLAID_EINVAL, "t_cs is NaN");
    DeviceGuard g(ix->device);
    if (!g.ok) return fail(PLAID_EHIP, "hipSetDevice(%d) failed", ix->device);
    hipStream_t st = (hipStream_t)hip_stream;

    const int64_t C = ix->C, P = ix->P;
    const int32_t m3 = ndocs / 4 > 1 ? ndocs / 4 : 1;
    const Plan pl = make_plan(P, nprobe, ndocs, k);
    int qc = choose_chunk(ix, nq, pl);
    char *ws_base = nullptr;
    if (fixed_ws) {
        while (qc > 1 && carve(nullptr, ix, qc, pl).total > fixed_bytes) qc = qc > 2 ? qc - (qc + 7) / 8 : 1;
        const size_t need = carve(nullptr, ix, qc, pl).total;
        if (need > fixed_bytes)
            return fail(PLAID_EINVAL, "one query of this search needs %zu bytes of workspace, the static workspace holds %zu", need,
                        fixed_bytes);
        ws_base = fixed_ws;
    } else {
        const Workspace wsz = carve(nullptr, ix, qc, pl);
        const int rc = ensure_workspace(ix, wsz.total);
        if (rc) return rc;
        ws_base = (char *)ix->ws;
    }

    // the split-fp16 kernel pairs with the fast probe kernel only: larger nprobe values take a double-precision form
    const int form = (ix->scq_form == PLAID_SCQ_SPLIT16 && nprobe > PLAID_PROBE_FAST_MAX)
                         ? (ix->scq_matrix_form ? PLAID_SCQ_MATRIX : PLAID_SCQ_VECTOR)
                         : ix->scq_form;
    const bool timing = ix->timing != 0;
    if (timing) {
        for (int s = 0; s < PLAID_NUM_STAGES; ++s) ix->stage_ms[s] = 0.f;
        if (ix->score_clocks) HIP_TRY(hipMemsetAsync(ix->score_clocks, 0, 16, st));
    }

    for (int32_t q0 = 0; q0 < nq; q0 += qc) {
        const int n = nq - q0 < qc ? nq - q0 : qc;
        const Workspace w = carve(ws_base, ix, n, pl);
        const float *Qc = Q + (int64_t)q0 * QLEN * DIM;
        const SelScratch sc3 = plaid_select_scratch_carve2(w.sel3_zero, w.sel3_body, n, pl.nd, pl.m3);
        const SelScratch sc4 = plaid_select_scratch_carve2(w.sel4_zero, w.sel4_body, n, pl.m3, pl.kk);
        int e = 0;
#define STAMP()                                            \
    do {                                                   \
        if (timing) HIP_TRY(hipEventRecord(ix->ev[e++], st)); \
    } while (0)

        STAMP();
        // stage 1: S_cq (Eq. 2), pruning map (Eq. 5), probes and candidates (Section 4.1)
        for (int phase = PLAID_STAGE1_PREP; phase <= PLAID_STAGE1_PROBES; phase <<= 1) {
            plaid_launch_stage1(st, phase, ix->centroids, C, Qc, w.Qd, form, ix->A16, n, t_cs, nprobe, w.S, w.keepbits, w.ambbits,
                                w.keep_words, w.tilemax, (uint32_t *)w.zero_base, (int64_t)(w.zero_bytes / 4), w.probed,
                                w.uniq, w.uniq_stride, w.n_uniq, w.s2, w.probe_scratch, w.probe_scratch_bytes,
                                timing ? ix->score_clocks : nullptr);
            STAMP();
        }
        if (!ix->ivr_table)
            plaid_launch_ivf_union(st, w.uniq, w.n_uniq, w.uniq_stride, ix->ivf_offsets, ix->ivf_pids, n, w.candbits,
                                   w.cand_words);
        STAMP();
        // stage 2: centroid interaction with pruning over every candidate (Eq. 3-5), keep ndocs
        if (ix->ivr_table)
            plaid_launch_stage2_inverted(st, w.uniq, w.n_uniq, w.uniq_stride, ix->ivf_offsets, ix->ivf_pids, ix->ivr_table, w.S,
                                         C, w.keepbits, w.keep_words, ix->codes, ix->doc_offsets, P, n, w.s2, w.candbits,
                                         w.cand_words, w.keys2, P, ix->dense_id, ix->dense_bits, ix->ivr_shift);
        else
            plaid_launch_stage2(st, w.S, C, w.keepbits, w.keep_words, w.probed, nprobe, w.candbits, w.cand_words, P, ix->N,
                                ix->doc_offsets, ix->codes, n, w.s2, w.keys2, P);
        STAMP();
        plaid_launch_select2(st, w.keys2, P, w.candbits, n, P, w.cand_words, pl.nd, w.s2, w.sel2, pl.nd, w.n2);
        STAMP();
        // stage 3: centroid interaction without pruning (Eq. 3-4), keep ndocs/4
        plaid_launch_ci_list(st, w.S, C, ix->doc_offsets, ix->codes, n, w.sel2, pl.nd, w.n2, pl.nd, w.keys3, pl.nd);
        STAMP();
        plaid_launch_select(st, w.keys3, pl.nd, w.n2, n, pl.nd, pl.m3, w.sel3, pl.m3, w.n3, 0, sc3, 0);
        STAMP();
        // stage 4: decompression (Section 4.5) + exact MaxSim (Eq. 1), best k
        plaid_launch_decompress_maxsim(st, Qc, w.S, C, ix->doc_offsets, ix->codes, ix->residuals, ix->weights,
                                       ix->nbits, n, w.sel3, pl.m3, w.n3, pl.m3, w.keys4, pl.m3,
                                       ix->renormalize ? ix->inv_norm : nullptr);
        STAMP();
        if (pl.m3 <= SEL_SORT_CAP) {
            plaid_launch_rank_output(st, w.keys4, pl.m3, w.n3, n, pl.m3, k, out_ids + (int64_t)q0 * k,
                                     out_scores + (int64_t)q0 * k);
        } else {
            plaid_launch_select(st, w.keys4, pl.m3, w.n3, n, pl.m3, pl.kk, w.topk, pl.kk, w.n_out, 1, sc4, 0);
            plaid_launch_keys_to_output(st, w.topk, pl.kk, w.n_out, n, k, out_ids + (int64_t)q0 * k,
                                        out_scores + (int64_t)q0 * k);
        }
        STAMP();
#undef STAMP
        HIP_TRY(hipGetLastError());

        if (dbg) {
            if (dbg->S_cq)
                HIP_TRY(hipMemcpyAsync(dbg->S_cq + (int64_t)q0 * C * QLEN, w.S, (size_t)n * C * QLEN * 4,
                                       hipMemcpyDeviceToDevice, st));
            if (dbg->keep)
                HIP_TRY(hipMemcpyAsync(dbg->keep + (int64_t)q0 * w.keep_words, w.keepbits, (size_t)n * w.keep_words * 4,
                                       hipMemcpyDeviceToDevice, st));
            if (dbg->probed)
                HIP_TRY(hipMemcpyAsync(dbg->probed + (int64_t)q0 * QLEN * nprobe, w.probed, (size_t)n * QLEN * nprobe * 4,
                                       hipMemcpyDeviceToDevice, st));
            if (dbg->cand || dbg->n_cand)
                plaid_launch_bitmap_to_list(st, w.candbits, w.cand_words, P, n, dbg->cand ? dbg->cand + (int64_t)q0 * P : nullptr,
                                            P, dbg->n_cand ? dbg->n_cand + q0 : nullptr);
            if (dbg->sel2_ids || dbg->sel2_scores || dbg->n2)
                plaid_launch_keys_to_pairs(st, w.sel2, pl.nd, w.n2, n, ndocs,
                                           dbg->sel2_ids ? dbg->sel2_ids + (int64_t)q0 * ndocs : nullptr,
                                           dbg->sel2_scores ? dbg->sel2_scores + (int64_t)q0 * ndocs : nullptr,
                                           dbg->n2 ? dbg->n2 + q0 : nullptr);
            if (dbg->sel3_ids || dbg->sel3_scores || dbg->n3)
                plaid_launch_keys_to_pairs(st, w.sel3, pl.m3, w.n3, n, m3,
                                           dbg->sel3_ids ? dbg->sel3_ids + (int64_t)q0 * m3 : nullptr,
                                           dbg->sel3_scores ? dbg->sel3_scores + (int64_t)q0 * m3 : nullptr,
                                           dbg->n3 ? dbg->n3 + q0 : nullptr);
            HIP_TRY(hipGetLastError());
        }
        if (timing) {
            HIP_TRY(hipEventSynchronize(ix->ev[e - 1]));
            for (int s = 0; s + 1 < e && s < PLAID_NUM_STAGES; ++s) {
                float ms = 0.f;
                HIP_TRY(hipEventElapsedTime(&ms, ix->ev[s], ix->ev[s + 1]));
                ix->stage_ms[s] += ms;
            }
        }
    }
    return PLAID_OK;
}

extern "C" int plaid_search(plaid_index *idx, const float *Q, int32_t nq, int32_t nprobe, float t_cs, int32_t ndocs,
                            int32_t k, int32_t *out_ids, float *out_scores, void *hip_stream)
{
    return search_impl(idx, Q, nq, nprobe, t_cs, ndocs, k, out_ids, out_scores, hip_stream, nullptr);
}

extern "C" int plaid_search_debug(plaid_index *idx, const float *Q, int32_t nq, int32_t nprobe, float t_cs, int32_t ndocs,
                                  int32_t k, int32_t *out_ids, float *out_scores, void *hip_stream,
                                  const plaid_debug_buffers *dbg)
{
    return search_impl(idx, Q, nq, nprobe, t_cs, ndocs, k, out_ids, out_scores, hip_stream, dbg);
}

extern "C" int plaid_search_static(plaid_index *idx, const float *Q, int32_t nq, int32_t nprobe, float t_cs, int32_t ndocs,
                                   int32_t k, int32_t *out_ids, float *out_scores, void *hip_stream)
{
    if (!idx) return fail(PLAID_EINVAL, "null index");
    if (!idx->static_ws) return fail(PLAID_EHIP, "the static workspace has no address on device %d", idx->device);
    return search_impl(idx, Q, nq, nprobe, t_cs, ndocs, k, out_ids, out_scores, hip_stream, nullptr, idx->static_ws,
                       PLAID_STATIC_WORKSPACE_BYTES);
}

// ------------------------------------------------------------------ vanilla ColBERTv2 retrieval (the paper's baseline)
static int ensure_vanilla_structures(plaid_index *ix)
{
    if (ix->emb_offsets) return PLAID_OK;
    if (ix->N >= (1ll << 31)) return fail(PLAID_EINVAL, "vanilla retrieval needs fewer than 2^31 embeddings (index has %lld)", (long long)ix->N);
    HIP_TRY(hipDeviceSynchronize());
    void *off = nullptr, *ids = nullptr, *t2p = nullptr, *scratch = nullptr;
    const size_t sb = plaid_embedding_lists_scratch_bytes(ix->N, ix->C) + 256;
    const size_t nb = (size_t)(ix->N > 0 ? ix->N : 1) * 4;
    if (hipMalloc(&off, (size_t)(ix->C + 1) * 8) != hipSuccess || hipMalloc(&ids, nb) != hipSuccess ||
        hipMalloc(&t2p, nb) != hipSuccess || hipMalloc(&scratch, sb) != hipSuccess) {
        (void)hipGetLastError();
        if (off) (void)hipFree(off);
        if (ids) (void)hipFree(ids);
        if (t2p) (void)hipFree(t2p);
        if (scratch) (void)hipFree(scratch);
        return fail(PLAID_ENOMEM, "device allocation for the embedding-level inverted lists failed");
    }
    ix->owned.push_back(off);
    ix->owned.push_back(ids);
    ix->owned.push_back(t2p);
    int32_t bad = 0;
    hipError_t e = hipMemset(scratch, 0, sb);
    if (e == hipSuccess) {
        int32_t *bad_d = (int32_t *)((char *)scratch + sb - 256);
        plaid_launch_embedding_lists(nullptr, ix->codes, ix->N, ix->C, scratch, (int64_t *)off, (int32_t *)ids, bad_d);
        plaid_launch_tok2pid(nullptr, ix->doc_offsets, ix->P, ix->N, (int32_t *)t2p);
        e = hipGetLastError();
        if (e == hipSuccess) e = hipMemcpy(&bad, bad_d, 4, hipMemcpyDeviceToHost);
    }
    (void)hipFree(scratch);
    if (e != hipSuccess) return fail(PLAID_EHIP, "building the embedding-level inverted lists: %s", hipGetErrorString(e));
    if (bad) return fail(PLAID_EINVAL, "a centroid id is outside [0, %lld)", (long long)ix->C);
    ix->emb_offsets = (int64_t *)off;
    ix->emb_ids = (int32_t *)ids;
    ix->tok2pid = (int32_t *)t2p;
    return PLAID_OK;
}

extern "C" int plaid_search_vanilla(plaid_index *ix, const float *Q, int32_t nq, int32_t nprobe, int32_t ncandidates, int32_t k,
                                    int32_t *out_ids, float *out_scores, void *hip_stream, const plaid_vanilla_debug *dbg)
{
    if (!ix) return fail(PLAID_EINVAL, "null index");
    if (!Q || !out_ids || !out_scores) return fail(PLAID_EINVAL, "null buffer");
    if ((uintptr_t)Q & 15) return fail(PLAID_EINVAL, "Q must be aligned to 16 bytes");
    if (nq < 1) return fail(PLAID_EINVAL, "nq must be >= 1 (got %d)", nq);
    if (nprobe < 1 || nprobe > ix->C) return fail(PLAID_EINVAL, "nprobe must be in [1, C] (got %d, C = %lld)", nprobe, (long long)ix->C);
    if (ncandidates < 1) return fail(PLAID_EINVAL, "ncandidates must be >= 1 (got %d)", ncandidates);
    if (k < 1) return fail(PLAID_EINVAL, "k must be >= 1 (got %d)", k);
    if (ix->renormalize)
        return fail(PLAID_EINVAL, "vanilla retrieval is not available while reconstructed vectors are scaled to unit length "
                                  "(plaid_index_set_renormalize)");
    DeviceGuard g(ix->device);
    if (!g.ok) return fail(PLAID_EHIP, "hipSetDevice(%d) failed", ix->device);
    int rc = ensure_vanilla_structures(ix);
    if (rc) return rc;
    hipStream_t st = (hipStream_t)hip_stream;
    const int64_t C = ix->C, P = ix->P;
    Plan pl;
    pl.nprobe = nprobe;
    pl.nd = (int32_t)(ncandidates < P ? ncandidates : P);  // candidates kept by the cap
    pl.m3 = pl.nd;
    pl.kk = k < pl.nd ? k : pl.nd;
    const int form = (ix->scq_form == PLAID_SCQ_SPLIT16 && nprobe > PLAID_PROBE_FAST_MAX)
                         ? (ix->scq_matrix_form ? PLAID_SCQ_MATRIX : PLAID_SCQ_VECTOR)
                         : ix->scq_form;
    const int qc = choose_chunk(ix, nq, pl);
    const Workspace wsz = carve(nullptr, ix, qc, pl);
    // beyond the search workspace: the state and the lists of the selection that applies the ncandidates cap
    const size_t selz = a256(plaid_select_zero_bytes(qc)), selb = a256(plaid_select_body_bytes(qc, P, pl.nd));
    rc = ensure_workspace(ix, wsz.total + selz + selb);
    if (rc) return rc;
    for (int32_t q0 = 0; q0 < nq; q0 += qc) {
        const int n = nq - q0 < qc ? nq - q0 : qc;
        const Workspace w = carve((char *)ix->ws, ix, n, pl);
        char *extra = (char *)ix->ws + wsz.total;
        const SelScratch scp = plaid_select_scratch_carve2(extra, extra + selz, n, P, pl.nd);
        const SelScratch sc4 = plaid_select_scratch_carve2(w.sel4_zero, w.sel4_body, n, pl.m3, pl.kk);
        const float *Qc = Q + (int64_t)q0 * QLEN * DIM;
        // Eq. 2 and the probes, as in plaid_search (no pruning map is needed: t_cs = +infinity)
        for (int phase = PLAID_STAGE1_PREP; phase <= PLAID_STAGE1_PROBES; phase <<= 1)
            plaid_launch_stage1(st, phase, ix->centroids, C, Qc, w.Qd, form, ix->A16, n, INFINITY, nprobe, w.S, w.keepbits, w.ambbits,
                                w.keep_words, w.tilemax, (uint32_t *)w.zero_base, (int64_t)(w.zero_bytes / 4), w.probed, w.uniq,
                                w.uniq_stride, w.n_uniq, w.s2, w.probe_scratch, w.probe_scratch_bytes);
        // candidate passages from the embedding lists of the probed centroids (Section 4.1)
        uint32_t *probebits = w.ambbits;       // free once the probes are known
        int32_t *cand = (int32_t *)w.s2.blist;  // [n][P]
        plaid_launch_fill_u32(st, probebits, (int64_t)n * w.keep_words, 0u);
        plaid_launch_fill_u32(st, (uint32_t *)scp.state, (int64_t)(plaid_select_zero_bytes(n) / 4), 0u);
        plaid_launch_vanilla_candidates(st, w.uniq, w.n_uniq, w.uniq_stride, ix->emb_offsets, ix->emb_ids, ix->tok2pid, n,
                                        w.keep_words, probebits, w.candbits, w.cand_words);
        plaid_launch_bitmap_to_list(st, w.candbits, w.cand_words, P, n, cand, P, w.n2);
        // more than ncandidates: scored on the embeddings of the probed lists alone, the best ncandidates stay
        plaid_launch_vanilla_prune(st, Qc, w.S, C, ix->doc_offsets, ix->codes, ix->residuals, ix->weights, ix->nbits, probebits,
                                   w.keep_words, n, cand, P, w.n2, P, pl.nd, w.keys2, P);
        plaid_launch_select(st, w.keys2, P, w.n2, n, P, pl.nd, w.sel2, pl.nd, w.n3, 0, scp, 0);
        // every token of every remaining candidate: decompression + exact MaxSim (Section 3.2, Eq. 1), best k
        plaid_launch_decompress_maxsim(st, Qc, w.S, C, ix->doc_offsets, ix->codes, ix->residuals, ix->weights, ix->nbits, n,
                                       w.sel2, pl.nd, w.n3, pl.nd, w.keys4, pl.m3);
        if (pl.m3 <= SEL_SORT_CAP) {
            plaid_launch_rank_output(st, w.keys4, pl.m3, w.n3, n, pl.m3, k, out_ids + (int64_t)q0 * k, out_scores + (int64_t)q0 * k);
        } else {
            plaid_launch_select(st, w.keys4, pl.m3, w.n3, n, pl.m3, pl.kk, w.topk, pl.kk, w.n_out, 1, sc4, 0);
            plaid_launch_keys_to_output(st, w.topk, pl.kk, w.n_out, n, k, out_ids + (int64_t)q0 * k, out_scores + (int64_t)q0 * k);
        }
        HIP_TRY(hipGetLastError());
        if (dbg) {
            if (dbg->cand)
                HIP_TRY(hipMemcpy2DAsync(dbg->cand + (int64_t)q0 * P, (size_t)P * 4, cand, (size_t)P * 4, (size_t)P * 4, n,
                                         hipMemcpyDeviceToDevice, st));
            if (dbg->n_cand) HIP_TRY(hipMemcpyAsync(dbg->n_cand + q0, w.n2, (size_t)n * 4, hipMemcpyDeviceToDevice, st));
            if (dbg->kept_ids || dbg->kept_scores || dbg->n_kept)
                plaid_launch_keys_to_pairs(st, w.sel2, pl.nd, w.n3, n, ncandidates,
                                           dbg->kept_ids ? dbg->kept_ids + (int64_t)q0 * ncandidates : nullptr,
                                           dbg->kept_scores ? dbg->kept_scores + (int64_t)q0 * ncandidates : nullptr,
                                           dbg->n_kept ? dbg->n_kept + q0 : nullptr);
            HIP_TRY(hipGetLastError());
        }
    }
    return PLAID_OK;
}

// ------------------------------------------------------------------ workspace size (host arithmetic only)
extern "C" int plaid_workspace_bytes(int64_t C, int64_t P, int32_t nq, int32_t nprobe, int32_t ndocs, int32_t k,
                                     int32_t max_queries_per_chunk, int64_t *bytes, int32_t *queries_per_chunk)
{
    if (!bytes) return fail(PLAID_EINVAL, "null output");
    if (C < 1 || C >= (1ll << 31)) return fail(PLAID_EINVAL, "num_centroids out of range (%lld)", (long long)C);
    if (P < 1 || P >= (1ll << 31)) return fail(PLAID_EINVAL, "num_passages out of range (%lld)", (long long)P);
    if (nq < 1 || nprobe < 1 || nprobe > C || ndocs < 1 || k < 1 || max_queries_per_chunk < 0)
        return fail(PLAID_EINVAL, "search parameters out of range");
    plaid_index fake;
    fake.C = C;
    fake.P = P;
    fake.max_chunk = max_queries_per_chunk;
    const Plan pl = make_plan(P, nprobe, ndocs, k);
    const int qc = choose_chunk(&fake, nq, pl);
    *bytes = (int64_t)carve(nullptr, &fake, qc, pl).total;
    if (queries_per_chunk) *queries_per_chunk = qc;
    return PLAID_OK;
}

// ------------------------------------------------------------------ index construction
extern "C" int plaid_assign_centroids(const float *centroids, int64_t C, const float *x, int64_t n, int32_t *codes, int device,
                                      void *hip_stream)
{
    if (!centroids || (n > 0 && (!x || !codes))) return fail(PLAID_EINVAL, "null buffer");
    if (C < 1 || C >= (1ll << 31)) return fail(PLAID_EINVAL, "num_centroids out of range (%lld)", (long long)C);
    if (n < 0) return fail(PLAID_EINVAL, "negative vector count");
    if (((uintptr_t)centroids | (uintptr_t)x) & 15) return fail(PLAID_EINVAL, "centroids and x must be aligned to 16 bytes");
    if (n == 0) return PLAID_OK;
    DeviceGuard g(device);
    if (!g.ok) return fail(PLAID_EHIP, "hipSetDevice(%d) failed", device);
    hipStream_t st = (hipStream_t)hip_stream;
    // the score kernel of the search path, 32 vectors in the place of a query's 32 tokens, and its top-1 probes
    plaid_index fake;
    fake.device = device;
    fake.C = C;
    fake.P = 1;
    int rc = choose_scq_form(&fake);
    if (rc) return rc;
    if (fake.scq_form == PLAID_SCQ_SPLIT16) {
        rc = scq16_check_centroids(&fake, centroids, C, st);
        if (rc) return rc;
    }
    TempAlloc a16;
    if (fake.scq_form == PLAID_SCQ_SPLIT16) {
        const size_t ab = plaid_scq16_centroid_bytes(C);
        if (hipMalloc(&a16.p, ab) != hipSuccess) {
            (void)hipGetLastError();
            return fail(PLAID_ENOMEM, "hipMalloc(%zu) for the centroids' matrix operands failed", ab);
        }
        plaid_launch_scq16_split_centroids(st, centroids, C, a16.p);
        // The probe kernel ranks by scores it re-evaluates in double and needs the tile maxima only to find the rows worth
        // re-evaluating: the scores themselves (4 C bytes per vector, the kernel's whole memory traffic) are not stored.
        fake.no_scores = true;
    }
    Plan pl;
    pl.nprobe = 1;
    pl.nd = pl.m3 = pl.kk = 1;
    const int64_t groups = (n + QLEN - 1) / QLEN;
    const Workspace one = carve(nullptr, &fake, 1, pl);
    int64_t qc = (int64_t)(((size_t)4 << 30) / (one.total ? one.total : 1));  // about 4 GiB of workspace
    if (qc > 512) qc = 512;
    if (qc > groups) qc = groups;
    if (qc < 1) qc = 1;
    const Workspace wsz = carve(nullptr, &fake, (int)qc, pl);
    TempAlloc ws, tailbuf;
    if (hipMalloc(&ws.p, wsz.total) != hipSuccess) {
        (void)hipGetLastError();
        return fail(PLAID_ENOMEM, "hipMalloc(%zu) for the assignment workspace failed", wsz.total);
    }
    const int64_t tail = n % QLEN;  // vectors of a last, incomplete group: staged in a zero-padded buffer
    if (tail) {
        if (hipMalloc(&tailbuf.p, (size_t)QLEN * DIM * 4) != hipSuccess) {
            (void)hipGetLastError();
            return fail(PLAID_ENOMEM, "hipMalloc for the assignment tail failed");
        }
        HIP_TRY(hipMemsetAsync(tailbuf.p, 0, (size_t)QLEN * DIM * 4, st));
        HIP_TRY(hipMemcpyAsync(tailbuf.p, x + (n - tail) * DIM, (size_t)tail * DIM * 4, hipMemcpyDeviceToDevice, st));
    }
    const int64_t full = n / QLEN;
    // ng groups of 32 vectors from src -> the first cnt of their codes to dst
    auto run = [&](const float *src, int64_t ng, int32_t *dst, int64_t cnt) -> int {
        const Workspace w = carve((char *)ws.p, &fake, (int)ng, pl);
        for (int phase = PLAID_STAGE1_PREP; phase <= PLAID_STAGE1_PROBES; phase <<= 1)
            plaid_launch_stage1(st, phase, centroids, C, src, w.Qd, fake.scq_form, a16.p, (int)ng, INFINITY, 1, w.S, w.keepbits,
                                w.ambbits, w.keep_words, w.tilemax, (uint32_t *)w.zero_base, (int64_t)(w.zero_bytes / 4), w.probed,
                                w.uniq, w.uniq_stride, w.n_uniq, w.s2, w.probe_scratch, w.probe_scratch_bytes);
        HIP_TRY(hipGetLastError());
        HIP_TRY(hipMemcpyAsync(dst, w.probed, (size_t)cnt * 4, hipMemcpyDeviceToDevice, st));  // probed is [group][32][1]
        return PLAID_OK;
    };
    for (int64_t g0 = 0; g0 < full; g0 += qc) {
        const int64_t ng = full - g0 < qc ? full - g0 : qc;
        rc = run(x + g0 * QLEN * DIM, ng, codes + g0 * QLEN, ng * QLEN);
        if (rc) return rc;
    }
    if (tail) {
        rc = run((const float *)tailbuf.p, 1, codes + full * QLEN, tail);
        if (rc) return rc;
    }
    HIP_TRY(hipStreamSynchronize(st));  // the workspace is released on return
    return PLAID_OK;
}

extern "C" int plaid_encode_residuals(const float *centroids, int64_t C, const float *x, const int32_t *codes, int64_t n,
                                      const float *cutoffs, int32_t nbits, uint8_t *residuals, int device, void *hip_stream)
{
    if (!centroids || !cutoffs || (n > 0 && (!x || !codes || !residuals))) return fail(PLAID_EINVAL, "null buffer");
    if (nbits != 1 && nbits != 2) return fail(PLAID_EINVAL, "nbits must be 1 or 2 (got %d)", nbits);
    if (C < 1 || C >= (1ll << 31)) return fail(PLAID_EINVAL, "num_centroids out of range (%lld)", (long long)C);
    if (n < 0) return fail(PLAID_EINVAL, "negative vector count");
    if (((uintptr_t)centroids | (uintptr_t)x) & 15) return fail(PLAID_EINVAL, "centroids and x must be aligned to 16 bytes");
    if ((uintptr_t)residuals & 3) return fail(PLAID_EINVAL, "residuals must be aligned to 4 bytes");
    if (n == 0) return PLAID_OK;
    DeviceGuard g(device);
    if (!g.ok) return fail(PLAID_EHIP, "hipSetDevice(%d) failed", device);
    hipStream_t st = (hipStream_t)hip_stream;
    TempAlloc flag;
    if (hipMalloc(&flag.p, 4) != hipSuccess) {
        (void)hipGetLastError();
        return fail(PLAID_ENOMEM, "hipMalloc failed");
    }
    HIP_TRY(hipMemsetAsync(flag.p, 0, 4, st));
    plaid_launch_encode_residuals(st, centroids, C, x, codes, n, cutoffs, nbits, residuals, (int32_t *)flag.p);
    HIP_TRY(hipGetLastError());
    int32_t bad = 0;
    HIP_TRY(hipMemcpyAsync(&bad, flag.p, 4, hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    if (bad) return fail(PLAID_EINVAL, "a centroid id is outside [0, %lld)", (long long)C);
    return PLAID_OK;
}

extern "C" int plaid_build_ivf(const int32_t *codes, const int64_t *doc_offsets, int64_t P, int64_t N, int64_t C,
                               int64_t *ivf_offsets, int32_t *ivf_pids, int64_t capacity, int64_t *ivf_len, int device,
                               void *hip_stream)
{
    if (!doc_offsets || !ivf_offsets || (N > 0 && !codes)) return fail(PLAID_EINVAL, "null buffer");
    if (C < 1 || C >= (1ll << 31)) return fail(PLAID_EINVAL, "num_centroids out of range (%lld)", (long long)C);
    if (P < 1 || P >= (1ll << 31)) return fail(PLAID_EINVAL, "num_passages out of range (%lld)", (long long)P);
    if (N < 0 || capacity < 0) return fail(PLAID_EINVAL, "negative size");
    DeviceGuard g(device);
    if (!g.ok) return fail(PLAID_EHIP, "hipSetDevice(%d) failed", device);
    hipStream_t st = (hipStream_t)hip_stream;
    int64_t ends[2] = {0, 0};
    HIP_TRY(hipMemcpyAsync(&ends[0], doc_offsets, 8, hipMemcpyDeviceToHost, st));
    HIP_TRY(hipMemcpyAsync(&ends[1], doc_offsets + P, 8, hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    if (ends[0] != 0 || ends[1] != N) return fail(PLAID_EINVAL, "doc_offsets must run from 0 to num_embeddings (%lld)", (long long)N);
    // scratch: the list builder's area (counters first, they start at zero), then 256 bytes for the error flag
    const size_t sb = plaid_ivf_lists_scratch_bytes(N, C), zb = plaid_ivf_lists_scratch_zero_bytes(N, C);
    TempAlloc scratch;
    if (hipMalloc(&scratch.p, sb + 256) != hipSuccess) {
        (void)hipGetLastError();
        return fail(PLAID_ENOMEM, "hipMalloc(%zu) for the inverted-list scratch failed", sb);
    }
    HIP_TRY(hipMemsetAsync(scratch.p, 0, zb, st));
    int32_t *bad_d = (int32_t *)((char *)scratch.p + sb);
    HIP_TRY(hipMemsetAsync(bad_d, 0, 256, st));
    plaid_launch_ivf_build_offsets(st, codes, doc_offsets, P, N, C, scratch.p, ivf_offsets, bad_d);
    HIP_TRY(hipGetLastError());
    int32_t bad = 0;
    int64_t total = 0;
    HIP_TRY(hipMemcpyAsync(&bad, bad_d, 4, hipMemcpyDeviceToHost, st));
    HIP_TRY(hipMemcpyAsync(&total, ivf_offsets + C, 8, hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    if (bad) return fail(PLAID_EINVAL, "a centroid id is outside [0, %lld) or doc_offsets is not monotone within [0, N]", (long long)C);
    if (ivf_len) *ivf_len = total;
    if (!ivf_pids) return PLAID_OK;
    if (capacity < total) return fail(PLAID_EINVAL, "the inverted lists hold %lld entries, capacity is %lld", (long long)total, (long long)capacity);
    plaid_launch_ivf_build_fill(st, codes, doc_offsets, P, N, C, scratch.p, ivf_offsets, ivf_pids, capacity);
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipStreamSynchronize(st));  // the scratch area is released on return
    return PLAID_OK;
}

// ------------------------------------------------------------------ decompression alone
extern "C" int plaid_decompress_passages(plaid_index *ix, const int32_t *pids, int32_t n, int64_t *out_offsets,
                                         float *out_vectors, uint8_t *out_indices, int64_t capacity, void *hip_stream)
{
    if (!ix) return fail(PLAID_EINVAL, "null index");
    if (n < 0 || (n > 0 && !pids)) return fail(PLAID_EINVAL, "bad passage list");
    if (capacity < 0) return fail(PLAID_EINVAL, "negative capacity");
    DeviceGuard g(ix->device);
    if (!g.ok) return fail(PLAID_EHIP, "hipSetDevice(%d) failed", ix->device);
    hipStream_t st = (hipStream_t)hip_stream;
    // the passage ids come from the caller: check them on the host before any kernel dereferences them
    std::vector<int32_t> hp;
    try {
        hp.resize((size_t)(n > 0 ? n : 1));
    } catch (...) {
        return fail(PLAID_ENOMEM, "host allocation for %d passage ids failed", n);
    }
    if (n > 0) {
        HIP_TRY(hipMemcpyAsync(hp.data(), pids, (size_t)n * 4, hipMemcpyDeviceToHost, st));
        HIP_TRY(hipStreamSynchronize(st));
        for (int32_t a = 0; a < n; ++a)
            if (hp[a] < 0 || hp[a] >= ix->P) return fail(PLAID_EINVAL, "pids[%d] = %d out of range", a, hp[a]);
    }
    int64_t *offs = out_offsets;
    const size_t need = a256((size_t)(n + 1) * 8);
    if (!offs) {
        int rc = ensure_workspace(ix, need);
        if (rc) return rc;
        offs = (int64_t *)ix->ws;
    }
    plaid_launch_passage_offsets(st, ix->doc_offsets, pids, n, offs);
    int64_t total = 0;
    HIP_TRY(hipMemcpyAsync(&total, offs + n, 8, hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    if (total > capacity && (out_vectors || out_indices))
        return fail(PLAID_EINVAL, "passages hold %lld tokens, capacity is %lld", (long long)total, (long long)capacity);
    if (out_vectors || out_indices)
        plaid_launch_decompress_dump(st, ix->centroids, ix->doc_offsets, ix->codes, ix->residuals, ix->weights, ix->nbits,
                                     pids, n, offs, out_vectors, out_indices, ix->renormalize ? ix->inv_norm : nullptr);
    HIP_TRY(hipGetLastError());
    return PLAID_OK;
}
