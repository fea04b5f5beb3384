// C ABI of libvlq: argument checks, memory ownership, kernel sequencing.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <mutex>
#include <new>
#include <vector>

#include "common.h"

// ---------------------------------------------------------------------------
// errors
// ---------------------------------------------------------------------------
static thread_local char g_err[512] = "";

static int fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

#define HIPCHK(expr)                                                                                   \
    do {                                                                                               \
        hipError_t e_ = (expr);                                                                        \
        if (e_ != hipSuccess)                                                                          \
            return fail(e_ == hipErrorOutOfMemory ? VLQ_ENOMEM : VLQ_EHIP, "%s: %s (%s:%d)", #expr,    \
                        hipGetErrorString(e_), __FILE__, __LINE__);                                    \
    } while (0)

#define LAUNCHCHK() HIPCHK(hipGetLastError())

extern "C" const char *vlq_last_error(void) { return g_err; }
extern "C" int vlq_version(void) { return VLQ_VERSION; }

// ---------------------------------------------------------------------------
// static scratch of the entry point that allocates nothing
// ---------------------------------------------------------------------------
// The scratch memory of vlq_search_noalloc: one array per GPU, part of the loaded code object and
// held until the process ends.  In host code the array's name is only a handle for
// hipGetSymbolAddress; the address it yields, per device, is what kernels are given.
static __device__ __align__(256) unsigned char scratch[VLQ_NOALLOC_SCRATCH_BYTES];

#define VLQ_MAX_DEVICES 64
static std::mutex g_scratch_mu;
static void *g_scratch_ptr[VLQ_MAX_DEVICES] = {};

// Address of the current device's copy of `scratch` (looked up once per device).
static int static_scratch(void **out)
{
    int dev = -1;
    HIPCHK(hipGetDevice(&dev));
    if (dev < 0 || dev >= VLQ_MAX_DEVICES) return fail(VLQ_EINVAL, "device ordinal %d outside [0, %d)", dev, VLQ_MAX_DEVICES);
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        HIPCHK(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return fail(VLQ_EHIP, "hipGetSymbolAddress returned a null address");
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return VLQ_OK;
}

// ---------------------------------------------------------------------------
// index object
// ---------------------------------------------------------------------------
#define VLQ_MAX_PARTS 8

struct ProfRec {
    int stage;
    hipEvent_t t0, t1;
};

struct vlq_index {
    vlq_params_t p;
    float lam_step, lam_zero;
    double lam_step_d;
    // codebooks and graph
    float *C = nullptr, *P = nullptr, *E = nullptr;
    int32_t *S = nullptr;
    // Distances do not depend on the origin, the rounding error of an inner product does: the
    // contractions and the scan's tables work relative to the mean of the centroids.
    //   mu   [D] the mean, for the scan (s_x and the query's table);
    //   mu_c [D] the mean rounded to integers, for the contractions (integer-valued vectors minus
    //        an integer vector stay exactly representable in bf16);
    //   cn   [k] ||c - mu_c||^2;  Cc [k x D] c - mu_c, the operand of the fp32 contraction.
    float *mu = nullptr, *mu_c = nullptr, *cn = nullptr, *Cc = nullptr;
    // kernel choices (vlq_index_set_option) and the query-side lambda range
    int opt[VLQ_OPT_COUNT] = {0, 0, -1, 0, 0, 0, 64, 0};
    // second stream (default priority) and the events that order it against the caller's stream
    hipStream_t side = nullptr;
    hipEvent_t ev_go[VLQ_MAX_PARTS] = {}, ev_done[VLQ_MAX_PARTS] = {};
    float qlam_lo = -INFINITY, qlam_hi = INFINITY;
    // centroids split into bf16 (hi, lo) for the matrix-core shortlist; null when D does not allow it
    void *Cimg = nullptr;
    int32_t *flags = nullptr;
    // staged points, in insertion order
    int64_t ntotal = 0, cap = 0;
    int32_t *st_label = nullptr, *st_ids = nullptr;
    uint8_t *st_lam = nullptr, *st_codes = nullptr;
    // inverted lists
    bool finalized = false;
    int64_t lists_cap = 0;
    int64_t *off = nullptr;
    int32_t *ids = nullptr;
    uint8_t *codes = nullptr, *lam = nullptr;
    float *sx = nullptr; // query-independent part of the distance, per stored point
    // scratch
    void *ws = nullptr;
    size_t ws_bytes = 0;
    // profiling
    bool prof = false;
    std::vector<ProfRec> recs;
};

struct Bump {
    char *base;
    size_t off = 0;
    explicit Bump(void *b) : base((char *)b) {}
    template <typename T>
    T *take(size_t count)
    {
        off = (off + 255) & ~(size_t)255;
        T *p = base ? (T *)(base + off) : nullptr;
        off += count * sizeof(T);
        return p;
    }
};

static int ws_reserve(vlq_index *idx, size_t bytes)
{
    if (bytes <= idx->ws_bytes) return VLQ_OK;
    if (idx->ws) {
        HIPCHK(hipDeviceSynchronize()); // queued kernels may still use the old block
        HIPCHK(hipFree(idx->ws));
        idx->ws = nullptr;
        idx->ws_bytes = 0;
    }
    bytes += bytes / 8;
    HIPCHK(hipMalloc(&idx->ws, bytes));
    idx->ws_bytes = bytes;
    return VLQ_OK;
}

struct StageTimer {
    vlq_index *idx;
    hipStream_t st;
    int stage;
    hipEvent_t t0 = nullptr;
    StageTimer(vlq_index *i, hipStream_t s, int g, bool on = true) : idx(i), st(s), stage(g)
    {
        if (on && idx->prof && hipEventCreate(&t0) == hipSuccess) (void)hipEventRecord(t0, st);
    }
    ~StageTimer()
    {
        if (!t0) return;
        hipEvent_t t1;
        if (hipEventCreate(&t1) != hipSuccess) {
            (void)hipEventDestroy(t0);
            return;
        }
        (void)hipEventRecord(t1, st);
        idx->recs.push_back({stage, t0, t1});
    }
};

extern "C" void vlq_index_free(vlq_index_t *idx)
{
    if (!idx) return;
    (void)hipDeviceSynchronize();
    void *ptrs[] = {idx->C, idx->cn, idx->P, idx->E, idx->S, idx->st_label, idx->st_ids, idx->st_lam,
                    idx->st_codes, idx->off, idx->ids, idx->codes, idx->lam, idx->sx, idx->ws,
                    idx->Cimg, idx->flags, idx->mu, idx->mu_c, idx->Cc};
    for (void *p : ptrs)
        if (p) (void)hipFree(p);
    for (auto &r : idx->recs) {
        (void)hipEventDestroy(r.t0);
        (void)hipEventDestroy(r.t1);
    }
    for (int p = 0; p < VLQ_MAX_PARTS; ++p) {
        if (idx->ev_go[p]) (void)hipEventDestroy(idx->ev_go[p]);
        if (idx->ev_done[p]) (void)hipEventDestroy(idx->ev_done[p]);
    }
    if (idx->side) (void)hipStreamDestroy(idx->side);
    delete idx;
}

// ---------------------------------------------------------------------------
// build
// ---------------------------------------------------------------------------
static int check_params(const vlq_params_t *p, double *step, float *zero)
{
    if (!p) return fail(VLQ_EINVAL, "params is NULL");
    if (p->d < 1 || p->d > VLQ_MAX_DIM) return fail(VLQ_EINVAL, "d = %d outside [1, %d]", p->d, VLQ_MAX_DIM);
    if (p->m < 1 || p->m > VLQ_MAX_M) return fail(VLQ_EINVAL, "m = %d outside [1, %d]", p->m, VLQ_MAX_M);
    if (p->d % p->m) return fail(VLQ_EINVAL, "d = %d is not a multiple of m = %d", p->d, p->m);
    if (p->n_edges < 1 || p->n_edges > VLQ_MAX_EDGES)
        return fail(VLQ_EINVAL, "n_edges = %d outside [1, %d]", p->n_edges, VLQ_MAX_EDGES);
    if (p->nlist <= p->n_edges) return fail(VLQ_EINVAL, "nlist = %d must exceed n_edges = %d", p->nlist, p->n_edges);
    if ((int64_t)p->nlist * p->n_edges > 0x7FFFFFFF) return fail(VLQ_EINVAL, "nlist * n_edges overflows int32");
    double lo = p->lambda_lo, hi = p->lambda_hi;
    if (lo == 0.0 && hi == 0.0) {
        lo = -0.25;
        hi = 0.5;
    }
    if (!(lo <= 0.0 && hi > 0.0 && hi > lo)) return fail(VLQ_EINVAL, "lambda grid [%g, %g] must contain 0", lo, hi);
    const double s = (hi - lo) / 255.0, z = -lo / s;
    if (fabs(z - rint(z)) > 1e-6) return fail(VLQ_EINVAL, "lambda_lo * 255 / (lambda_hi - lambda_lo) is not an integer");
    *step = s;
    *zero = (float)rint(z);
    return VLQ_OK;
}

static int build_graph(vlq_index *idx, hipStream_t st)
{
    const int k = idx->p.nlist, D = idx->p.d, n = idx->p.n_edges;
    int64_t TR = ((int64_t)256 << 20) / ((int64_t)4 * k);
    if (TR < 128) TR = 128;
    if (TR > k) TR = k;
    Bump plan(nullptr);
    plan.take<float>((size_t)TR * k);
    int rc = ws_reserve(idx, plan.off + 256);
    if (rc) return rc;
    Bump b(idx->ws);
    float *dist = b.take<float>((size_t)TR * k);
    for (int64_t r0 = 0; r0 < k; r0 += TR) {
        const int rows = (int)(k - r0 < TR ? k - r0 : TR);
        launch_coarse_gemm_full(idx->Cc + r0 * D, rows, idx->Cc, k, D, idx->cn + r0, idx->cn, dist, k, st);
        LAUNCHCHK();
        launch_select_cells(dist, k, rows, k, idx->C + r0 * D, D, idx->cn + r0, idx->C, idx->cn, n, (int)r0,
                            idx->S + r0 * n, idx->E + r0 * n, st);
        LAUNCHCHK();
    }
    return VLQ_OK;
}

extern "C" int vlq_build_index(const vlq_params_t *params, const float *d_centroids, const float *d_pq,
                               const float *d_base, int64_t N, const int32_t *d_ids, void *stream,
                               vlq_index_t **out)
{
    double step;
    float zero;
    int rc = check_params(params, &step, &zero);
    if (rc) return rc;
    if (!d_centroids || !d_pq || !out) return fail(VLQ_EINVAL, "d_centroids, d_pq and out must not be NULL");
    if (N < 0 || N > 0x7FFFFFFF) return fail(VLQ_EINVAL, "N = %lld outside [0, 2^31)", (long long)N);
    if (N > 0 && !d_base) return fail(VLQ_EINVAL, "d_base is NULL with N > 0");
    hipStream_t st = (hipStream_t)stream;
    vlq_index *idx = new (std::nothrow) vlq_index();
    if (!idx) return fail(VLQ_ENOMEM, "host allocation failed");
    idx->p = *params;
    idx->lam_step = (float)step;
    idx->lam_step_d = step;
    idx->lam_zero = zero;
    if (params->lambda_lo == 0.f && params->lambda_hi == 0.f) {
        idx->p.lambda_lo = -0.25f;
        idx->p.lambda_hi = 0.5f;
    }
    const int k = params->nlist, D = params->d, n = params->n_edges, m = params->m;
    auto body = [&]() -> int {
        {
            // set-up: the address of this device's static scratch array (vlq_search_noalloc)
            void *sp = nullptr;
            int r0 = static_scratch(&sp);
            if (r0) return r0;
        }
        HIPCHK(hipStreamCreateWithFlags(&idx->side, hipStreamNonBlocking));
        for (int p = 0; p < VLQ_MAX_PARTS; ++p) {
            HIPCHK(hipEventCreateWithFlags(&idx->ev_go[p], hipEventDisableTiming));
            HIPCHK(hipEventCreateWithFlags(&idx->ev_done[p], hipEventDisableTiming));
        }
        HIPCHK(hipMalloc(&idx->C, (size_t)k * D * 4));
        HIPCHK(hipMalloc(&idx->cn, (size_t)k * 4));
        HIPCHK(hipMalloc(&idx->Cc, (size_t)k * D * 4));
        HIPCHK(hipMalloc(&idx->mu, (size_t)D * 4));
        HIPCHK(hipMalloc(&idx->mu_c, (size_t)D * 4));
        HIPCHK(hipMalloc(&idx->P, (size_t)256 * D * 4));
        HIPCHK(hipMalloc(&idx->S, (size_t)k * n * 4));
        HIPCHK(hipMalloc(&idx->E, (size_t)k * n * 4));
        HIPCHK(hipMalloc(&idx->off, ((size_t)k * n + 1) * 8));
        HIPCHK(hipMemcpyAsync(idx->C, d_centroids, (size_t)k * D * 4, hipMemcpyDeviceToDevice, st));
        HIPCHK(hipMemcpyAsync(idx->P, d_pq, (size_t)256 * D * 4, hipMemcpyDeviceToDevice, st));
        HIPCHK(hipMemsetAsync(idx->off, 0, ((size_t)k * n + 1) * 8, st));
        launch_col_means(idx->C, k, D, idx->mu, idx->mu_c, st);
        LAUNCHCHK();
        launch_center_rows(idx->C, k, D, idx->mu_c, idx->Cc, st);
        LAUNCHCHK();
        launch_row_norms(idx->C, k, D, idx->mu_c, idx->cn, st);
        LAUNCHCHK();
        if (coarse_bf16_supported(D)) {
            HIPCHK(hipMalloc(&idx->Cimg, coarse_bf16_image_bytes(k, D)));
            HIPCHK(hipMalloc(&idx->flags, 256));
            launch_split_bf16(idx->C, k, D, idx->mu_c, idx->Cimg, idx->flags, st);
            LAUNCHCHK();
        }
        int r = build_graph(idx, st);
        if (r) return r;
        idx->finalized = true; // an empty index is searchable
        if (N > 0) {
            r = vlq_index_add(idx, d_base, N, d_ids, stream);
            if (r) return r;
            r = vlq_index_finalize(idx, stream);
            if (r) return r;
        }
        HIPCHK(hipStreamSynchronize(st));
        return VLQ_OK;
    };
    (void)m;
    rc = body();
    if (rc) {
        char keep[sizeof(g_err)];
        memcpy(keep, g_err, sizeof(keep));
        vlq_index_free(idx);
        memcpy(g_err, keep, sizeof(keep));
        return rc;
    }
    *out = idx;
    return VLQ_OK;
}

extern "C" int64_t vlq_index_ntotal(const vlq_index_t *idx) { return idx ? idx->ntotal : -1; }
extern "C" int vlq_index_is_finalized(const vlq_index_t *idx) { return idx ? (idx->finalized ? 1 : 0) : 0; }
extern "C" int vlq_index_params(const vlq_index_t *idx, vlq_params_t *out)
{
    if (!idx || !out) return fail(VLQ_EINVAL, "NULL argument");
    *out = idx->p;
    return VLQ_OK;
}

// ---------------------------------------------------------------------------
// encode / add
// ---------------------------------------------------------------------------
#define ENC_CHUNK ((int64_t)1 << 18)

static int encode_impl(vlq_index *idx, const float *d_x, int64_t nb, int32_t *d_cell, int32_t *d_edge,
                       uint8_t *d_lambda, uint8_t *d_codes, int32_t *d_label, hipStream_t st, float *d_res = nullptr)
{
    const int k = idx->p.nlist, D = idx->p.d, n = idx->p.n_edges, m = idx->p.m;
    const int64_t chunk = nb < ENC_CHUNK ? nb : ENC_CHUNK;
    const int nsplit = coarse_gemm_nn_splits((int)chunk, k);
    // shortlist on the bf16 matrix cores unless the dimension rules it out (or the fp32 product is
    // asked for: VLQ_OPT_COARSE_FP32)
    const bool bf16 = idx->Cimg && !idx->opt[VLQ_OPT_COARSE_FP32];
    float *xn, *xc = nullptr;
    uint64_t *cand;
    uint8_t *ximg = nullptr;
    int32_t *tcell, *tedge, *flag;
    auto carve = [&](Bump &b) {
        xn = b.take<float>((size_t)chunk);
        if (bf16)
            ximg = b.take<uint8_t>(coarse_bf16_image_bytes(chunk, D));
        else
            xc = b.take<float>((size_t)chunk * D);
        cand = b.take<uint64_t>((size_t)chunk * nsplit * VLQ_NN_CANDS);
        tcell = b.take<int32_t>((size_t)chunk);
        tedge = b.take<int32_t>((size_t)chunk);
        flag = b.take<int32_t>(64);
    };
    Bump plan(nullptr);
    carve(plan);
    int rc = ws_reserve(idx, plan.off + 256);
    if (rc) return rc;
    Bump b(idx->ws);
    carve(b);
    for (int64_t s = 0; s < nb; s += chunk) {
        const int64_t cnt = nb - s < chunk ? nb - s : chunk;
        const float *x = d_x + s * D;
        // the split count is fixed by the buffer; a short tail only leaves less work per split
        launch_row_norms(x, cnt, D, idx->mu_c, xn, st);
        LAUNCHCHK();
        EncodeArgs a;
        if (bf16) {
            launch_split_bf16(x, cnt, D, idx->mu_c, ximg, flag + 1, st);
            LAUNCHCHK();
            HIPCHK((hipError_t)launch_coarse_gemm_nn_bf16(ximg, flag + 1, (int)cnt, idx->Cimg, k, D, xn, idx->cn, cand,
                                                          nsplit, &a.band_norm, &a.band_dist, st));
        } else {
            launch_center_rows(x, cnt, D, idx->mu_c, xc, st);
            LAUNCHCHK();
            launch_coarse_gemm_nn(xc, (int)cnt, idx->Cc, k, D, xn, idx->cn, cand, nsplit, st);
            a.band_norm = vlq_fp32_band_norm(D);
            a.band_dist = 0.f;
        }
        LAUNCHCHK();
        a.mu = idx->mu_c;
        a.lam_step_d = idx->lam_step_d;
        a.wave_per_vector = idx->opt[VLQ_OPT_ENCODE_WAVE] != 0;
        a.X = x;
        a.nb = cnt;
        a.D = D;
        a.k = k;
        a.n = n;
        a.m = m;
        a.C = idx->C;
        a.S = idx->S;
        a.E = idx->E;
        a.P = idx->P;
        a.lam_step = idx->lam_step;
        a.lam_zero = idx->lam_zero;
        a.cand = cand;
        a.nsplit = nsplit;
        a.cell = d_cell ? d_cell + s : (d_label ? tcell : nullptr);
        a.edge = d_edge ? d_edge + s : (d_label ? tedge : nullptr);
        a.lamq = d_lambda ? d_lambda + s : nullptr;
        a.codes = d_codes ? d_codes + s * m : nullptr;
        a.res = d_res ? d_res + s * D : nullptr;
        launch_encode_finish(a, st);
        LAUNCHCHK();
        if (d_label) {
            launch_pack_labels(a.cell, a.edge, n, k, d_label + s, cnt, flag, st);
            LAUNCHCHK();
        }
    }
    return VLQ_OK;
}

extern "C" int vlq_encode(const vlq_index_t *cidx, const float *d_x, int64_t nb, int32_t *d_cell,
                          int32_t *d_edge, uint8_t *d_lambda, uint8_t *d_codes, void *stream)
{
    vlq_index *idx = const_cast<vlq_index *>(cidx);
    if (!idx) return fail(VLQ_EINVAL, "idx is NULL");
    if (nb < 0) return fail(VLQ_EINVAL, "nb = %lld is negative", (long long)nb);
    if (nb == 0) return VLQ_OK;
    if (!d_x) return fail(VLQ_EINVAL, "d_x is NULL");
    return encode_impl(idx, d_x, nb, d_cell, d_edge, d_lambda, d_codes, nullptr, (hipStream_t)stream);
}

extern "C" int vlq_line_residuals(const vlq_index_t *cidx, const float *d_x, int64_t nb, float *d_res, void *stream)
{
    vlq_index *idx = const_cast<vlq_index *>(cidx);
    if (!idx) return fail(VLQ_EINVAL, "idx is NULL");
    if (nb < 0) return fail(VLQ_EINVAL, "nb = %lld is negative", (long long)nb);
    if (nb == 0) return VLQ_OK;
    if (!d_x || !d_res) return fail(VLQ_EINVAL, "d_x and d_res must not be NULL");
    return encode_impl(idx, d_x, nb, nullptr, nullptr, nullptr, nullptr, nullptr, (hipStream_t)stream, d_res);
}

// ---------------------------------------------------------------------------
// k-means
// ---------------------------------------------------------------------------
namespace {
struct DevBuf { // device allocations of one call, freed on every way out
    std::vector<void *> ptrs;
    ~DevBuf()
    {
        for (void *p : ptrs) (void)hipFree(p);
    }
    template <typename T>
    hipError_t get(T **out, size_t count)
    {
        void *p = nullptr;
        hipError_t e = hipMalloc(&p, count * sizeof(T) + 256);
        if (e == hipSuccess) ptrs.push_back(p);
        *out = (T *)p;
        return e;
    }
};
} // namespace

extern "C" int vlq_kmeans(const float *d_x, int64_t nt, int32_t d, int32_t k, int32_t iters, float *d_centroids,
                          int32_t *d_assign, int32_t *d_counts, void *stream)
{
    if (!d_x || !d_centroids) return fail(VLQ_EINVAL, "d_x and d_centroids must not be NULL");
    if (d < 1 || d > VLQ_MAX_DIM) return fail(VLQ_EINVAL, "d = %d outside [1, %d]", d, VLQ_MAX_DIM);
    if (k < 1) return fail(VLQ_EINVAL, "k = %d must be positive", k);
    if (nt < 1 || nt > 0x7FFFFFFF) return fail(VLQ_EINVAL, "nt = %lld outside [1, 2^31)", (long long)nt);
    if (iters < 0) return fail(VLQ_EINVAL, "iters = %d is negative", iters);
    hipStream_t st = (hipStream_t)stream;
    const int D = d;
    const int64_t chunk = nt < ENC_CHUNK ? nt : ENC_CHUNK;
    const int nsplit = coarse_gemm_nn_splits((int)chunk, k);
    const bool bf16 = coarse_bf16_supported(D);
    int shift = 62;
    while (shift > 0 && ((int64_t)1 << (62 - shift)) < nt) --shift;

    DevBuf buf;
    float *xn, *cn, *mu, *mu_c, *xc = nullptr, *cc = nullptr;
    uint64_t *cand;
    int32_t *assign, *cnt, *flag;
    long long *sums;
    uint32_t *absmax;
    uint8_t *ximg = nullptr, *cimg = nullptr;
    HIPCHK(buf.get(&xn, (size_t)chunk));
    HIPCHK(buf.get(&cn, (size_t)k));
    HIPCHK(buf.get(&mu, (size_t)D));
    HIPCHK(buf.get(&mu_c, (size_t)D));
    HIPCHK(buf.get(&cand, (size_t)chunk * nsplit * VLQ_NN_CANDS));
    HIPCHK(buf.get(&assign, (size_t)nt));
    HIPCHK(buf.get(&cnt, (size_t)k));
    HIPCHK(buf.get(&flag, 64));
    HIPCHK(buf.get(&sums, (size_t)k * D));
    HIPCHK(buf.get(&absmax, 64));
    if (bf16) {
        HIPCHK(buf.get(&ximg, coarse_bf16_image_bytes(chunk, D)));
        HIPCHK(buf.get(&cimg, coarse_bf16_image_bytes(k, D)));
    } else {
        HIPCHK(buf.get(&xc, (size_t)chunk * D));
        HIPCHK(buf.get(&cc, (size_t)k * D));
    }
    HIPCHK(hipMemsetAsync(absmax, 0, 4, st));
    launch_absmax(d_x, nt * D, absmax, st);
    LAUNCHCHK();

    // nearest centroid of every vector (Eq. 2): the encoder's shortlist + exact re-evaluation; the
    // product works relative to the (integer-rounded) mean of the current centroids
    auto assign_all = [&]() -> int {
        launch_col_means(d_centroids, k, D, mu, mu_c, st);
        LAUNCHCHK();
        launch_row_norms(d_centroids, k, D, mu_c, cn, st);
        LAUNCHCHK();
        if (bf16) {
            launch_split_bf16(d_centroids, k, D, mu_c, cimg, flag, st);
        } else {
            launch_center_rows(d_centroids, k, D, mu_c, cc, st);
        }
        LAUNCHCHK();
        for (int64_t s = 0; s < nt; s += chunk) {
            const int64_t n = nt - s < chunk ? nt - s : chunk;
            const float *x = d_x + s * D;
            launch_row_norms(x, n, D, mu_c, xn, st);
            LAUNCHCHK();
            EncodeArgs a = {};
            if (bf16) {
                launch_split_bf16(x, n, D, mu_c, ximg, flag + 1, st);
                LAUNCHCHK();
                HIPCHK((hipError_t)launch_coarse_gemm_nn_bf16(ximg, flag + 1, (int)n, cimg, k, D, xn, cn, cand, nsplit,
                                                              &a.band_norm, &a.band_dist, st));
            } else {
                launch_center_rows(x, n, D, mu_c, xc, st);
                LAUNCHCHK();
                launch_coarse_gemm_nn(xc, (int)n, cc, k, D, xn, cn, cand, nsplit, st);
                a.band_norm = vlq_fp32_band_norm(D);
                a.band_dist = 0.f;
            }
            LAUNCHCHK();
            a.mu = mu_c;
            a.X = x;
            a.nb = n;
            a.D = D;
            a.k = k;
            a.n = 0;
            a.m = 1;
            a.C = d_centroids;
            a.cand = cand;
            a.nsplit = nsplit;
            a.cell = assign + s;
            launch_encode_finish(a, st);
            LAUNCHCHK();
        }
        return VLQ_OK;
    };
    for (int it = 0; it < iters; ++it) {
        int rc = assign_all();
        if (rc) return rc;
        HIPCHK(hipMemsetAsync(cnt, 0, (size_t)k * 4, st));
        HIPCHK(hipMemsetAsync(sums, 0, (size_t)k * D * 8, st));
        launch_kmeans_accumulate(d_x, nt, D, assign, absmax, shift, sums, cnt, st);
        LAUNCHCHK();
        launch_kmeans_update(d_centroids, k, D, sums, cnt, absmax, shift, st);
        LAUNCHCHK();
    }
    if (d_assign || d_counts) {
        int rc = assign_all();
        if (rc) return rc;
        if (d_assign) HIPCHK(hipMemcpyAsync(d_assign, assign, (size_t)nt * 4, hipMemcpyDeviceToDevice, st));
        if (d_counts) {
            // counts only: the accumulation kernel is run over a one-dimensional view of the sample
            HIPCHK(hipMemsetAsync(cnt, 0, (size_t)k * 4, st));
            HIPCHK(hipMemsetAsync(sums, 0, (size_t)k * 8, st));
            launch_kmeans_accumulate(d_x, nt, 1, assign, absmax, shift, sums, cnt, st);
            LAUNCHCHK();
            HIPCHK(hipMemcpyAsync(d_counts, cnt, (size_t)k * 4, hipMemcpyDeviceToDevice, st));
        }
    }
    HIPCHK(hipStreamSynchronize(st)); // the temporaries are freed on return
    return VLQ_OK;
}

static int grow_staging(vlq_index *idx, int64_t need, hipStream_t st)
{
    if (need <= idx->cap) return VLQ_OK;
    int64_t ncap = idx->cap * 2;
    if (ncap < need) ncap = need;
    if (ncap < 1024) ncap = 1024;
    const int m = idx->p.m;
    int32_t *nl = nullptr, *ni = nullptr;
    uint8_t *nlam = nullptr, *nc = nullptr;
    HIPCHK(hipMalloc(&nl, (size_t)ncap * 4));
    HIPCHK(hipMalloc(&ni, (size_t)ncap * 4));
    HIPCHK(hipMalloc(&nlam, (size_t)ncap));
    HIPCHK(hipMalloc(&nc, (size_t)ncap * m));
    if (idx->ntotal > 0) {
        HIPCHK(hipMemcpyAsync(nl, idx->st_label, (size_t)idx->ntotal * 4, hipMemcpyDeviceToDevice, st));
        HIPCHK(hipMemcpyAsync(ni, idx->st_ids, (size_t)idx->ntotal * 4, hipMemcpyDeviceToDevice, st));
        HIPCHK(hipMemcpyAsync(nlam, idx->st_lam, (size_t)idx->ntotal, hipMemcpyDeviceToDevice, st));
        HIPCHK(hipMemcpyAsync(nc, idx->st_codes, (size_t)idx->ntotal * m, hipMemcpyDeviceToDevice, st));
    }
    HIPCHK(hipDeviceSynchronize());
    void *old[] = {idx->st_label, idx->st_ids, idx->st_lam, idx->st_codes};
    for (void *p : old)
        if (p) HIPCHK(hipFree(p));
    idx->st_label = nl;
    idx->st_ids = ni;
    idx->st_lam = nlam;
    idx->st_codes = nc;
    idx->cap = ncap;
    return VLQ_OK;
}

extern "C" int vlq_index_reserve(vlq_index_t *idx, int64_t total)
{
    if (!idx) return fail(VLQ_EINVAL, "idx is NULL");
    if (total < 0 || total > 0x7FFFFFFF) return fail(VLQ_EINVAL, "total outside [0, 2^31)");
    return grow_staging(idx, total, nullptr);
}

static int stage_ids(vlq_index *idx, const int32_t *d_ids, int64_t nb, hipStream_t st)
{
    if (d_ids) {
        HIPCHK(hipMemcpyAsync(idx->st_ids + idx->ntotal, d_ids, (size_t)nb * 4, hipMemcpyDeviceToDevice, st));
    } else {
        launch_iota_i32(idx->st_ids + idx->ntotal, nb, (int32_t)idx->ntotal, st);
        LAUNCHCHK();
    }
    return VLQ_OK;
}

extern "C" int vlq_index_add(vlq_index_t *idx, const float *d_x, int64_t nb, const int32_t *d_ids, void *stream)
{
    if (!idx) return fail(VLQ_EINVAL, "idx is NULL");
    if (nb < 0) return fail(VLQ_EINVAL, "nb is negative");
    if (nb == 0) return VLQ_OK;
    if (!d_x) return fail(VLQ_EINVAL, "d_x is NULL");
    if (idx->ntotal + nb > 0x7FFFFFFF) return fail(VLQ_EINVAL, "more than 2^31 - 1 points");
    hipStream_t st = (hipStream_t)stream;
    int rc = grow_staging(idx, idx->ntotal + nb, st);
    if (rc) return rc;
    rc = encode_impl(idx, d_x, nb, nullptr, nullptr, idx->st_lam + idx->ntotal,
                     idx->st_codes + idx->ntotal * idx->p.m, idx->st_label + idx->ntotal, st);
    if (rc) return rc;
    rc = stage_ids(idx, d_ids, nb, st);
    if (rc) return rc;
    idx->ntotal += nb;
    idx->finalized = false;
    return VLQ_OK;
}

extern "C" int vlq_index_add_encoded(vlq_index_t *idx, const int32_t *d_cell, const int32_t *d_edge,
                                     const uint8_t *d_lambda, const uint8_t *d_codes, const int32_t *d_ids,
                                     int64_t nb, void *stream)
{
    if (!idx) return fail(VLQ_EINVAL, "idx is NULL");
    if (nb < 0) return fail(VLQ_EINVAL, "nb is negative");
    if (nb == 0) return VLQ_OK;
    if (!d_cell || !d_edge || !d_lambda || !d_codes) return fail(VLQ_EINVAL, "encoded fields must not be NULL");
    if (idx->ntotal + nb > 0x7FFFFFFF) return fail(VLQ_EINVAL, "more than 2^31 - 1 points");
    hipStream_t st = (hipStream_t)stream;
    int rc = grow_staging(idx, idx->ntotal + nb, st);
    if (rc) return rc;
    rc = ws_reserve(idx, 256);
    if (rc) return rc;
    int32_t *bad = (int32_t *)idx->ws;
    HIPCHK(hipMemsetAsync(bad, 0, 4, st));
    launch_pack_labels(d_cell, d_edge, idx->p.n_edges, idx->p.nlist, idx->st_label + idx->ntotal, nb, bad, st);
    LAUNCHCHK();
    int32_t hbad = 0;
    HIPCHK(hipMemcpyAsync(&hbad, bad, 4, hipMemcpyDeviceToHost, st));
    HIPCHK(hipStreamSynchronize(st));
    if (hbad) return fail(VLQ_EINVAL, "a cell or edge index is out of range");
    const int m = idx->p.m;
    HIPCHK(hipMemcpyAsync(idx->st_lam + idx->ntotal, d_lambda, (size_t)nb, hipMemcpyDeviceToDevice, st));
    HIPCHK(hipMemcpyAsync(idx->st_codes + idx->ntotal * m, d_codes, (size_t)nb * m, hipMemcpyDeviceToDevice, st));
    rc = stage_ids(idx, d_ids, nb, st);
    if (rc) return rc;
    idx->ntotal += nb;
    idx->finalized = false;
    return VLQ_OK;
}

// ---------------------------------------------------------------------------
// finalize
// ---------------------------------------------------------------------------
#define MAX_LONG (1 << 20)

extern "C" int vlq_index_finalize(vlq_index_t *idx, void *stream)
{
    if (!idx) return fail(VLQ_EINVAL, "idx is NULL");
    hipStream_t st = (hipStream_t)stream;
    const int m = idx->p.m;
    const int64_t nl = (int64_t)idx->p.nlist * idx->p.n_edges;
    const int64_t N = idx->ntotal;
    if (N > idx->lists_cap) {
        HIPCHK(hipDeviceSynchronize());
        void *old[] = {idx->ids, idx->codes, idx->lam, idx->sx};
        for (void *p : old)
            if (p) HIPCHK(hipFree(p));
        idx->ids = nullptr;
        idx->codes = nullptr;
        idx->lam = nullptr;
        idx->sx = nullptr;
        idx->lists_cap = 0;
        HIPCHK(hipMalloc(&idx->ids, (size_t)N * 4));
        HIPCHK(hipMalloc(&idx->codes, (size_t)N * m + 16));
        HIPCHK(hipMalloc(&idx->lam, (size_t)N + 16));
        HIPCHK(hipMalloc(&idx->sx, (size_t)N * 4 + 16));
        idx->lists_cap = N;
    }
    Bump plan(nullptr);
    plan.take<int32_t>((size_t)nl);
    plan.take<int32_t>((size_t)nl);
    plan.take<int32_t>(MAX_LONG + 1);
    plan.take<int32_t>(MAX_LONG + 1);
    int rc = ws_reserve(idx, plan.off + 256);
    if (rc) return rc;
    Bump b(idx->ws);
    int32_t *cnt = b.take<int32_t>((size_t)nl);
    int32_t *cursor = b.take<int32_t>((size_t)nl);
    int32_t *longs = b.take<int32_t>(MAX_LONG + 1);
    int32_t *n_long = longs + MAX_LONG;
    int32_t *longs2 = b.take<int32_t>(MAX_LONG + 1);
    int32_t *n_long2 = longs2 + MAX_LONG;
    HIPCHK(hipMemsetAsync(cnt, 0, (size_t)nl * 4, st));
    HIPCHK(hipMemsetAsync(cursor, 0, (size_t)nl * 4, st));
    launch_list_histogram(idx->st_label, N, cnt, st);
    LAUNCHCHK();
    launch_exclusive_scan(cnt, nl, idx->off, st);
    LAUNCHCHK();
    launch_list_scatter(idx->st_label, idx->st_ids, idx->st_codes, idx->st_lam, N, m, idx->off, cursor, idx->ids,
                        idx->codes, idx->lam, st);
    LAUNCHCHK();
    // Per-list order by id in three tiers: up to 1 024 points in a 64-thread workgroup's LDS; the
    // longer ones it reports go to 256-thread workgroups with up to 150 KB of LDS; what is longer
    // still is sorted in global memory, one list at a time.
    std::vector<int64_t> hoff; // host copy of the offsets, fetched only if the third tier is needed
    for (int round = 0; round < 1 << 20; ++round) {
        HIPCHK(hipMemsetAsync(n_long, 0, 4, st));
        launch_list_sort(idx->off, nl, m, idx->ids, idx->codes, idx->lam, longs, n_long, MAX_LONG, st);
        LAUNCHCHK();
        int32_t hn = 0;
        HIPCHK(hipMemcpyAsync(&hn, n_long, 4, hipMemcpyDeviceToHost, st));
        HIPCHK(hipStreamSynchronize(st));
        if (hn == 0) break;
        int take = hn < MAX_LONG ? hn : MAX_LONG;
        if (list_sort_mid_max(m) > 0) {
            HIPCHK(hipMemsetAsync(n_long2, 0, 4, st));
            launch_list_sort_mid(idx->off, m, longs, take, idx->ids, idx->codes, idx->lam, longs2, n_long2, MAX_LONG, st);
            LAUNCHCHK();
            int32_t hn2 = 0;
            HIPCHK(hipMemcpyAsync(&hn2, n_long2, 4, hipMemcpyDeviceToHost, st));
            HIPCHK(hipStreamSynchronize(st));
            take = hn2; // at most `take` <= MAX_LONG lists went in
        }
        if (take > 0) {
            std::vector<int32_t> hl(take);
            HIPCHK(hipMemcpy(hl.data(), list_sort_mid_max(m) > 0 ? longs2 : longs, (size_t)take * 4, hipMemcpyDeviceToHost));
            if (hoff.empty()) {
                hoff.resize((size_t)nl + 1);
                HIPCHK(hipMemcpy(hoff.data(), idx->off, ((size_t)nl + 1) * 8, hipMemcpyDeviceToHost));
            }
            int64_t maxlen = 0;
            for (int i = 0; i < take; ++i) maxlen = std::max(maxlen, hoff[hl[i] + 1] - hoff[hl[i]]);
            int64_t maxsz = 1;
            while (maxsz < maxlen) maxsz <<= 1;
            uint64_t *skeys = nullptr;
            uint8_t *spay = nullptr;
            HIPCHK(hipMalloc(&skeys, (size_t)maxsz * 8));
            hipError_t e2 = hipMalloc(&spay, (size_t)maxlen * (m + 1));
            if (e2 != hipSuccess) {
                (void)hipFree(skeys);
                HIPCHK(e2);
            }
            for (int i = 0; i < take; ++i) // same stream: the scratch is reused list after list
                launch_long_list_sort_at(hoff[hl[i]], hoff[hl[i] + 1] - hoff[hl[i]], m, idx->ids, idx->codes, idx->lam,
                                         skeys, spay, st);
            hipError_t e3 = hipStreamSynchronize(st);
            (void)hipFree(skeys);
            (void)hipFree(spay);
            HIPCHK(e3);
            HIPCHK(hipGetLastError());
        }
        if (hn <= MAX_LONG) break;
    }
    if (N > 0) {
        launch_list_static(idx->off, nl, idx->p.n_edges, idx->p.d, m, idx->C, idx->S, idx->P, idx->mu, idx->codes,
                           idx->lam, idx->lam_step_d, idx->lam_zero, idx->sx, st);
        LAUNCHCHK();
    }
    HIPCHK(hipStreamSynchronize(st));
    idx->finalized = true;
    return VLQ_OK;
}

// ---------------------------------------------------------------------------
// search
// ---------------------------------------------------------------------------
// Scratch memory of one part of a batch (a part is a run of consecutive queries that goes through
// the whole path on its own).
struct PartBufs {
    int q0 = 0, nq = 0;
    bool bf16 = false, by_cell = false, from_matrix = false;
    int csplit = 0, ccap = 0, nsplit = 1;
    int64_t TQ = 0;
    uint4 *desc = nullptr;
    uint8_t *qimg = nullptr, *cws = nullptr, *nws = nullptr;
    int32_t *qflag = nullptr, *cells = nullptr, *slab = nullptr;
    float *qc = nullptr, *qn = nullptr, *dist = nullptr, *cell_dist = nullptr, *sg = nullptr;
    uint64_t *partial = nullptr;
};

// `fixed` (optional): a caller-provided block of `fixed_bytes` that serves as the scratch memory
// of this call instead of the index's own (which grows on demand); the call then allocates nothing
// and fails when the block is too small.
//
// Large batches are cut into parts.  The region traversal of part p + 1 (coarse distances, cells,
// sub-regions: matrix cores and latency-bound selections) is queued on the index's second stream
// beside the list scan of part p (bandwidth-bound), so that only the first part's traversal is
// exposed; events order the two streams, and the caller's stream has everything behind it when
// the call returns.
static int search_impl(vlq_index *idx, const float *d_q, int32_t nq, int32_t w1, int32_t w2, int32_t K,
                       float *d_out_dist, int32_t *d_out_ids, int32_t *d_cells, float *d_cell_dist,
                       int32_t *d_sub, float *d_sub_score, hipStream_t st, void *fixed = nullptr,
                       size_t fixed_bytes = 0)
{
    if (!idx) return fail(VLQ_EINVAL, "idx is NULL");
    const int k = idx->p.nlist, D = idx->p.d, n = idx->p.n_edges, m = idx->p.m;
    if (nq < 0) return fail(VLQ_EINVAL, "nq is negative");
    if (w1 < 1 || w1 > k || w1 > VLQ_MAX_W1)
        return fail(VLQ_EINVAL, "w1 = %d outside [1, min(nlist, %d)]", w1, VLQ_MAX_W1);
    if ((int64_t)w1 * n > VLQ_MAX_SUBREGIONS)
        return fail(VLQ_EINVAL, "w1 * n_edges = %lld exceeds %d", (long long)w1 * n, VLQ_MAX_SUBREGIONS);
    if (w2 < 1 || w2 > w1 * n || w2 > VLQ_MAX_W2)
        return fail(VLQ_EINVAL, "w2 = %d outside [1, min(w1 * n_edges, %d)]", w2, VLQ_MAX_W2);
    if (K < 1 || K > VLQ_MAX_K) return fail(VLQ_EINVAL, "K = %d outside [1, %d]", K, VLQ_MAX_K);
    if (!idx->finalized) return fail(VLQ_EINVAL, "index has staged points: call vlq_index_finalize first");
    if (nq == 0) return VLQ_OK;
    if (!d_q || !d_out_dist || !d_out_ids) return fail(VLQ_EINVAL, "d_q, d_out_dist and d_out_ids must not be NULL");

    const bool timed = !fixed; // (recording stage times creates events)
    // parts: VLQ_OPT_PIPELINE_PARTS; one by default (measured: the scan's workgroups refill every
    // compute unit as fast as they leave, the traversal kernels of the next part starve beside them
    // and the next scan waits for them, so two or more parts take longer than one)
    int parts = idx->opt[VLQ_OPT_PIPELINE_PARTS];
    if (parts <= 0) parts = 1;
    if (parts > VLQ_MAX_PARTS) parts = VLQ_MAX_PARTS;
    if (parts > nq) parts = nq;
    if (!idx->side) parts = 1;

    PartBufs pb[VLQ_MAX_PARTS];
    auto carve = [&](Bump &b) {
        for (int p = 0; p < parts; ++p) {
            PartBufs &c = pb[p];
            c.q0 = (int)((int64_t)nq * p / parts);
            c.nq = (int)((int64_t)nq * (p + 1) / parts) - c.q0;
            const int nqp = c.nq;
            // cells from two sweeps of the bf16 product where the shape allows it (VLQ_OPT_COARSE_FP32
            // asks for the fp32 distance matrix instead)
            // (a few queries: the fp32 matrix and one selection kernel per query are three launches
            // against six of the two-sweep form, and at that size the launches are what counts)
            c.bf16 = idx->Cimg && !idx->opt[VLQ_OPT_COARSE_FP32] && nqp > idx->opt[VLQ_OPT_SMALL_BATCH] &&
                     cells_bf16_plan(nqp, k, D, w1, !idx->opt[VLQ_OPT_COARSE_SPLIT], &c.csplit, &c.ccap);
            c.TQ = ((int64_t)512 << 20) / ((int64_t)4 * k);
            if (c.TQ < 128) c.TQ = 128;
            if (c.TQ > nqp) c.TQ = nqp;
            c.nsplit = scan_pick_nsplit(nqp, w2, K);
            c.by_cell = neighbour_dists_by_cell(nqp, k, n, D, w1) && !idx->opt[VLQ_OPT_NEIGHBOURS_PER_QUERY];
            c.desc = b.take<uint4>((size_t)nqp * w2);
            c.qn = b.take<float>((size_t)nqp);
            if (c.bf16) {
                size_t o0, o1, o2, o3;
                c.dist = nullptr;
                c.qimg = b.take<uint8_t>(coarse_bf16_image_bytes(nqp, D));
                c.qflag = b.take<int32_t>(64);
                c.cws = b.take<uint8_t>(cells_bf16_workspace(nqp, c.csplit, c.ccap, &o0, &o1, &o2, &o3));
            } else {
                c.dist = b.take<float>((size_t)c.TQ * k + (size_t)c.TQ * 1024); // (room for the small form's group minima)
                c.qc = b.take<float>((size_t)c.TQ * D);
                // a handful of queries: exact distances in one pass over the codebook, cells straight from them
                c.from_matrix = nqp <= idx->opt[VLQ_OPT_SMALL_BATCH] && nqp <= c.TQ && !idx->opt[VLQ_OPT_COARSE_FP32] &&
                                cells_small_supported(nqp, k, D, w1);
            }
            if (c.by_cell) c.nws = b.take<uint8_t>(neighbour_dists_workspace(nqp, k, n, w1));
            c.cells = b.take<int32_t>((size_t)nqp * w1);
            c.cell_dist = b.take<float>((size_t)nqp * w1);
            c.slab = b.take<int32_t>((size_t)nqp * w2);
            c.sg = b.take<float>((size_t)nqp * w2);
            c.partial = c.nsplit > 1 ? b.take<uint64_t>((size_t)nqp * c.nsplit * K) : nullptr;
        }
    };
    Bump plan(nullptr);
    carve(plan);
    void *wsbase;
    if (fixed) {
        if (plan.off + 256 > fixed_bytes)
            return fail(VLQ_EINVAL, "this search needs %zu bytes of scratch memory, the fixed block holds %zu",
                        plan.off + 256, fixed_bytes);
        wsbase = fixed;
    } else {
        int rc = ws_reserve(idx, plan.off + 256);
        if (rc) return rc;
        wsbase = idx->ws;
    }
    Bump b(wsbase);
    carve(b);

    auto scan_args = [&](const PartBufs &c) {
        ScanArgs a;
        a.Q = d_q + (int64_t)c.q0 * D;
        a.nq = c.nq;
        a.D = D;
        a.n = n;
        a.m = m;
        a.w2 = w2;
        a.K = K;
        a.nsplit = c.nsplit;
        a.C = idx->C;
        a.S = idx->S;
        a.E = idx->E;
        a.P = idx->P;
        a.off = idx->off;
        a.ids = idx->ids;
        a.codes = idx->codes;
        a.lam = idx->lam;
        a.sx = idx->sx;
        a.mu = idx->mu;
        a.desc = c.desc;
        // lists of a few tens of points: several of them share a chunk of 64 lanes
        // (VLQ_OPT_SCAN_PACKED forces either form)
        const int64_t nl = (int64_t)k * n;
        a.packed = idx->opt[VLQ_OPT_SCAN_PACKED] >= 0 ? idx->opt[VLQ_OPT_SCAN_PACKED] : (idx->ntotal < 64 * nl);
        a.force_generic = idx->opt[VLQ_OPT_SCAN_GENERIC] != 0;
        a.lam_step = idx->lam_step;
        a.lam_zero = idx->lam_zero;
        a.scan_label = c.slab;
        a.scan_g = c.sg;
        a.partial = c.partial;
        a.out_dist = d_out_dist + (int64_t)c.q0 * K;
        a.out_ids = d_out_ids + (int64_t)c.q0 * K;
        return a;
    };

    // Region traversal of one part (Alg. 3, first loop; Sec. 3.3.1) on stream s
    auto traverse = [&](const PartBufs &c, hipStream_t s) -> int {
        const float *q = d_q + (int64_t)c.q0 * D;
        const int nqp = c.nq;
        if (!c.from_matrix) {
            launch_row_norms(q, nqp, D, idx->mu_c, c.qn, s);
            LAUNCHCHK();
        }
        // with the bf16 cell selection the (query, cell) pairs are counted per cell as the cells are written
        PairWs pw = {};
        bool pairs_counted = false;
        const bool grouped = c.by_cell && neighbour_dists_grouped(nqp, w1);
        if (c.by_cell) pw = neighbour_dists_carve(c.nws, nqp, k, n, w1);
        if (c.bf16 && grouped) {
            launch_pair_counts_zero(pw, k, s);
            LAUNCHCHK();
        }
        if (c.bf16) {
            {
                StageTimer t(idx, s, VLQ_STAGE_COARSE, timed);
                launch_split_bf16(q, nqp, D, idx->mu_c, c.qimg, c.qflag, s);
                LAUNCHCHK();
                HIPCHK((hipError_t)launch_cells_bf16_coarse(c.qimg, c.qflag, nqp, idx->Cimg, k, D, c.qn, idx->cn,
                                                            !idx->opt[VLQ_OPT_COARSE_SPLIT], w1, c.csplit, c.ccap, c.cws, s));
            }
            LAUNCHCHK();
            {
                StageTimer t(idx, s, VLQ_STAGE_SELECT_CELLS, timed);
                launch_cells_bf16_exact(q, nqp, D, idx->C, k, w1, c.ccap, c.cws, c.csplit, c.cells, c.cell_dist,
                                        grouped ? pw.cnt : nullptr, grouped ? pw.rank : nullptr, s);
                pairs_counted = grouped;
            }
            LAUNCHCHK();
        } else if (c.from_matrix) {
            StageTimer t(idx, s, VLQ_STAGE_COARSE, timed);
            launch_cells_small(q, nqp, D, idx->C, k, w1, c.dist, c.cells, c.cell_dist, s);
            LAUNCHCHK();
        } else {
            for (int64_t r0 = 0; r0 < nqp; r0 += c.TQ) {
                const int rows = (int)(nqp - r0 < c.TQ ? nqp - r0 : c.TQ);
                {
                    StageTimer t(idx, s, VLQ_STAGE_COARSE, timed);
                    launch_center_rows(q + r0 * D, rows, D, idx->mu_c, c.qc, s);
                    launch_coarse_gemm_full(c.qc, rows, idx->Cc, k, D, c.qn + r0, idx->cn, c.dist, k, s);
                }
                LAUNCHCHK();
                {
                    StageTimer t(idx, s, VLQ_STAGE_SELECT_CELLS, timed);
                    launch_select_cells(c.dist, k, rows, k, q + r0 * D, D, c.qn + r0, idx->C, idx->cn, w1, -1,
                                        c.cells + r0 * w1, c.cell_dist + r0 * w1, s);
                }
                LAUNCHCHK();
            }
        }
        {
            StageTimer t(idx, s, VLQ_STAGE_SUBREGIONS, timed);
            // the streaming scan takes the visited sub-regions from desc alone, in any order
            const bool stream = scan_will_stream(scan_args(c));
            launch_subregions(q, nqp, D, idx->C, idx->S, idx->E, n, k, c.cells, c.cell_dist, w1, w2, idx->qlam_lo,
                              idx->qlam_hi, d_sub ? d_sub + (int64_t)c.q0 * w2 : nullptr,
                              d_sub_score ? d_sub_score + (int64_t)c.q0 * w2 : nullptr, stream ? nullptr : c.slab,
                              stream ? nullptr : c.sg, idx->off, c.desc, c.nws, pairs_counted, s);
        }
        LAUNCHCHK();
        if (d_cells)
            HIPCHK(hipMemcpyAsync(d_cells + (int64_t)c.q0 * w1, c.cells, (size_t)nqp * w1 * 4, hipMemcpyDeviceToDevice, s));
        if (d_cell_dist)
            HIPCHK(hipMemcpyAsync(d_cell_dist + (int64_t)c.q0 * w1, c.cell_dist, (size_t)nqp * w1 * 4, hipMemcpyDeviceToDevice, s));
        return VLQ_OK;
    };
    // Lookup tables, list scan, K-selection of one part (Sec. 3.3.2 - 3.3.3) on stream s
    auto scan = [&](const PartBufs &c, hipStream_t s) -> int {
        const ScanArgs a = scan_args(c);
        {
            StageTimer t(idx, s, VLQ_STAGE_SCAN, timed);
            launch_scan(a, s);
        }
        LAUNCHCHK();
        if (c.nsplit > 1) {
            StageTimer t(idx, s, VLQ_STAGE_MERGE, timed);
            launch_merge(c.partial, c.nq, c.nsplit, K, a.out_dist, a.out_ids, s);
        }
        LAUNCHCHK();
        return VLQ_OK;
    };

    if (parts == 1) {
        int rc = traverse(pb[0], st);
        if (rc) return rc;
        return scan(pb[0], st);
    }
    // st:    traverse(0) . scan(0) ........ scan(1) ........ scan(2) ...
    // side:              traverse(1) ....... traverse(2) ....
    // traverse(p + 1) starts when scan(p) is queued and must have finished before scan(p + 1) starts.
    int rc = traverse(pb[0], st);
    if (rc) return rc;
    for (int p = 0; p < parts; ++p) {
        if (p + 1 < parts) {
            HIPCHK(hipEventRecord(idx->ev_go[p], st)); // everything queued on st so far, traverse(p) or scan(p - 1) included
            HIPCHK(hipStreamWaitEvent(idx->side, idx->ev_go[p], 0));
        }
        rc = scan(pb[p], st);
        if (rc) return rc;
        if (p + 1 < parts) {
            rc = traverse(pb[p + 1], idx->side);
            if (rc) return rc;
            HIPCHK(hipEventRecord(idx->ev_done[p], idx->side));
            HIPCHK(hipStreamWaitEvent(st, idx->ev_done[p], 0));
        }
    }
    return VLQ_OK;
}

// Batches beyond SEARCH_TILE queries are served tile by tile (every query is independent of the
// rest of its batch), which bounds the scratch memory: the argument checks of the first tile
// cover the whole call, so nothing is written when they fail.
#define SEARCH_TILE 32768

static int search_tiled(vlq_index *idx, const float *d_q, int32_t nq, int32_t w1, int32_t w2, int32_t K,
                        float *d_out_dist, int32_t *d_out_ids, int32_t *d_cells, float *d_cell_dist, int32_t *d_sub,
                        float *d_sub_score, hipStream_t st)
{
    if (nq <= SEARCH_TILE || !idx)
        return search_impl(idx, d_q, nq, w1, w2, K, d_out_dist, d_out_ids, d_cells, d_cell_dist, d_sub, d_sub_score, st);
    const int D = idx->p.d;
    for (int64_t q0 = 0; q0 < nq; q0 += SEARCH_TILE) {
        const int32_t n = (int32_t)(nq - q0 < SEARCH_TILE ? nq - q0 : SEARCH_TILE);
        int rc = search_impl(idx, d_q ? d_q + q0 * D : nullptr, n, w1, w2, K, d_out_dist ? d_out_dist + q0 * K : nullptr,
                             d_out_ids ? d_out_ids + q0 * K : nullptr, d_cells ? d_cells + q0 * w1 : nullptr,
                             d_cell_dist ? d_cell_dist + q0 * w1 : nullptr, d_sub ? d_sub + q0 * w2 : nullptr,
                             d_sub_score ? d_sub_score + q0 * w2 : nullptr, st);
        if (rc) return rc;
    }
    return VLQ_OK;
}

extern "C" int vlq_search(const vlq_index_t *idx, const float *d_q, int32_t nq, int32_t w1, int32_t w2,
                          int32_t K, float *d_out_dist, int32_t *d_out_ids, void *stream)
{
    return search_tiled(const_cast<vlq_index *>(idx), d_q, nq, w1, w2, K, d_out_dist, d_out_ids, nullptr, nullptr,
                        nullptr, nullptr, (hipStream_t)stream);
}

extern "C" int vlq_search_debug(const vlq_index_t *idx, const float *d_q, int32_t nq, int32_t w1, int32_t w2,
                                int32_t K, float *d_out_dist, int32_t *d_out_ids, int32_t *d_cells,
                                float *d_cell_dist, int32_t *d_sub, float *d_sub_score, void *stream)
{
    return search_tiled(const_cast<vlq_index *>(idx), d_q, nq, w1, w2, K, d_out_dist, d_out_ids, d_cells, d_cell_dist,
                        d_sub, d_sub_score, (hipStream_t)stream);
}

// ---------------------------------------------------------------------------
// search without allocation
// ---------------------------------------------------------------------------
extern "C" int vlq_search_noalloc(const vlq_index_t *idx, const float *d_q, int32_t nq, int32_t w1, int32_t w2,
                                  int32_t K, float *d_out_dist, int32_t *d_out_ids, void *stream)
{
    void *ptr = nullptr;
    int rc = static_scratch(&ptr);
    if (rc) return rc;
    return search_impl(const_cast<vlq_index *>(idx), d_q, nq, w1, w2, K, d_out_dist, d_out_ids, nullptr, nullptr,
                       nullptr, nullptr, (hipStream_t)stream, ptr, (size_t)VLQ_NOALLOC_SCRATCH_BYTES);
}

// ---------------------------------------------------------------------------
// options
// ---------------------------------------------------------------------------
extern "C" int vlq_index_set_option(vlq_index_t *idx, int option, int value)
{
    if (!idx) return fail(VLQ_EINVAL, "idx is NULL");
    if (option < 0 || option >= VLQ_OPT_COUNT) return fail(VLQ_EINVAL, "unknown option %d", option);
    if (option == VLQ_OPT_SCAN_PACKED) {
        if (value < -1 || value > 1) return fail(VLQ_EINVAL, "VLQ_OPT_SCAN_PACKED takes -1, 0 or 1");
    } else if (option == VLQ_OPT_SMALL_BATCH) {
        if (value < 0) return fail(VLQ_EINVAL, "VLQ_OPT_SMALL_BATCH takes a size >= 0");
    } else if (option == VLQ_OPT_PIPELINE_PARTS) {
        if (value < 0 || value > VLQ_MAX_PARTS) return fail(VLQ_EINVAL, "VLQ_OPT_PIPELINE_PARTS takes 0 .. %d", VLQ_MAX_PARTS);
    } else if (value != 0 && value != 1) {
        return fail(VLQ_EINVAL, "option %d takes 0 or 1", option);
    }
    idx->opt[option] = value;
    return VLQ_OK;
}

extern "C" int vlq_index_set_query_lambda_range(vlq_index_t *idx, float lo, float hi)
{
    if (!idx) return fail(VLQ_EINVAL, "idx is NULL");
    if (!(lo <= hi)) return fail(VLQ_EINVAL, "query lambda range [%g, %g] is empty", (double)lo, (double)hi);
    idx->qlam_lo = lo;
    idx->qlam_hi = hi;
    return VLQ_OK;
}

// ---------------------------------------------------------------------------
// copies out
// ---------------------------------------------------------------------------
extern "C" int vlq_index_get_graph(const vlq_index_t *idx, int32_t *d_S, float *d_E, void *stream)
{
    if (!idx) return fail(VLQ_EINVAL, "idx is NULL");
    hipStream_t st = (hipStream_t)stream;
    const size_t cnt = (size_t)idx->p.nlist * idx->p.n_edges;
    if (d_S) HIPCHK(hipMemcpyAsync(d_S, idx->S, cnt * 4, hipMemcpyDeviceToDevice, st));
    if (d_E) HIPCHK(hipMemcpyAsync(d_E, idx->E, cnt * 4, hipMemcpyDeviceToDevice, st));
    return VLQ_OK;
}

extern "C" int vlq_index_get_lists(const vlq_index_t *idx, int64_t *d_off, int32_t *d_ids, uint8_t *d_codes,
                                   uint8_t *d_lambda, void *stream)
{
    if (!idx) return fail(VLQ_EINVAL, "idx is NULL");
    if (!idx->finalized) return fail(VLQ_EINVAL, "index is not finalised");
    hipStream_t st = (hipStream_t)stream;
    const size_t nl = (size_t)idx->p.nlist * idx->p.n_edges, N = (size_t)idx->ntotal;
    if (d_off) HIPCHK(hipMemcpyAsync(d_off, idx->off, (nl + 1) * 8, hipMemcpyDeviceToDevice, st));
    if (N > 0) {
        if (d_ids) HIPCHK(hipMemcpyAsync(d_ids, idx->ids, N * 4, hipMemcpyDeviceToDevice, st));
        if (d_codes) HIPCHK(hipMemcpyAsync(d_codes, idx->codes, N * idx->p.m, hipMemcpyDeviceToDevice, st));
        if (d_lambda) HIPCHK(hipMemcpyAsync(d_lambda, idx->lam, N, hipMemcpyDeviceToDevice, st));
    }
    return VLQ_OK;
}

// ---------------------------------------------------------------------------
// profiling
// ---------------------------------------------------------------------------
extern "C" int vlq_profile_enable(vlq_index_t *idx, int enable)
{
    if (!idx) return fail(VLQ_EINVAL, "idx is NULL");
    idx->prof = enable != 0;
    return VLQ_OK;
}

extern "C" int vlq_profile_read(vlq_index_t *idx, float *ms, int32_t *launches)
{
    if (!idx || !ms) return fail(VLQ_EINVAL, "NULL argument");
    for (int s = 0; s < VLQ_STAGE_COUNT; ++s) {
        ms[s] = 0.f;
        if (launches) launches[s] = 0;
    }
    int rc = VLQ_OK;
    for (auto &r : idx->recs) {
        float t = 0.f;
        hipError_t e = hipEventSynchronize(r.t1);
        if (e == hipSuccess) e = hipEventElapsedTime(&t, r.t0, r.t1);
        if (e != hipSuccess) rc = fail(VLQ_EHIP, "event timing failed: %s", hipGetErrorString(e));
        ms[r.stage] += t;
        if (launches) launches[r.stage] += 1;
        (void)hipEventDestroy(r.t0);
        (void)hipEventDestroy(r.t1);
    }
    idx->recs.clear();
    return rc;
}
