// C ABI of the gfx950 SVG2 library: argument validation, workspace carving and
// the whole-layer entry point.  Every check happens before anything is
// launched, so an error code means no work was enqueued.
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <vector>

#include "svg2_common.h"

namespace svg2 {

static thread_local char g_err[512] = "";

int fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

void clear_error() { g_err[0] = '\0'; }

static int check_common(int dtype, int H, int N, int d)
{
    SVG2_REQUIRE(dtype == SVG2_F32 || dtype == SVG2_BF16, SVG2_UNSUPPORTED, "dtype %d is not SVG2_F32 or SVG2_BF16", dtype);
    SVG2_REQUIRE(d == 64 || d == 128, SVG2_UNSUPPORTED, "head dimension %d is not 64 or 128", d);
    SVG2_REQUIRE(H >= 1 && N >= 1, SVG2_INVALID_ARG, "H = %d and N = %d must be positive", H, N);
    SVG2_REQUIRE((double)H * (double)N * (double)d < 1099511627776.0, SVG2_INVALID_ARG, "H*N*d is 2^40 or more");
    SVG2_REQUIRE(H <= 65535, SVG2_INVALID_ARG, "H = %d exceeds 65535", H);
    return SVG2_OK;
}

// the attention kernels address the rows of one head's K and V by 32-bit signed byte offsets
static int check_head_bytes(int dtype, int N, int d)
{
    const double bytes = (double)N * (double)d * (dtype == SVG2_F32 ? 4.0 : 2.0);
    SVG2_REQUIRE(bytes < 2147483648.0, SVG2_INVALID_ARG,
                 "one head of N = %d rows of d = %d elements has 2^31 bytes or more: the attention kernels cannot address it",
                 N, d);
    return SVG2_OK;
}

// the E4M3 attention kernel exists for bf16 inputs / outputs and 128-byte rows only
static int check_fp8(int dtype, int d)
{
    SVG2_REQUIRE(dtype == SVG2_BF16, SVG2_UNSUPPORTED, "the FP8 path takes SVG2_BF16 tensors, not dtype %d", dtype);
    SVG2_REQUIRE(d == 128, SVG2_UNSUPPORTED, "the FP8 path needs head dimension 128, not %d", d);
    return SVG2_OK;
}

static int check_clusters(const char *name, int C, int N)
{
    SVG2_REQUIRE(C >= 1 && C <= SVG2_MAX_CLUSTERS && C <= N, SVG2_INVALID_ARG,
                 "%s = %d must be in 1..min(N = %d, %d)", name, C, N, SVG2_MAX_CLUSTERS);
    return SVG2_OK;
}

static int check_ws(const void *ws, size_t have, size_t need)
{
    SVG2_REQUIRE(ws != nullptr, SVG2_INVALID_ARG, "workspace pointer is null");
    SVG2_REQUIRE((reinterpret_cast<uintptr_t>(ws) & 255) == 0, SVG2_INVALID_ARG, "workspace is not 256-byte aligned");
    SVG2_REQUIRE(have >= need, SVG2_WORKSPACE_TOO_SMALL, "workspace has %zu bytes, %zu needed", have, need);
    return SVG2_OK;
}

// (kernel, device) pairs whose dynamic-LDS limit has been raised, with the size it was raised to
struct LdsAttr {
    const void *kernel;
    int device;
    size_t bytes;
};
static std::mutex g_lds_mu;
static std::vector<LdsAttr> g_lds_done;

int set_dynamic_lds(const void *kernel, size_t bytes)
{
    int dev = -1;
    SVG2_HIP_CHECK(hipGetDevice(&dev));
    std::lock_guard<std::mutex> lk(g_lds_mu);
    for (const LdsAttr &e : g_lds_done)
        if (e.kernel == kernel && e.device == dev && e.bytes >= bytes) return SVG2_OK;
    SVG2_HIP_CHECK(hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes));
    g_lds_done.push_back({kernel, dev, bytes});
    return SVG2_OK;
}

// Layout of svg2_forward's workspace.
struct ForwardLayout {
    int32_t *labels_q, *labels_k, *counts_q, *counts_k, *offsets_q, *offsets_k, *perm_q, *perm_k, *row_ptr, *col_idx;
    float *density;
    void *Qp, *Kp, *Vp;
    void *Q8, *K8, *V8;                  // E4M3 copies in token order (fp8 mode only)
    float *sq, *sk, *sv;                 // their per-head scales
    void *stage_ws;
    size_t stage_bytes, total;
};

// mode of svg2_forward: physical permutation, gather-free (no permuted copies of Q, K, V: the attention
// kernel reads rows through the permutations), or gather-free on E4M3 copies of Q, K, V
enum ForwardMode { FWD_PERMUTE = 0, FWD_GATHER_FREE = 1, FWD_FP8 = 2 };

static ForwardLayout forward_layout(void *ws, int dtype, int H, int N, int d, int Cq, int Ck, int mode)
{
    const bool gather_free = mode != FWD_PERMUTE;
    const bool fp8 = mode == FWD_FP8;
    ForwardLayout L;
    Carver c(ws);
    const size_t es = dtype == SVG2_BF16 ? 2 : 4;
    L.labels_q = c.take<int32_t>((size_t)H * N);
    L.labels_k = c.take<int32_t>((size_t)H * N);
    L.counts_q = c.take<int32_t>((size_t)H * Cq);
    L.counts_k = c.take<int32_t>((size_t)H * Ck);
    L.offsets_q = c.take<int32_t>((size_t)H * (Cq + 1));
    L.offsets_k = c.take<int32_t>((size_t)H * (Ck + 1));
    L.perm_q = c.take<int32_t>((size_t)H * N);
    L.perm_k = c.take<int32_t>((size_t)H * N);
    L.row_ptr = c.take<int32_t>((size_t)H * (Cq + 1));
    L.col_idx = c.take<int32_t>((size_t)H * Cq * Ck);
    L.density = c.take<float>((size_t)H);
    L.Qp = c.take<char>(gather_free ? 0 : (size_t)H * N * d * es);
    L.Kp = c.take<char>(gather_free ? 0 : (size_t)H * N * d * es);
    L.Vp = c.take<char>(gather_free ? 0 : (size_t)H * N * d * es);
    L.Q8 = c.take<char>(fp8 ? (size_t)H * N * d : 0);
    L.K8 = c.take<char>(fp8 ? (size_t)H * N * d : 0);
    L.V8 = c.take<char>(fp8 ? (size_t)H * N * d : 0);
    L.sq = c.take<float>(fp8 ? (size_t)H : 0);
    L.sk = c.take<float>(fp8 ? (size_t)H : 0);
    L.sv = c.take<float>(fp8 ? (size_t)H : 0);
    // the stages run one after another on one stream and share one scratch area
    size_t s = kmeans_pair_ws_bytes(dtype, H, N, d, Cq, Ck);     // both sides run in the same launches
    size_t t = permute_ws_bytes(H, N, Cq) + permute_ws_bytes(H, N, Ck);
    if (t > s) s = t;
    t = select_ws_bytes(H, Cq, Ck);
    if (t > s) s = t;
    t = attn_ws_bytes(dtype, H, N, d, Cq, Ck);
    if (t > s) s = t;
    t = fp8 ? fp8_quant_ws_bytes(H) : 0;
    if (t > s) s = t;
    L.stage_bytes = s;
    L.stage_ws = c.take<char>(s);
    L.total = c.used;
    return L;
}

// ---- optional timing (svg2_profile_*) ------------------------------------------
// Level 1: HIP events around the stages of svg2_forward.  Level 2: additionally an event pair around every kernel
// launch of the stages that consist of several kernels (k-means, permutation), summed per kernel class.  The events
// of level 2 sit between kernels that otherwise run back to back, so a level-2 pass is for attributing time, not
// for timing the layer.
struct Profiler {
    std::mutex mu;
    int level = 0;
    int ncalls = 0;
    std::vector<hipEvent_t> ev;          // (SVG2_N_STAGES + 1) events per recorded call
    std::vector<hipEvent_t> kev;         // pool of event pairs for kernel spans
    std::vector<int> ktag;               // tag of span i (events 2 i, 2 i + 1 of kev)
    size_t nspans = 0;
};
static Profiler g_prof;

// Returns the event slot base for this call, or -1 when not recording.
static int profile_begin_call()
{
    std::lock_guard<std::mutex> lk(g_prof.mu);
    if (g_prof.level == 0 || g_prof.ncalls >= SVG2_PROFILE_MAX_CALLS) return -1;
    const size_t need = (size_t)(g_prof.ncalls + 1) * (SVG2_N_STAGES + 1);
    while (g_prof.ev.size() < need) {
        hipEvent_t e;
        if (hipEventCreate(&e) != hipSuccess) return -1;
        g_prof.ev.push_back(e);
    }
    return (g_prof.ncalls++) * (SVG2_N_STAGES + 1);
}

static void profile_mark(int base, int k, hipStream_t st)
{
    if (base >= 0) (void)hipEventRecord(g_prof.ev[base + k], st);
}

// kernel spans (level 2): span_begin returns a handle for span_end, or -1 when not recording
int profile_span_begin(int tag, hipStream_t st)
{
    if (g_prof.level < 2) return -1;
    std::lock_guard<std::mutex> lk(g_prof.mu);
    if (g_prof.nspans >= (size_t)SVG2_PROFILE_MAX_SPANS) return -1;
    while (g_prof.kev.size() < 2 * (g_prof.nspans + 1)) {
        hipEvent_t e;
        if (hipEventCreate(&e) != hipSuccess) return -1;
        g_prof.kev.push_back(e);
    }
    const int i = (int)g_prof.nspans++;
    if (g_prof.ktag.size() <= (size_t)i) g_prof.ktag.resize(i + 1);
    g_prof.ktag[i] = tag;
    (void)hipEventRecord(g_prof.kev[2 * i], st);
    return i;
}

void profile_span_end(int handle, hipStream_t st)
{
    if (handle >= 0) (void)hipEventRecord(g_prof.kev[2 * handle + 1], st);
}

}  // namespace svg2

using namespace svg2;

extern "C" {

const char *svg2_last_error(void) { return g_err; }

int svg2_version(void) { return 100; }

size_t svg2_kmeans_workspace_size(int dtype, int H, int N, int d, int C)
{
    if (check_common(dtype, H, N, d) != SVG2_OK || check_clusters("C", C, N) != SVG2_OK) return 256;
    return kmeans_ws_bytes(dtype, H, N, d, C);
}

int svg2_kmeans(const void *X, int dtype, int H, int N, int d, int C, int iters, const float *init_centroids,
                float *centroids, int32_t *labels, int32_t *counts, float *objective, void *ws, size_t ws_bytes,
                void *stream)
{
    clear_error();
    SVG2_TRY(check_common(dtype, H, N, d));
    SVG2_TRY(check_clusters("C", C, N));
    SVG2_REQUIRE(iters >= 1, SVG2_INVALID_ARG, "iters = %d must be at least 1", iters);
    SVG2_REQUIRE(X && init_centroids && centroids && labels && counts, SVG2_INVALID_ARG,
                 "X, init_centroids, centroids, labels and counts must be non-null");
    SVG2_TRY(check_ws(ws, ws_bytes, kmeans_ws_bytes(dtype, H, N, d, C)));
    SVG2_TRY(kmeans_prepare(dtype, d));
    return kmeans_launch(X, dtype, H, N, d, C, iters, init_centroids, centroids, labels, counts, objective, ws,
                         static_cast<hipStream_t>(stream));
}

size_t svg2_permute_workspace_size(int H, int N, int C)
{
    if (H < 1 || N < 1 || C < 1 || C > SVG2_MAX_CLUSTERS) return 256;
    return permute_ws_bytes(H, N, C);
}

int svg2_permute(const int32_t *labels, int H, int N, int C, int32_t *offsets, int32_t *perm, int32_t *inv_perm,
                 int n_tensors, const void *const *src, void *const *dst, int dtype, int d, void *ws,
                 size_t ws_bytes, void *stream)
{
    clear_error();
    SVG2_REQUIRE(H >= 1 && H <= 65535 && N >= 1, SVG2_INVALID_ARG, "H = %d (1..65535) and N = %d must be positive", H, N);
    SVG2_REQUIRE(C >= 1 && C <= SVG2_MAX_CLUSTERS, SVG2_INVALID_ARG, "C = %d must be in 1..%d", C, SVG2_MAX_CLUSTERS);
    SVG2_REQUIRE(labels && offsets && perm, SVG2_INVALID_ARG, "labels, offsets and perm must be non-null");
    SVG2_REQUIRE(n_tensors >= 0 && n_tensors <= 2, SVG2_INVALID_ARG, "n_tensors = %d must be 0, 1 or 2", n_tensors);
    if (n_tensors > 0) {
        SVG2_TRY(check_common(dtype, H, N, d));
        SVG2_REQUIRE(src && dst, SVG2_INVALID_ARG, "src and dst must be non-null when n_tensors > 0");
        for (int t = 0; t < n_tensors; ++t) {
            SVG2_REQUIRE(src[t] && dst[t], SVG2_INVALID_ARG, "src[%d] / dst[%d] is null", t, t);
            SVG2_REQUIRE(src[t] != dst[t], SVG2_INVALID_ARG, "dst[%d] must not alias src[%d]", t, t);
        }
    }
    SVG2_TRY(check_ws(ws, ws_bytes, permute_ws_bytes(H, N, C)));
    return permute_launch(labels, H, N, C, offsets, perm, inv_perm, n_tensors, src, dst, dtype, d, ws,
                          static_cast<hipStream_t>(stream));
}

int svg2_permute_noalloc(const int32_t *labels, int H, int N, int C, int32_t *offsets, int32_t *perm,
                         int32_t *inv_perm, int n_tensors, const void *const *src, void *const *dst, int dtype, int d,
                         void *stream)
{
    clear_error();
    SVG2_REQUIRE(H >= 1 && H <= 65535 && N >= 1, SVG2_INVALID_ARG, "H = %d (1..65535) and N = %d must be positive", H, N);
    SVG2_REQUIRE(C >= 1 && C <= SVG2_MAX_CLUSTERS, SVG2_INVALID_ARG, "C = %d must be in 1..%d", C, SVG2_MAX_CLUSTERS);
    SVG2_REQUIRE(labels && offsets && perm, SVG2_INVALID_ARG, "labels, offsets and perm must be non-null");
    SVG2_REQUIRE(n_tensors >= 0 && n_tensors <= 2, SVG2_INVALID_ARG, "n_tensors = %d must be 0, 1 or 2", n_tensors);
    if (n_tensors > 0) {
        SVG2_TRY(check_common(dtype, H, N, d));
        SVG2_REQUIRE(src && dst, SVG2_INVALID_ARG, "src and dst must be non-null when n_tensors > 0");
        for (int t = 0; t < n_tensors; ++t) {
            SVG2_REQUIRE(src[t] && dst[t], SVG2_INVALID_ARG, "src[%d] / dst[%d] is null", t, t);
            SVG2_REQUIRE(src[t] != dst[t], SVG2_INVALID_ARG, "dst[%d] must not alias src[%d]", t, t);
        }
    }
    const size_t need = permute_ws_bytes(H, N, C);
    SVG2_REQUIRE(need <= (size_t)SVG2_PERMUTE_NOALLOC_SCRATCH_BYTES, SVG2_WORKSPACE_TOO_SMALL,
                 "svg2_permute_noalloc: H = %d, N = %d, C = %d needs %zu bytes of scratch, the built-in array has %zu "
                 "(use svg2_permute with a workspace)",
                 H, N, C, need, (size_t)SVG2_PERMUTE_NOALLOC_SCRATCH_BYTES);
    void *scratch_ptr = nullptr;
    SVG2_TRY(permute_static_scratch(&scratch_ptr));
    return permute_launch(labels, H, N, C, offsets, perm, inv_perm, n_tensors, src, dst, dtype, d, scratch_ptr,
                          static_cast<hipStream_t>(stream));
}

size_t svg2_select_topp_workspace_size(int H, int Cq, int Ck)
{
    if (H < 1 || Cq < 1 || Ck < 1 || Cq > SVG2_MAX_CLUSTERS || Ck > SVG2_MAX_CLUSTERS) return 256;
    return select_ws_bytes(H, Cq, Ck);
}

int svg2_select_topp(const float *cq, const float *ck, const int32_t *counts_q, const int32_t *counts_k, int H,
                     int Cq, int Ck, int d, float top_p, int32_t *row_ptr, int32_t *col_idx, float *p_est,
                     float *density, void *ws, size_t ws_bytes, void *stream)
{
    clear_error();
    SVG2_REQUIRE(H >= 1 && H <= 65535, SVG2_INVALID_ARG, "H = %d must be in 1..65535", H);
    SVG2_REQUIRE(d == 64 || d == 128, SVG2_UNSUPPORTED, "head dimension %d is not 64 or 128", d);
    SVG2_REQUIRE(Cq >= 1 && Cq <= SVG2_MAX_CLUSTERS && Ck >= 1 && Ck <= SVG2_MAX_CLUSTERS, SVG2_INVALID_ARG,
                 "Cq = %d and Ck = %d must be in 1..%d", Cq, Ck, SVG2_MAX_CLUSTERS);
    SVG2_REQUIRE(top_p > 0.f && top_p <= 1.f, SVG2_INVALID_ARG, "top_p = %g must be in (0, 1]", (double)top_p);
    SVG2_REQUIRE(cq && ck && counts_k && row_ptr && col_idx, SVG2_INVALID_ARG,
                 "cq, ck, counts_k, row_ptr and col_idx must be non-null");
    SVG2_REQUIRE(!density || counts_q, SVG2_INVALID_ARG, "density needs counts_q");
    SVG2_TRY(check_ws(ws, ws_bytes, select_ws_bytes(H, Cq, Ck)));
    SVG2_TRY(select_prepare());
    return select_launch(cq, ck, counts_q, counts_k, H, Cq, Ck, d, top_p, row_ptr, col_idx, p_est, density, ws,
                         static_cast<hipStream_t>(stream));
}

size_t svg2_sparse_attn_workspace_size(int dtype, int H, int N, int d, int Cq, int Ck)
{
    if (check_common(dtype, H, N, d) != SVG2_OK || Cq < 1 || Ck < 1 || Cq > SVG2_MAX_CLUSTERS ||
        Ck > SVG2_MAX_CLUSTERS)
        return 256;
    return attn_ws_bytes(dtype, H, N, d, Cq, Ck);
}

int svg2_sparse_attn(const void *Qp, const void *Kp, const void *Vp, int dtype, int H, int N, int d, int Cq, int Ck,
                     const int32_t *offsets_q, const int32_t *offsets_k, const int32_t *row_ptr,
                     const int32_t *col_idx, const int32_t *perm_q, float scale, void *O, float *lse, void *ws,
                     size_t ws_bytes, void *stream)
{
    clear_error();
    SVG2_TRY(check_common(dtype, H, N, d));
    SVG2_TRY(check_head_bytes(dtype, N, d));
    SVG2_TRY(check_clusters("Cq", Cq, N));
    SVG2_TRY(check_clusters("Ck", Ck, N));
    SVG2_REQUIRE(Qp && Kp && Vp && O && offsets_q && offsets_k && row_ptr && col_idx, SVG2_INVALID_ARG,
                 "Qp, Kp, Vp, O, offsets_q, offsets_k, row_ptr and col_idx must be non-null");
    SVG2_REQUIRE(O != Qp && O != Kp && O != Vp, SVG2_INVALID_ARG, "O must not alias an input");
    SVG2_TRY(check_ws(ws, ws_bytes, attn_ws_bytes(dtype, H, N, d, Cq, Ck)));
    SVG2_TRY(attn_prepare(dtype, d));
    return attn_launch(Qp, Kp, Vp, dtype, H, N, d, Cq, Ck, offsets_q, offsets_k, row_ptr, col_idx, perm_q, nullptr,
                       scale, O, lse, ws, static_cast<hipStream_t>(stream));
}

int svg2_sparse_attn_gather_free(const void *Q, const void *K, const void *V, int dtype, int H, int N, int d, int Cq,
                                 int Ck, const int32_t *offsets_q, const int32_t *offsets_k, const int32_t *row_ptr,
                                 const int32_t *col_idx, const int32_t *perm_q, const int32_t *perm_k, float scale,
                                 void *O, float *lse, void *ws, size_t ws_bytes, void *stream)
{
    clear_error();
    SVG2_TRY(check_common(dtype, H, N, d));
    SVG2_TRY(check_head_bytes(dtype, N, d));
    SVG2_TRY(check_clusters("Cq", Cq, N));
    SVG2_TRY(check_clusters("Ck", Ck, N));
    SVG2_REQUIRE(Q && K && V && O && offsets_q && offsets_k && row_ptr && col_idx && perm_q && perm_k,
                 SVG2_INVALID_ARG,
                 "Q, K, V, O, offsets_q, offsets_k, row_ptr, col_idx, perm_q and perm_k must be non-null");
    SVG2_REQUIRE(O != Q && O != K && O != V, SVG2_INVALID_ARG, "O must not alias an input");
    SVG2_TRY(check_ws(ws, ws_bytes, attn_ws_bytes(dtype, H, N, d, Cq, Ck)));
    SVG2_TRY(attn_prepare(dtype, d));
    return attn_launch(Q, K, V, dtype, H, N, d, Cq, Ck, offsets_q, offsets_k, row_ptr, col_idx, perm_q, perm_k, scale,
                       O, lse, ws, static_cast<hipStream_t>(stream));
}

size_t svg2_forward_workspace_size(int dtype, int H, int N, int d, int Cq, int Ck)
{
    if (check_common(dtype, H, N, d) != SVG2_OK || check_clusters("Cq", Cq, N) != SVG2_OK ||
        check_clusters("Ck", Ck, N) != SVG2_OK)
        return 256;
    return forward_layout(nullptr, dtype, H, N, d, Cq, Ck, FWD_PERMUTE).total;
}

size_t svg2_forward_gather_free_workspace_size(int dtype, int H, int N, int d, int Cq, int Ck)
{
    if (check_common(dtype, H, N, d) != SVG2_OK || check_clusters("Cq", Cq, N) != SVG2_OK ||
        check_clusters("Ck", Ck, N) != SVG2_OK)
        return 256;
    return forward_layout(nullptr, dtype, H, N, d, Cq, Ck, FWD_GATHER_FREE).total;
}

}  // extern "C"

static int forward_impl(const void *Q, const void *K, const void *V, int dtype, int H, int N, int d, int Cq, int Ck,
                        float top_p, int iters, float *cq_inout, float *ck_inout, void *O,
                        const svg2_forward_aux *aux, void *ws, size_t ws_bytes, void *stream, int mode)
{
    clear_error();
    const bool gather_free = mode != FWD_PERMUTE;
    SVG2_TRY(check_common(dtype, H, N, d));
    // k-means runs the Q and the K side of every head in the same launches: 2 H entries in one grid dimension
    SVG2_REQUIRE(H <= 32767, SVG2_INVALID_ARG, "H = %d exceeds 32767, the limit of the svg2_forward calls", H);
    SVG2_TRY(check_head_bytes(dtype, N, d));
    if (mode == FWD_FP8) SVG2_TRY(check_fp8(dtype, d));
    SVG2_TRY(check_clusters("Cq", Cq, N));
    SVG2_TRY(check_clusters("Ck", Ck, N));
    SVG2_REQUIRE(iters >= 1, SVG2_INVALID_ARG, "iters = %d must be at least 1", iters);
    SVG2_REQUIRE(top_p > 0.f && top_p <= 1.f, SVG2_INVALID_ARG, "top_p = %g must be in (0, 1]", (double)top_p);
    SVG2_REQUIRE(Q && K && V && O && cq_inout && ck_inout, SVG2_INVALID_ARG,
                 "Q, K, V, O, cq_inout and ck_inout must be non-null");
    SVG2_REQUIRE(O != Q && O != K && O != V, SVG2_INVALID_ARG, "O must not alias an input");
    SVG2_REQUIRE(ws != nullptr, SVG2_INVALID_ARG, "workspace pointer is null");
    ForwardLayout L = forward_layout(ws, dtype, H, N, d, Cq, Ck, mode);
    SVG2_TRY(check_ws(ws, ws_bytes, L.total));
    float *lse = nullptr;
    if (aux) {
        if (aux->labels_q) L.labels_q = aux->labels_q;
        if (aux->labels_k) L.labels_k = aux->labels_k;
        if (aux->counts_q) L.counts_q = aux->counts_q;
        if (aux->counts_k) L.counts_k = aux->counts_k;
        if (aux->offsets_q) L.offsets_q = aux->offsets_q;
        if (aux->offsets_k) L.offsets_k = aux->offsets_k;
        if (aux->perm_q) L.perm_q = aux->perm_q;
        if (aux->perm_k) L.perm_k = aux->perm_k;
        if (aux->row_ptr) L.row_ptr = aux->row_ptr;
        if (aux->col_idx) L.col_idx = aux->col_idx;
        if (aux->density) L.density = aux->density;
        lse = aux->lse;
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    // everything that can fail without a kernel having been launched comes first
    SVG2_TRY(kmeans_prepare(dtype, d));
    SVG2_TRY(select_prepare());
    if (mode == FWD_FP8) SVG2_TRY(attn_fp8_prepare());
    else SVG2_TRY(attn_prepare(dtype, d));
    const int pb = profile_begin_call();
    profile_mark(pb, 0, st);
    // Section 4.1: cluster Q and K independently (both sides share every launch)
    SVG2_TRY(kmeans_pair_launch(Q, K, dtype, H, N, d, Cq, Ck, iters, cq_inout, ck_inout, L.labels_q, L.labels_k,
                                L.counts_q, L.counts_k, L.stage_ws, st));
    profile_mark(pb, 1, st);
    // Section 4.1: permutations; K and V share pi_k
    // (gather-free: only the index vectors; the rows are fetched through them in the attention kernel)
    SVG2_TRY(permute_pair_launch(L.labels_q, L.labels_k, H, N, Cq, Ck, L.offsets_q, L.offsets_k, L.perm_q, L.perm_k,
                                 !gather_free, Q, K, V, L.Qp, L.Kp, L.Vp, dtype, d, L.stage_ws, st));
    if (mode == FWD_FP8) {              // E4M3 copies in token order, one scale per head and tensor
        SVG2_TRY(fp8_quant_launch(Q, dtype, H, N, d, L.Q8, L.sq, L.stage_ws, st));
        SVG2_TRY(fp8_quant_launch(K, dtype, H, N, d, L.K8, L.sk, L.stage_ws, st));
        SVG2_TRY(fp8_quant_launch(V, dtype, H, N, d, L.V8, L.sv, L.stage_ws, st));
    }
    profile_mark(pb, 2, st);
    // Section 4.2: which (query cluster, key cluster) pairs to compute
    SVG2_TRY(select_launch(cq_inout, ck_inout, L.counts_q, L.counts_k, H, Cq, Ck, d, top_p, L.row_ptr, L.col_idx,
                           nullptr, L.density, L.stage_ws, st));
    profile_mark(pb, 3, st);
    // Section 4.3: attention over the selected pairs, result back in token order
    SVG2_TRY(attn_plan_launch(dtype, H, N, Cq, Ck, L.offsets_q, L.offsets_k, L.row_ptr, L.col_idx, L.stage_ws, st));
    profile_mark(pb, 4, st);
    if (mode == FWD_FP8)
        SVG2_TRY(attn_fp8_main_launch(L.Q8, L.K8, L.V8, L.sq, L.sk, L.sv, H, N, d, Cq, Ck, L.row_ptr, L.perm_q, L.perm_k,
                                      0.f, O, lse, L.stage_ws, st));
    else if (gather_free)
        SVG2_TRY(attn_main_launch(Q, K, V, dtype, H, N, d, Cq, Ck, L.row_ptr, L.perm_q, L.perm_k, 0.f, O, lse,
                                  L.stage_ws, st));
    else
        SVG2_TRY(attn_main_launch(L.Qp, L.Kp, L.Vp, dtype, H, N, d, Cq, Ck, L.row_ptr, L.perm_q, nullptr, 0.f, O, lse,
                                  L.stage_ws, st));
    profile_mark(pb, 5, st);
    return SVG2_OK;
}

extern "C" {

int svg2_forward(const void *Q, const void *K, const void *V, int dtype, int H, int N, int d, int Cq, int Ck,
                 float top_p, int iters, float *cq_inout, float *ck_inout, void *O, const svg2_forward_aux *aux,
                 void *ws, size_t ws_bytes, void *stream)
{
    return forward_impl(Q, K, V, dtype, H, N, d, Cq, Ck, top_p, iters, cq_inout, ck_inout, O, aux, ws, ws_bytes,
                        stream, FWD_PERMUTE);
}

int svg2_forward_gather_free(const void *Q, const void *K, const void *V, int dtype, int H, int N, int d, int Cq,
                             int Ck, float top_p, int iters, float *cq_inout, float *ck_inout, void *O,
                             const svg2_forward_aux *aux, void *ws, size_t ws_bytes, void *stream)
{
    return forward_impl(Q, K, V, dtype, H, N, d, Cq, Ck, top_p, iters, cq_inout, ck_inout, O, aux, ws, ws_bytes,
                        stream, FWD_GATHER_FREE);
}

size_t svg2_forward_fp8_workspace_size(int dtype, int H, int N, int d, int Cq, int Ck)
{
    if (check_common(dtype, H, N, d) != SVG2_OK || check_fp8(dtype, d) != SVG2_OK ||
        check_clusters("Cq", Cq, N) != SVG2_OK || check_clusters("Ck", Ck, N) != SVG2_OK)
        return 256;
    return forward_layout(nullptr, dtype, H, N, d, Cq, Ck, FWD_FP8).total;
}

int svg2_forward_fp8(const void *Q, const void *K, const void *V, int dtype, int H, int N, int d, int Cq, int Ck,
                     float top_p, int iters, float *cq_inout, float *ck_inout, void *O, const svg2_forward_aux *aux,
                     void *ws, size_t ws_bytes, void *stream)
{
    return forward_impl(Q, K, V, dtype, H, N, d, Cq, Ck, top_p, iters, cq_inout, ck_inout, O, aux, ws, ws_bytes,
                        stream, FWD_FP8);
}

size_t svg2_quantize_fp8_workspace_size(int H)
{
    if (H < 1) return 256;
    return fp8_quant_ws_bytes(H);
}

int svg2_quantize_fp8(const void *X, int dtype, int H, int N, int d, void *X8, float *scale, void *ws, size_t ws_bytes,
                      void *stream)
{
    clear_error();
    SVG2_TRY(check_common(dtype, H, N, d));
    SVG2_REQUIRE(X && X8 && scale, SVG2_INVALID_ARG, "X, X8 and scale must be non-null");
    SVG2_REQUIRE(X != X8, SVG2_INVALID_ARG, "X8 must not alias X");
    SVG2_TRY(check_ws(ws, ws_bytes, fp8_quant_ws_bytes(H)));
    return fp8_quant_launch(X, dtype, H, N, d, X8, scale, ws, static_cast<hipStream_t>(stream));
}

int svg2_sparse_attn_fp8(const void *Q8, const void *K8, const void *V8, const float *scale_q, const float *scale_k,
                         const float *scale_v, int H, int N, int d, int Cq, int Ck, const int32_t *offsets_q,
                         const int32_t *offsets_k, const int32_t *row_ptr, const int32_t *col_idx,
                         const int32_t *perm_q, const int32_t *perm_k, float scale, void *O, float *lse, void *ws,
                         size_t ws_bytes, void *stream)
{
    clear_error();
    SVG2_TRY(check_common(SVG2_BF16, H, N, d));
    SVG2_TRY(check_head_bytes(SVG2_BF16, N, d));
    SVG2_TRY(check_fp8(SVG2_BF16, d));
    SVG2_TRY(check_clusters("Cq", Cq, N));
    SVG2_TRY(check_clusters("Ck", Ck, N));
    SVG2_REQUIRE(Q8 && K8 && V8 && scale_q && scale_k && scale_v && O && offsets_q && offsets_k && row_ptr && col_idx,
                 SVG2_INVALID_ARG,
                 "Q8, K8, V8, the three scales, O, offsets_q, offsets_k, row_ptr and col_idx must be non-null");
    SVG2_REQUIRE(!perm_k || perm_q, SVG2_INVALID_ARG, "perm_k (operands in token order) needs perm_q");
    SVG2_REQUIRE(O != Q8 && O != K8 && O != V8, SVG2_INVALID_ARG, "O must not alias an input");
    SVG2_TRY(check_ws(ws, ws_bytes, attn_ws_bytes(SVG2_BF16, H, N, d, Cq, Ck)));
    SVG2_TRY(attn_fp8_prepare());
    hipStream_t st = static_cast<hipStream_t>(stream);
    SVG2_TRY(attn_plan_launch(SVG2_BF16, H, N, Cq, Ck, offsets_q, offsets_k, row_ptr, col_idx, ws, st));
    return attn_fp8_main_launch(Q8, K8, V8, scale_q, scale_k, scale_v, H, N, d, Cq, Ck, row_ptr, perm_q, perm_k, scale,
                                O, lse, ws, st);
}

size_t svg2_attention_recall_workspace_size(int H, int N)
{
    if (H < 1 || N < 1) return 256;
    return recall_ws_bytes(H, N);
}

int svg2_attention_recall(const float *lse_selected, const float *lse_all, int H, int N, float *recall,
                          float *recall_mean, void *ws, size_t ws_bytes, void *stream)
{
    clear_error();
    SVG2_REQUIRE(H >= 1 && H <= 65535 && N >= 1, SVG2_INVALID_ARG, "H = %d (1..65535) and N = %d must be positive", H, N);
    SVG2_REQUIRE(lse_selected && lse_all && recall_mean, SVG2_INVALID_ARG,
                 "lse_selected, lse_all and recall_mean must be non-null");
    SVG2_TRY(check_ws(ws, ws_bytes, recall_ws_bytes(H, N)));
    return recall_launch(lse_selected, lse_all, H, N, recall, recall_mean, ws, static_cast<hipStream_t>(stream));
}

size_t svg2_kmeans_pp_init_workspace_size(int H, int N, int C)
{
    if (H < 1 || N < 1 || C < 1 || C > SVG2_MAX_CLUSTERS) return 256;
    return kpp_ws_bytes(H, N, C);
}

int svg2_kmeans_pp_init(const void *X, int dtype, int H, int N, int d, int C, const double *u, float *centroids,
                        int32_t *picked, void *ws, size_t ws_bytes, void *stream)
{
    clear_error();
    SVG2_TRY(check_common(dtype, H, N, d));
    SVG2_TRY(check_clusters("C", C, N));
    SVG2_REQUIRE(X && u && centroids, SVG2_INVALID_ARG, "X, u and centroids must be non-null");
    SVG2_TRY(check_ws(ws, ws_bytes, kpp_ws_bytes(H, N, C)));
    return kpp_launch(X, dtype, H, N, d, C, u, centroids, picked, ws, static_cast<hipStream_t>(stream));
}

int svg2_profile_enable(int level)
{
    std::lock_guard<std::mutex> lk(g_prof.mu);
    g_prof.level = level < 0 ? 0 : (level > 2 ? 2 : level);
    return SVG2_OK;
}

int svg2_profile_read(float *stage_ms, int *n_calls)
{
    clear_error();
    SVG2_REQUIRE(stage_ms && n_calls, SVG2_INVALID_ARG, "stage_ms and n_calls must be non-null");
    std::lock_guard<std::mutex> lk(g_prof.mu);
    for (int k = 0; k < SVG2_N_STAGES; ++k) stage_ms[k] = 0.f;
    for (int c = 0; c < g_prof.ncalls; ++c) {
        const int base = c * (SVG2_N_STAGES + 1);
        SVG2_HIP_CHECK(hipEventSynchronize(g_prof.ev[base + SVG2_N_STAGES]));
        for (int k = 0; k < SVG2_N_STAGES; ++k) {
            float ms = 0.f;
            SVG2_HIP_CHECK(hipEventElapsedTime(&ms, g_prof.ev[base + k], g_prof.ev[base + k + 1]));
            stage_ms[k] += ms;
        }
    }
    *n_calls = g_prof.ncalls;
    g_prof.ncalls = 0;
    return SVG2_OK;
}

int svg2_profile_read_kernels(float *kernel_ms, int *launches)
{
    clear_error();
    SVG2_REQUIRE(kernel_ms && launches, SVG2_INVALID_ARG, "kernel_ms and launches must be non-null");
    std::lock_guard<std::mutex> lk(g_prof.mu);
    for (int k = 0; k < SVG2_N_KERNEL_CLASSES; ++k) { kernel_ms[k] = 0.f; launches[k] = 0; }
    for (size_t i = 0; i < g_prof.nspans; ++i) {
        float ms = 0.f;
        SVG2_HIP_CHECK(hipEventSynchronize(g_prof.kev[2 * i + 1]));
        SVG2_HIP_CHECK(hipEventElapsedTime(&ms, g_prof.kev[2 * i], g_prof.kev[2 * i + 1]));
        const int tag = g_prof.ktag[i];
        if (tag >= 0 && tag < SVG2_N_KERNEL_CLASSES) { kernel_ms[tag] += ms; launches[tag] += 1; }
    }
    g_prof.nspans = 0;
    return SVG2_OK;
}

}  // extern "C"
