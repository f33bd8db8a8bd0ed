// Shared host/device helpers of the gfx950 SVG2 library (internal header).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "svg2.h"

namespace svg2 {

// ---- error reporting -------------------------------------------------------
int fail(int code, const char *fmt, ...);      // records the message, returns code
void clear_error();

#define SVG2_REQUIRE(cond, code, ...)                         \
    do {                                                      \
        if (!(cond)) return ::svg2::fail((code), __VA_ARGS__); \
    } while (0)

#define SVG2_HIP_CHECK(expr)                                                        \
    do {                                                                            \
        hipError_t e_ = (expr);                                                     \
        if (e_ != hipSuccess)                                                       \
            return ::svg2::fail(SVG2_HIP_ERROR, "%s: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

#define SVG2_TRY(expr)                    \
    do {                                  \
        int rc_ = (expr);                 \
        if (rc_ != SVG2_OK) return rc_;   \
    } while (0)

// Raises the dynamic-LDS limit of a kernel to `bytes` on the current device (once per kernel and device; later
// calls with the same or a smaller size return at once).  Called from the *_prepare functions, which run before
// the first launch of an entry point so that a failure leaves nothing enqueued.
int set_dynamic_lds(const void *kernel, size_t bytes);

// Kernel-level timing spans (svg2_profile_enable(2)): no-ops unless that level is on.
int profile_span_begin(int tag, hipStream_t st);
void profile_span_end(int handle, hipStream_t st);
struct ProfileSpan {            // RAII: the span covers what is enqueued on `st` during its lifetime
    int h;
    hipStream_t st;
    ProfileSpan(int tag, hipStream_t s) : h(profile_span_begin(tag, s)), st(s) {}
    ~ProfileSpan() { profile_span_end(h, st); }
    ProfileSpan(const ProfileSpan &) = delete;
    ProfileSpan &operator=(const ProfileSpan &) = delete;
};

// ---- workspace carving -----------------------------------------------------
inline size_t align256(size_t x) { return (x + 255) & ~size_t(255); }

struct Carver {
    char *base;
    size_t used;
    explicit Carver(void *p) : base(static_cast<char *>(p)), used(0) {}
    template <typename T> T *take(size_t n)
    {
        T *r = base ? reinterpret_cast<T *>(base + used) : nullptr;
        used += align256(n * sizeof(T));
        return r;
    }
};

inline int cdiv(int a, int b) { return (a + b - 1) / b; }

// ---- bf16 ------------------------------------------------------------------
typedef unsigned short bf16_t;          // raw bits

__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float(((unsigned)b) << 16); }

// round to nearest, ties to even (inputs are finite here)
__device__ __forceinline__ bf16_t f32_to_bf16(float f)
{
    unsigned u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

typedef __attribute__((address_space(3))) unsigned char lds_u8;      // byte in LDS (32-bit address)

// 16 bytes per lane from global memory (base + per-lane byte offset) straight into LDS: lane l lands at dst + 16 l.
// Written as inline assembly on purpose.  The compiler knows that its own builtin for this instruction writes LDS, cannot
// tell which part, and therefore waits for ALL outstanding loads (s_waitcnt vmcnt(0)) in front of the next LDS read of
// any address -- which turned the prefetch of the next tiles into a wait for them.  Here the order is kept by hand: a
// buffer filled this way is only read after an explicit vmcnt(0) wait and a barrier.  M0 (the LDS address of the
// instruction) is written inside the statement and named as clobbered, so that the compiler's own M0 set-ups (it keeps M0
// for itself and merges equal initialisations across blocks) are never carried over one of these statements; clang warns
// that a clobber of a register it reserves "may not be preserved", which is exactly what the clobber says.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void load_to_lds_16(const char *base, unsigned byte_off, const unsigned char *dst)
{
    const unsigned lds_addr = (unsigned)(size_t)(const lds_u8 *)dst;
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :
                 : "v"(byte_off), "s"(base), "s"(lds_addr)
                 : "memory", "m0");
}
#pragma clang diagnostic pop

template <typename T> struct Elem;
template <> struct Elem<float> {
    static __device__ __forceinline__ float load(const float *p) { return *p; }
    static __device__ __forceinline__ void store(float *p, float v) { *p = v; }
};
template <> struct Elem<bf16_t> {
    static __device__ __forceinline__ float load(const bf16_t *p) { return bf16_to_f32(*p); }
    static __device__ __forceinline__ void store(bf16_t *p, float v) { *p = f32_to_bf16(v); }
};

// ---- stage launchers (defined in the per-stage .hip files) -----------------
// All of them assume validated arguments and a workspace of the right size.

size_t kmeans_ws_bytes(int dtype, int H, int N, int d, int C);
int kmeans_prepare(int dtype, int d);
int kmeans_launch(const void *X, int dtype, int H, int N, int d, int C, int iters,
                  const float *init, float *centroids, int32_t *labels, int32_t *counts,
                  float *objective, void *ws, hipStream_t st);
// k-means of the Q tokens and of the K tokens of a layer together (one launch per step for both sides); the
// workspace holds both sides' scratch (kmeans_pair_ws_bytes)
size_t kmeans_pair_ws_bytes(int dtype, int H, int N, int d, int Cq, int Ck);
int kmeans_pair_launch(const void *Q, const void *K, int dtype, int H, int N, int d, int Cq, int Ck, int iters,
                       float *cq_inout, float *ck_inout, int32_t *labels_q, int32_t *labels_k, int32_t *counts_q,
                       int32_t *counts_k, void *ws, hipStream_t st);

// One problem of the counting sort (all heads of one side: the Q tokens or the K tokens of a layer).
struct SortSide {
    const int32_t *labels;      // [H,N] values in [0,C)
    int C, nbits;               // nbits: bits of a label (set by sort_launch)
    int32_t *hist;              // [H, ceil(N / 1024), C] scratch
    int32_t *offsets;           // [H,C+1] out
    int32_t *perm;              // [H,N] out
    int32_t *inv_perm;          // [H,N] out or null
    // optional (k-means update step): pieces of at most seg sorted rows inside one cluster
    int4 *pieces;               // [H,max_pieces] out or null
    int32_t *first_piece;       // [H,C+1] out
    int32_t *n_pieces;          // [H] out
    int max_pieces, seg;
};
struct SortArgs {
    SortSide s[2];
};
int sort_launch(SortArgs a, int nsides, int H, int N, hipStream_t st);

size_t permute_ws_bytes(int H, int N, int C);
int permute_pair_launch(const int32_t *labels_q, const int32_t *labels_k, int H, int N, int Cq, int Ck,
                        int32_t *offsets_q, int32_t *offsets_k, int32_t *perm_q, int32_t *perm_k, bool copy,
                        const void *Q, const void *K, const void *V, void *Qp, void *Kp, void *Vp, int dtype, int d,
                        void *ws, hipStream_t st);
int permute_launch(const int32_t *labels, int H, int N, int C, int32_t *offsets, int32_t *perm,
                   int32_t *inv_perm, int n_tensors, const void *const *src, void *const *dst,
                   int dtype, int d, void *ws, hipStream_t st);

// device address (on the current device) of the library's own scratch array for svg2_permute_noalloc
int permute_static_scratch(void **out);

size_t select_ws_bytes(int H, int Cq, int Ck);
int select_prepare();
int select_launch(const float *cq, const float *ck, const int32_t *counts_q, const int32_t *counts_k,
                  int H, int Cq, int Ck, int d, float top_p, int32_t *row_ptr, int32_t *col_idx,
                  float *p_est, float *density, void *ws, hipStream_t st);

size_t attn_ws_bytes(int dtype, int H, int N, int d, int Cq, int Ck);
int attn_prepare(int dtype, int d);
int attn_fp8_prepare();
int attn_launch(const void *Qp, const void *Kp, const void *Vp, int dtype, int H, int N, int d,
                int Cq, int Ck, const int32_t *offsets_q, const int32_t *offsets_k,
                const int32_t *row_ptr, const int32_t *col_idx, const int32_t *perm_q,
                const int32_t *perm_k, float scale, void *O, float *lse, void *ws, hipStream_t st);

// perm_k == nullptr: Qp, Kp, Vp are permuted copies; perm_k given: they are in token order (gather-free).
// the two halves of attn_launch, separately (so a caller can time them)
int attn_plan_launch(int dtype, int H, int N, int Cq, int Ck, const int32_t *offsets_q, const int32_t *offsets_k,
                     const int32_t *row_ptr, const int32_t *col_idx, void *ws, hipStream_t st);
int attn_main_launch(const void *Qp, const void *Kp, const void *Vp, int dtype, int H, int N, int d, int Cq, int Ck,
                     const int32_t *row_ptr, const int32_t *perm_q, const int32_t *perm_k, float scale, void *O,
                     float *lse, void *ws, hipStream_t st);

// E4M3 storage (svg2_fp8.hip)
size_t fp8_quant_ws_bytes(int H);
int fp8_quant_launch(const void *X, int dtype, int H, int N, int d, void *X8, float *scale, void *ws, hipStream_t st);
// the plan is the bf16 one (attn_plan_launch with SVG2_BF16); perm_k as in attn_main_launch
int attn_fp8_main_launch(const void *Q8, const void *K8, const void *V8, const float *scale_q, const float *scale_k,
                         const float *scale_v, int H, int N, int d, int Cq, int Ck, const int32_t *row_ptr,
                         const int32_t *perm_q, const int32_t *perm_k, float scale, void *O, float *lse, void *ws,
                         hipStream_t st);

size_t recall_ws_bytes(int H, int N);
int recall_launch(const float *lse_sel, const float *lse_all, int H, int N, float *recall, float *recall_mean,
                  void *ws, hipStream_t st);

size_t kpp_ws_bytes(int H, int N, int C);
int kpp_launch(const void *X, int dtype, int H, int N, int d, int C, const double *u, float *centroids,
               int32_t *picked, void *ws, hipStream_t st);

}  // namespace svg2
