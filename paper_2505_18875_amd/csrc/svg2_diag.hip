// Two pieces around the layer path that the paper uses but that are not on the per-step hot path:
//
//   attention recall (Section 3.1)   the share of a query's true attention mass that its
//                                    selected keys capture.  With lse_sel the log-sum-exp of the
//                                    scores over the selected keys (svg2_sparse_attn's lse) and
//                                    lse_all the one over all keys (the dense special case),
//                                    recall = exp(lse_sel - lse_all).
//   k-means++ seeding (Section 4.3)  the initialisation an un-cached k-means starts from: the
//                                    first centre is a given token, every further centre is drawn
//                                    with probability D2 / sum(D2), D2 = squared distance to the
//                                    nearest centre so far.  The uniform random numbers are an
//                                    input, so the draw is reproducible and can be checked.  All
//                                    arithmetic is fp64 (the draw compares a running sum of D2
//                                    with a threshold; fp32 would move the boundaries).
#include "svg2_common.h"

namespace svg2 {

static constexpr int DG_BLOCK = 1024;       // tokens per workgroup in the recall kernel (256 threads x 4)
static constexpr int KPP_BLOCK = 256;       // tokens per block sum in k-means++

// ---------------------------------------------------------------- recall
// grid (nblk, H), block 256
__global__ __launch_bounds__(256) void recall_rows_kernel(const float *__restrict__ lse_sel,
                                                          const float *__restrict__ lse_all, int N, int nblk,
                                                          float *__restrict__ recall, float *__restrict__ partial)
{
    __shared__ float s_red[256];
    const int h = blockIdx.y, tid = threadIdx.x;
    float acc = 0.f;
    for (int k = 0; k < 4; ++k) {
        const int n = blockIdx.x * DG_BLOCK + k * 256 + tid;
        if (n < N) {
            const float a = lse_sel[(size_t)h * N + n], b = lse_all[(size_t)h * N + n];
            const float r = (a == -INFINITY) ? 0.f : expf(a - b);
            if (recall) recall[(size_t)h * N + n] = r;
            acc += r;
        }
    }
    s_red[tid] = acc;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {         // fixed order: reproducible
        if (tid < o) s_red[tid] += s_red[tid + o];
        __syncthreads();
    }
    if (tid == 0) partial[(size_t)h * nblk + blockIdx.x] = s_red[0];
}

// grid (H), block 64
__global__ void recall_mean_kernel(const float *__restrict__ partial, int N, int nblk, float *__restrict__ mean)
{
    const int h = blockIdx.x;
    if (threadIdx.x == 0) {
        double s = 0.0;
        for (int b = 0; b < nblk; ++b) s += (double)partial[(size_t)h * nblk + b];
        mean[h] = (float)(s / (double)N);
    }
}

size_t recall_ws_bytes(int H, int N) { return align256((size_t)H * cdiv(N, DG_BLOCK) * sizeof(float)); }

int recall_launch(const float *lse_sel, const float *lse_all, int H, int N, float *recall, float *recall_mean,
                  void *ws, hipStream_t st)
{
    const int nblk = cdiv(N, DG_BLOCK);
    float *partial = static_cast<float *>(ws);
    hipLaunchKernelGGL(recall_rows_kernel, dim3(nblk, H), dim3(256), 0, st, lse_sel, lse_all, N, nblk, recall, partial);
    hipLaunchKernelGGL(recall_mean_kernel, dim3(H), dim3(64), 0, st, partial, N, nblk, recall_mean);
    SVG2_HIP_CHECK(hipGetLastError());
    return SVG2_OK;
}

// ---------------------------------------------------------------- k-means++
// One draw.  grid (H), block 256.  k = 0: token floor(u * N).  Otherwise the first token whose running
// sum of D2 exceeds u * sum(D2): the workgroup first finds the block of KPP_BLOCK tokens in which the running sum
// crosses the threshold (block sums come from the update kernel), then the token inside it.
template <typename T>
__global__ __launch_bounds__(256) void kpp_pick_kernel(const T *__restrict__ X, const double *__restrict__ u,
                                                       const double *__restrict__ d2,
                                                       const double *__restrict__ bsum, int N, int d, int C, int k,
                                                       int nblk, int32_t *__restrict__ picked,
                                                       float *__restrict__ centroids)
{
    __shared__ double s_scan[256];
    __shared__ int s_pick;
    const int h = blockIdx.x, tid = threadIdx.x;
    const double uk = u[(size_t)h * C + k];
    const double *dh = d2 + (size_t)h * N;
    // The running sum is taken hierarchically (block sums, then groups of 4 tokens, then tokens), every level
    // with a 256-wide inclusive scan in LDS; the first position whose inclusive sum exceeds the threshold wins.
    __shared__ double s_base;
    __shared__ int s_blk;
    auto scan256 = [&](double v) {              // inclusive scan over the workgroup (Hillis-Steele in LDS)
        s_scan[tid] = v;
        __syncthreads();
        for (int o = 1; o < 256; o <<= 1) {
            const double t = (tid >= o) ? s_scan[tid - o] : 0.0;
            __syncthreads();
            s_scan[tid] += t;
            __syncthreads();
        }
        return s_scan[tid];
    };
    if (tid == 0) { s_pick = -1; s_blk = 0x7FFFFFFF; s_base = 0.0; }
    __syncthreads();
    if (k > 0) {
        double total = 0.0;
        for (int b0 = 0; b0 < nblk; b0 += 256) {
            const double incl = scan256(b0 + tid < nblk ? bsum[(size_t)h * nblk + b0 + tid] : 0.0);
            total += s_scan[255];
            (void)incl;
            __syncthreads();
        }
        const double target = uk * total;
        if (total > 0.0) {
            double base = 0.0;                  // running sum before the current chunk of 256 blocks
            for (int b0 = 0; b0 < nblk; b0 += 256) {
                const double v = b0 + tid < nblk ? bsum[(size_t)h * nblk + b0 + tid] : 0.0;
                const double incl = base + scan256(v);
                if (b0 + tid < nblk && incl > target) atomicMin(&s_blk, b0 + tid);
                __syncthreads();
                if (s_blk != 0x7FFFFFFF) {
                    if (tid == s_blk - b0) s_base = incl - v;      // running sum before the crossing block
                    __syncthreads();
                    break;
                }
                base += s_scan[255];
                __syncthreads();
            }
            // inside the block: one token per thread
            for (int blk = s_blk; blk < nblk; ++blk) {
                const int n = blk * KPP_BLOCK + tid;
                const double v = (n < N) ? dh[n] : 0.0;
                const double incl = s_base + scan256(v);
                __shared__ int s_tok;
                if (tid == 0) s_tok = 0x7FFFFFFF;
                __syncthreads();
                if (n < N && incl > target) atomicMin(&s_tok, n);
                __syncthreads();
                if (s_tok != 0x7FFFFFFF) {
                    if (tid == 0) s_pick = s_tok;
                    __syncthreads();
                    break;
                }
                __syncthreads();
                if (tid == 255) s_base = incl;  // rounding pushed the crossing into the next block
                __syncthreads();
            }
            if (tid == 0 && s_pick < 0) {       // rounding left the running sum at the threshold
                for (int n = N - 1; n >= 0; --n)
                    if (dh[n] > 0.0) { s_pick = n; break; }
            }
        }
    }
    __syncthreads();
    if (tid == 0) {
        int pick = s_pick;
        if (pick < 0) pick = (int)floor(uk * (double)N);
        pick = max(0, min(N - 1, pick));
        s_pick = pick;
        picked[(size_t)h * C + k] = pick;
    }
    __syncthreads();
    const int pick = s_pick;
    for (int j = tid; j < d; j += 256)
        centroids[((size_t)h * C + k) * d + j] = Elem<T>::load(X + ((size_t)h * N + pick) * d + j);
}

// `per` (4 or 8) consecutive elements as doubles, with 8- or 16-byte loads
__device__ __forceinline__ void load_elems(const bf16_t *p, int per, double *out)
{
    if (per == 8) {
        const uint4 v = *reinterpret_cast<const uint4 *>(p);
        const unsigned w[4] = {v.x, v.y, v.z, v.w};
        for (int q = 0; q < 4; ++q) {
            out[2 * q] = (double)__uint_as_float(w[q] << 16);
            out[2 * q + 1] = (double)__uint_as_float(w[q] & 0xFFFF0000u);
        }
    } else {
        const uint2 v = *reinterpret_cast<const uint2 *>(p);
        const unsigned w[2] = {v.x, v.y};
        for (int q = 0; q < 2; ++q) {
            out[2 * q] = (double)__uint_as_float(w[q] << 16);
            out[2 * q + 1] = (double)__uint_as_float(w[q] & 0xFFFF0000u);
        }
    }
}
__device__ __forceinline__ void load_elems(const float *p, int per, double *out)
{
    for (int q = 0; q < per; q += 4) {
        const float4 v = *reinterpret_cast<const float4 *>(p + q);
        out[q] = v.x; out[q + 1] = v.y; out[q + 2] = v.z; out[q + 3] = v.w;
    }
}

// D2[n] = min(D2[n], ||x_n - c||^2) against the centre drawn last, and the sum of D2 per KPP_BLOCK tokens.
// grid (nblk, H), block 256; 16 lanes share a token (d / 16 elements each), 16 tokens per pass, 4 passes in flight.
template <typename T>
__global__ __launch_bounds__(256) void kpp_update_kernel(const T *__restrict__ X,
                                                         const int32_t *__restrict__ picked, int N, int d, int C,
                                                         int k, int nblk, double *__restrict__ d2,
                                                         double *__restrict__ bsum)
{
    __shared__ double s_red[256];
    const int h = blockIdx.y, tid = threadIdx.x;
    const int sub = tid >> 4, part = tid & 15;
    const int per = d / 16;                    // 4 or 8 elements per lane
    const T *Xh = X + (size_t)h * N * d;
    const T *c = Xh + (size_t)picked[(size_t)h * C + k] * d + part * per;
    double cv[8], xv[8];
    load_elems(c, per, cv);
    double acc = 0.0;
    for (int r = 0; r < KPP_BLOCK; r += 64) {
        double a[4], old[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int n = blockIdx.x * KPP_BLOCK + r + 16 * q + sub;
            a[q] = 0.0;
            old[q] = INFINITY;
            if (n < N) {
                load_elems(Xh + (size_t)n * d + part * per, per, xv);
                for (int j = 0; j < per; ++j) {
                    const double t = xv[j] - cv[j];
                    a[q] += t * t;
                }
                if (k > 0 && part == 0) old[q] = d2[(size_t)h * N + n];
            }
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            for (int o = 1; o < 16; o <<= 1) a[q] += __shfl_xor(a[q], o);
            const int n = blockIdx.x * KPP_BLOCK + r + 16 * q + sub;
            if (n < N && part == 0) {
                const double nv = a[q] < old[q] ? a[q] : old[q];
                d2[(size_t)h * N + n] = nv;
                acc += nv;
            }
        }
    }
    s_red[tid] = acc;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
        if (tid < o) s_red[tid] += s_red[tid + o];
        __syncthreads();
    }
    if (tid == 0) bsum[(size_t)h * nblk + blockIdx.x] = s_red[0];
}

struct KppWs {
    double *d2, *bsum;
    int32_t *picked;
    size_t total;
};

static KppWs kpp_carve(void *ws, int H, int N, int C)
{
    KppWs k;
    Carver c(ws);
    k.d2 = c.take<double>((size_t)H * N);
    k.bsum = c.take<double>((size_t)H * cdiv(N, KPP_BLOCK));
    k.picked = c.take<int32_t>((size_t)H * C);
    k.total = c.used;
    return k;
}

size_t kpp_ws_bytes(int H, int N, int C) { return kpp_carve(nullptr, H, N, C).total; }

template <typename T>
static int kpp_run(const T *X, int H, int N, int d, int C, const double *u, float *centroids, int32_t *picked,
                   void *ws, hipStream_t st)
{
    const KppWs w = kpp_carve(ws, H, N, C);
    int32_t *pk = picked ? picked : w.picked;
    const int nblk = cdiv(N, KPP_BLOCK);
    for (int k = 0; k < C; ++k) {
        hipLaunchKernelGGL(kpp_pick_kernel<T>, dim3(H), dim3(256), 0, st, X, u, w.d2, w.bsum, N, d, C, k, nblk, pk,
                           centroids);
        if (k + 1 < C)
            hipLaunchKernelGGL(kpp_update_kernel<T>, dim3(nblk, H), dim3(256), 0, st, X, pk, N, d, C, k, nblk, w.d2,
                               w.bsum);
    }
    SVG2_HIP_CHECK(hipGetLastError());
    return SVG2_OK;
}

int kpp_launch(const void *X, int dtype, int H, int N, int d, int C, const double *u, float *centroids,
               int32_t *picked, void *ws, hipStream_t st)
{
    if (dtype == SVG2_BF16)
        return kpp_run<bf16_t>(static_cast<const bf16_t *>(X), H, N, d, C, u, centroids, picked, ws, st);
    return kpp_run<float>(static_cast<const float *>(X), H, N, d, C, u, centroids, picked, ws, st);
}

}  // namespace svg2
