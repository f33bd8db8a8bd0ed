// Per-head Lloyd k-means (paper Section 4.1), batched over heads.
//
// One iteration = assign, update, finalize:
//   assign    token x centroid contraction with a fused argmin.
//             bf16 input: MFMA 32x32x16 bf16 with the centroid tile as the A
//             operand (rows) and the tokens as the B operand (columns), so a
//             lane's 16 accumulators are 16 centroids of ONE token and the
//             running argmin stays in registers.  dist = ||c||^2 - 2 x.c.
//             fp32 input: a plain FMA kernel (one token per thread).
//   update    LDS-privatised segmented sum: a workgroup owns a token range and
//             a slice of the d columns, accumulates sum[label][col] in LDS
//             with ds_add_f32, then writes its partial sums (no global
//             atomics; the partials are reduced in a fixed order).
//   finalize  mean = sum / count (an empty cluster keeps its centroid), the
//             bf16 copy of the centroids the next assign reads, and ||c||^2.
//
// For bf16 input the assign step sees the centroids rounded to bf16 (both in
// x.c and in ||c||^2); the centroids handed back stay fp32 means.
#include "svg2_common.h"

namespace svg2 {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

static constexpr int KM_CT = 128;      // centroids staged in LDS per step (bf16 kernel)
static constexpr int KM_TB = 4;        // 32-token blocks per wavefront (bf16 kernel)
static constexpr int KM_WG_TOKENS = 4 * KM_TB * 32;

// ---------------------------------------------------------------- finalize
// grid (C, H), block d.  do_update = 0: centroids <- init (first call).
template <bool BF16>
__global__ void kmeans_finalize_kernel(const float *__restrict__ init, float *__restrict__ centroids,
                                       const float *__restrict__ psum, const int32_t *__restrict__ pcnt,
                                       int nchunks, int C, int d, bf16_t *__restrict__ cb, float *__restrict__ cn,
                                       int32_t *__restrict__ counts_out, int do_update)
{
    __shared__ float s_red[2];
    const int j = blockIdx.x, h = blockIdx.y, k = threadIdx.x;
    const size_t idx = ((size_t)h * C + j) * d + k;
    float c;
    if (do_update) {
        int cnt = 0;
        for (int q = 0; q < nchunks; ++q) cnt += pcnt[((size_t)h * nchunks + q) * C + j];
        if (cnt > 0) {
            float s = 0.f;
            for (int q = 0; q < nchunks; ++q) s += psum[(((size_t)h * nchunks + q) * C + j) * d + k];
            c = s / (float)cnt;
        } else {
            c = centroids[idx];
        }
        if (k == 0 && counts_out) counts_out[(size_t)h * C + j] = cnt;
    } else {
        c = init[idx];
    }
    centroids[idx] = c;
    float cr = c;
    if (BF16) {
        const bf16_t b = f32_to_bf16(c);
        cb[idx] = b;
        cr = bf16_to_f32(b);
    }
    float sq = cr * cr;
    for (int o = 32; o > 0; o >>= 1) sq += __shfl_xor(sq, o);
    if ((k & 63) == 0) s_red[k >> 6] = sq;
    __syncthreads();
    if (k == 0) cn[(size_t)h * C + j] = (d > 64) ? s_red[0] + s_red[1] : s_red[0];
}

// ---------------------------------------------------------------- assign, bf16 MFMA
template <int D, bool OBJ>
__global__ __launch_bounds__(256) void kmeans_assign_bf16_kernel(const bf16_t *__restrict__ X,
                                                                 const bf16_t *__restrict__ cb,
                                                                 const float *__restrict__ cn, int N, int C,
                                                                 int32_t *__restrict__ labels,
                                                                 float *__restrict__ objective, int obj_stride)
{
    constexpr int KS = D / 16;              // MFMA k-steps
    constexpr int ROW = D + 8;              // LDS row stride in elements (16 bytes of padding)
    __shared__ __align__(16) bf16_t s_c[KM_CT * ROW];
    __shared__ float s_cn[KM_CT];

    const int h = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, col = lane & 31;
    const bf16_t *Xh = X + (size_t)h * N * D;
    const bf16_t *cbh = cb + (size_t)h * C * D;
    const float *cnh = cn + (size_t)h * C;
    const int tok0 = blockIdx.x * KM_WG_TOKENS + wave * (KM_TB * 32);

    // tokens as the B operand: lane (col, half) holds elements 16 s + 8 half .. + 8 of token `col`
    bf16x8 xb[KM_TB][KS];
    float xx[KM_TB];
#pragma unroll
    for (int tb = 0; tb < KM_TB; ++tb) {
        const int n = min(N - 1, tok0 + tb * 32 + col);
        const uint4 *src = reinterpret_cast<const uint4 *>(Xh + (size_t)n * D + 8 * half);
        xx[tb] = 0.f;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            const uint4 v = src[2 * s];
            __builtin_memcpy(&xb[tb][s], &v, 16);
            if (OBJ) {
                const unsigned w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float lo = __uint_as_float(w[q] << 16), hi = __uint_as_float(w[q] & 0xFFFF0000u);
                    xx[tb] = fmaf(lo, lo, xx[tb]);
                    xx[tb] = fmaf(hi, hi, xx[tb]);
                }
            }
        }
    }

    float best[KM_TB];
    int bidx[KM_TB];
#pragma unroll
    for (int tb = 0; tb < KM_TB; ++tb) { best[tb] = INFINITY; bidx[tb] = 0; }

    for (int c0 = 0; c0 < C; c0 += KM_CT) {
        __syncthreads();
        // stage KM_CT centroids (rows past C are zero with an infinite norm)
        for (int e = tid; e < KM_CT * (D / 8); e += 256) {
            const int r = e / (D / 8), part = e % (D / 8);
            uint4 v = make_uint4(0, 0, 0, 0);
            if (c0 + r < C) v = reinterpret_cast<const uint4 *>(cbh + (size_t)(c0 + r) * D)[part];
            *reinterpret_cast<uint4 *>(&s_c[r * ROW + part * 8]) = v;
        }
        if (tid < KM_CT) s_cn[tid] = (c0 + tid < C) ? cnh[c0 + tid] : INFINITY;
        __syncthreads();
        const int nrb = min(KM_CT / 32, (C - c0 + 31) / 32);
        for (int rb = 0; rb < nrb; ++rb) {
            f32x16 acc[KM_TB];
#pragma unroll
            for (int tb = 0; tb < KM_TB; ++tb)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[tb][i] = 0.f;
            const bf16_t *arow = &s_c[(rb * 32 + col) * ROW + 8 * half];
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                bf16x8 a;
                const uint4 v = *reinterpret_cast<const uint4 *>(arow + 16 * s);
                __builtin_memcpy(&a, &v, 16);
#pragma unroll
                for (int tb = 0; tb < KM_TB; ++tb)
                    acc[tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, xb[tb][s], acc[tb], 0, 0, 0);
            }
            // accumulator i of a lane is centroid rb*32 + 8 (i/4) + 4 half + i%4: ascending in i
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int r = rb * 32 + 8 * (i >> 2) + 4 * half + (i & 3);
                const float cnv = s_cn[r];
#pragma unroll
                for (int tb = 0; tb < KM_TB; ++tb) {
                    const float dist = fmaf(-2.f, acc[tb][i], cnv);
                    if (dist < best[tb]) { best[tb] = dist; bidx[tb] = c0 + r; }
                }
            }
        }
    }

    float obj = 0.f;
#pragma unroll
    for (int tb = 0; tb < KM_TB; ++tb) {
        const float ob = __shfl_xor(best[tb], 32);
        const int oi = __shfl_xor(bidx[tb], 32);
        if (ob < best[tb] || (ob == best[tb] && oi < bidx[tb])) { best[tb] = ob; bidx[tb] = oi; }
        const int n = tok0 + tb * 32 + col;
        if (half == 0 && n < N) labels[(size_t)h * N + n] = bidx[tb];
        if (OBJ) {
            const float x2 = xx[tb] + __shfl_xor(xx[tb], 32);
            if (half == 0 && n < N) obj += x2 + best[tb];
        }
    }
    if (OBJ) {
        for (int o = 32; o > 0; o >>= 1) obj += __shfl_xor(obj, o);
        if (lane == 0) atomicAdd(objective + (size_t)h * obj_stride, obj);
    }
}

// ---------------------------------------------------------------- assign, fp32 FMA
template <int D, bool OBJ>
__global__ __launch_bounds__(128) void kmeans_assign_f32_kernel(const float *__restrict__ X,
                                                                const float *__restrict__ cent,
                                                                const float *__restrict__ cn, int N, int C,
                                                                int32_t *__restrict__ labels,
                                                                float *__restrict__ objective, int obj_stride)
{
    constexpr int CT = 32;
    __shared__ __align__(16) float s_c[CT * D];
    __shared__ float s_cn[CT];
    const int h = blockIdx.y, tid = threadIdx.x;
    const int n = blockIdx.x * 128 + tid;
    const float *xr = X + ((size_t)h * N + min(n, N - 1)) * D;
    float x[D];
#pragma unroll
    for (int k = 0; k < D / 4; ++k) {
        const float4 v = reinterpret_cast<const float4 *>(xr)[k];
        x[4 * k] = v.x; x[4 * k + 1] = v.y; x[4 * k + 2] = v.z; x[4 * k + 3] = v.w;
    }
    float best = INFINITY;
    int bidx = 0;
    for (int c0 = 0; c0 < C; c0 += CT) {
        __syncthreads();
        for (int e = tid; e < CT * D; e += 128) {
            const int r = e / D;
            s_c[e] = (c0 + r < C) ? cent[((size_t)h * C + c0 + r) * D + (e % D)] : 0.f;
        }
        if (tid < CT) s_cn[tid] = (c0 + tid < C) ? cn[(size_t)h * C + c0 + tid] : INFINITY;
        __syncthreads();
        const int nr = min(CT, C - c0);
        for (int r = 0; r < nr; ++r) {
            float dot = 0.f;
#pragma unroll
            for (int k = 0; k < D; ++k) dot = fmaf(x[k], s_c[r * D + k], dot);
            const float dist = fmaf(-2.f, dot, s_cn[r]);
            if (dist < best) { best = dist; bidx = c0 + r; }
        }
    }
    if (n < N) labels[(size_t)h * N + n] = bidx;
    if (OBJ) {
        float v = 0.f;
        if (n < N) {
            float x2 = 0.f;
#pragma unroll
            for (int k = 0; k < D; ++k) x2 = fmaf(x[k], x[k], x2);
            v = x2 + best;
        }
        for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
        if ((tid & 63) == 0) atomicAdd(objective + (size_t)h * obj_stride, v);
    }
}

// ---------------------------------------------------------------- update
// grid (nchunks, D / DS, H), block 256.  A lane owns 4 consecutive columns of
// a token; DS / 4 lanes cover the slice; 256 / (DS / 4) tokens are in flight,
// each group of lanes walking its own contiguous sub-range of the chunk so
// that simultaneously processed tokens are far apart (neighbouring video
// tokens tend to share a label, which would serialise the LDS atomics).
template <typename T, int D>
__global__ __launch_bounds__(256) void kmeans_update_kernel(const T *__restrict__ X,
                                                            const int32_t *__restrict__ labels, int N, int C, int DS,
                                                            int chunk_tokens, int nchunks,
                                                            float *__restrict__ psum, int32_t *__restrict__ pcnt)
{
    extern __shared__ __align__(16) float s_sum[];                 // [C * DS], then int counts [C]
    int32_t *s_cnt = reinterpret_cast<int32_t *>(s_sum + (size_t)C * DS);
    const int chunk = blockIdx.x, slice = blockIdx.y, h = blockIdx.z, tid = threadIdx.x;
    for (int e = tid; e < C * DS; e += 256) s_sum[e] = 0.f;
    for (int e = tid; e < C; e += 256) s_cnt[e] = 0;
    __syncthreads();
    const int lpt = DS / 4;                       // lanes per token
    const int groups = 256 / lpt;                 // tokens in flight
    const int g = tid / lpt, part = tid % lpt;
    const int n0 = chunk * chunk_tokens, n1 = min(N, n0 + chunk_tokens);
    const int per = (n1 - n0 + groups - 1) / groups;
    const int a = min(n1, n0 + g * per), b = min(n1, a + per);
    const int col0 = slice * DS + part * 4;
    const T *Xh = X + (size_t)h * N * D;
    const int32_t *lab = labels + (size_t)h * N;
    for (int n = a; n < b; ++n) {
        const int l = lab[n];
        const T *p = Xh + (size_t)n * D + col0;
        float v0, v1, v2, v3;
        if (sizeof(T) == 2) {
            const uint2 w = *reinterpret_cast<const uint2 *>(p);
            v0 = __uint_as_float(w.x << 16); v1 = __uint_as_float(w.x & 0xFFFF0000u);
            v2 = __uint_as_float(w.y << 16); v3 = __uint_as_float(w.y & 0xFFFF0000u);
        } else {
            const float4 w = *reinterpret_cast<const float4 *>(p);
            v0 = w.x; v1 = w.y; v2 = w.z; v3 = w.w;
        }
        float *dst = s_sum + (size_t)l * DS + part * 4;
        atomicAdd(dst + 0, v0);
        atomicAdd(dst + 1, v1);
        atomicAdd(dst + 2, v2);
        atomicAdd(dst + 3, v3);
        if (slice == 0 && part == 0) atomicAdd(&s_cnt[l], 1);
    }
    __syncthreads();
    float *out = psum + ((size_t)h * nchunks + chunk) * C * D;
    for (int e = tid; e < C * DS; e += 256) {
        const int c = e / DS, k = e % DS;
        out[(size_t)c * D + slice * DS + k] = s_sum[e];
    }
    if (slice == 0) {
        int32_t *oc = pcnt + ((size_t)h * nchunks + chunk) * C;
        for (int e = tid; e < C; e += 256) oc[e] = s_cnt[e];
    }
}

__global__ void kmeans_zero_kernel(float *p, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0.f;
}

// ---------------------------------------------------------------- host side
struct KmeansPlan {
    int DS, nslices, nchunks, chunk_tokens;
};

static KmeansPlan kmeans_plan(int H, int N, int d, int C)
{
    KmeansPlan p;
    p.DS = 32;
    while (p.DS > 4 && (size_t)C * p.DS * sizeof(float) > 64 * 1024) p.DS >>= 1;
    p.nslices = d / p.DS;
    int want = cdiv(1024, H * p.nslices);
    int maxc = cdiv(N, 1024);
    p.nchunks = want < 1 ? 1 : (want > maxc ? maxc : want);
    p.chunk_tokens = cdiv(N, p.nchunks);
    p.nchunks = cdiv(N, p.chunk_tokens);
    return p;
}

size_t kmeans_ws_bytes(int dtype, int H, int N, int d, int C)
{
    (void)dtype;
    const KmeansPlan p = kmeans_plan(H, N, d, C);
    Carver c(nullptr);
    c.take<bf16_t>((size_t)H * C * d);                       // bf16 centroids
    c.take<float>((size_t)H * C);                            // ||c||^2
    c.take<float>((size_t)H * p.nchunks * C * d);            // partial sums
    c.take<int32_t>((size_t)H * p.nchunks * C);              // partial counts
    return c.used;
}

template <typename T, int D, bool BF16>
static int kmeans_run(const T *X, int H, int N, int C, int iters, const float *init, float *centroids,
                       int32_t *labels, int32_t *counts, float *objective, void *ws, hipStream_t st)
{
    const KmeansPlan p = kmeans_plan(H, N, D, C);
    Carver c(ws);
    bf16_t *cb = c.take<bf16_t>((size_t)H * C * D);
    float *cn = c.take<float>((size_t)H * C);
    float *psum = c.take<float>((size_t)H * p.nchunks * C * D);
    int32_t *pcnt = c.take<int32_t>((size_t)H * p.nchunks * C);

    if (objective)
        hipLaunchKernelGGL(kmeans_zero_kernel, dim3(cdiv(H * iters, 256)), dim3(256), 0, st, objective, H * iters);
    hipLaunchKernelGGL((kmeans_finalize_kernel<BF16>), dim3(C, H), dim3(D), 0, st, init, centroids, psum, pcnt,
                       p.nchunks, C, D, cb, cn, (int32_t *)nullptr, 0);
    const size_t upd_lds = (size_t)C * p.DS * sizeof(float) + (size_t)C * sizeof(int32_t);
    SVG2_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void *>(kmeans_update_kernel<T, D>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)upd_lds));
    for (int t = 0; t < iters; ++t) {
        float *obj = objective ? objective + t : nullptr;
        if (BF16) {
            const dim3 grid(cdiv(N, KM_WG_TOKENS), H);
            const bf16_t *Xb = reinterpret_cast<const bf16_t *>(X);
            if (obj)
                hipLaunchKernelGGL((kmeans_assign_bf16_kernel<D, true>), grid, dim3(256), 0, st, Xb, cb, cn, N, C,
                                   labels, obj, iters);
            else
                hipLaunchKernelGGL((kmeans_assign_bf16_kernel<D, false>), grid, dim3(256), 0, st, Xb, cb, cn, N, C,
                                   labels, obj, iters);
        } else {
            const dim3 grid(cdiv(N, 128), H);
            const float *Xf = reinterpret_cast<const float *>(X);
            if (obj)
                hipLaunchKernelGGL((kmeans_assign_f32_kernel<D, true>), grid, dim3(128), 0, st, Xf, centroids, cn, N,
                                   C, labels, obj, iters);
            else
                hipLaunchKernelGGL((kmeans_assign_f32_kernel<D, false>), grid, dim3(128), 0, st, Xf, centroids, cn, N,
                                   C, labels, obj, iters);
        }
        hipLaunchKernelGGL((kmeans_update_kernel<T, D>), dim3(p.nchunks, p.nslices, H), dim3(256), upd_lds, st, X,
                           labels, N, C, p.DS, p.chunk_tokens, p.nchunks, psum, pcnt);
        hipLaunchKernelGGL((kmeans_finalize_kernel<BF16>), dim3(C, H), dim3(D), 0, st, (const float *)nullptr,
                           centroids, psum, pcnt, p.nchunks, C, D, cb, cn, counts, 1);
    }
    return SVG2_OK;
}

int kmeans_launch(const void *X, int dtype, int H, int N, int d, int C, int iters, const float *init,
                  float *centroids, int32_t *labels, int32_t *counts, float *objective, void *ws, hipStream_t st)
{
    int rc;
    if (dtype == SVG2_BF16) {
        const bf16_t *Xb = static_cast<const bf16_t *>(X);
        if (d == 128) rc = kmeans_run<bf16_t, 128, true>(Xb, H, N, C, iters, init, centroids, labels, counts, objective, ws, st);
        else rc = kmeans_run<bf16_t, 64, true>(Xb, H, N, C, iters, init, centroids, labels, counts, objective, ws, st);
    } else {
        const float *Xf = static_cast<const float *>(X);
        if (d == 128) rc = kmeans_run<float, 128, false>(Xf, H, N, C, iters, init, centroids, labels, counts, objective, ws, st);
        else rc = kmeans_run<float, 64, false>(Xf, H, N, C, iters, init, centroids, labels, counts, objective, ws, st);
    }
    if (rc != SVG2_OK) return rc;
    SVG2_HIP_CHECK(hipGetLastError());
    return SVG2_OK;
}

}  // namespace svg2
