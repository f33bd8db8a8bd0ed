// Centroid-based top-p selection (paper Section 4.2).
//
//   select_row_kernel      one workgroup per (head, query cluster i):
//       S_ij  = cq_i . ck_j / sqrt(d)                                  (Eq. 1)
//       P'_ij = |K_j| exp(S_ij) / sum_k |K_k| exp(S_ik)                (Eq. 2)
//       sort j by (P' descending, j ascending), exclusive prefix sum of P',
//       keep sorted position t iff the mass before it is < top_p, write the
//       kept j in ascending order to a per-row list.
//   select_compact_kernel  one workgroup per head: row lengths -> CSR row_ptr,
//       lists -> col_idx, density (Section 5.1).
//
// The row maximum of S is subtracted before exp; it cancels in Eq. 2.
#include "svg2_common.h"

namespace svg2 {

static constexpr int SEL_THREADS = 256;

__device__ __forceinline__ float block_reduce_max(float v, float *s_red)
{
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    const int w = threadIdx.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) s_red[w] = v;
    __syncthreads();
    float r = s_red[0];
    for (int i = 1; i < SEL_THREADS / 64; ++i) r = fmaxf(r, s_red[i]);
    return r;
}

__device__ __forceinline__ float block_reduce_sum(float v, float *s_red)
{
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    const int w = threadIdx.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) s_red[w] = v;
    __syncthreads();
    float r = s_red[0];
    for (int i = 1; i < SEL_THREADS / 64; ++i) r += s_red[i];
    return r;
}

__device__ __forceinline__ double block_reduce_sum_f64(double v, double *s_red)
{
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    const int w = threadIdx.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) s_red[w] = v;
    __syncthreads();
    double r = s_red[0];
    for (int i = 1; i < SEL_THREADS / 64; ++i) r += s_red[i];
    return r;
}

// Exclusive prefix sums of per-thread values over the workgroup (thread order).
template <typename T> __device__ __forceinline__ T block_exclusive_scan(T v, T *s_scan, T *total)
{
    __syncthreads();
    s_scan[threadIdx.x] = v;
    __syncthreads();
    for (int o = 1; o < SEL_THREADS; o <<= 1) {
        T add = (threadIdx.x >= (unsigned)o) ? s_scan[threadIdx.x - o] : T(0);
        __syncthreads();
        s_scan[threadIdx.x] += add;
        __syncthreads();
    }
    T incl = s_scan[threadIdx.x];
    *total = s_scan[SEL_THREADS - 1];
    return incl - v;
}

// Dynamic LDS layout: u64 key[npow2] | float P[npow2] | float cq[d] | int flag[Ck]
__global__ __launch_bounds__(SEL_THREADS) void select_row_kernel(
    const float *__restrict__ cq, const float *__restrict__ ck, const int32_t *__restrict__ counts_q,
    const int32_t *__restrict__ counts_k, int Cq, int Ck, int d, int npow2, float top_p,
    float *__restrict__ p_est, int32_t *__restrict__ lists, int32_t *__restrict__ row_len,
    int32_t *__restrict__ row_keys)
{
    extern __shared__ __align__(16) unsigned char s_raw[];
    unsigned long long *s_key = reinterpret_cast<unsigned long long *>(s_raw);
    float *s_P = reinterpret_cast<float *>(s_key + npow2);
    float *s_cq = s_P + npow2;
    int32_t *s_flag = reinterpret_cast<int32_t *>(s_cq + d);
    __shared__ float s_red[SEL_THREADS / 64];
    __shared__ float s_scan_f[SEL_THREADS];
    __shared__ int32_t s_scan_i[SEL_THREADS];

    const int i = blockIdx.x, h = blockIdx.y, tid = threadIdx.x;
    const float *cqi = cq + ((size_t)h * Cq + i) * d;
    const float *ckh = ck + (size_t)h * Ck * d;
    const int32_t *cnt = counts_k + (size_t)h * Ck;
    for (int k = tid; k < d; k += SEL_THREADS) s_cq[k] = cqi[k];
    __syncthreads();

    // Eq. 1
    const float inv_sqrt_d = 1.0f / sqrtf((float)d);
    float mx = -INFINITY;
    for (int j = tid; j < Ck; j += SEL_THREADS) {
        const float4 *row = reinterpret_cast<const float4 *>(ckh + (size_t)j * d);
        float acc = 0.f;
        for (int k = 0; k < d / 4; ++k) {
            const float4 v = row[k];
            acc = fmaf(s_cq[4 * k + 0], v.x, acc);
            acc = fmaf(s_cq[4 * k + 1], v.y, acc);
            acc = fmaf(s_cq[4 * k + 2], v.z, acc);
            acc = fmaf(s_cq[4 * k + 3], v.w, acc);
        }
        const float s = acc * inv_sqrt_d;
        s_P[j] = s;
        if (cnt[j] > 0) mx = fmaxf(mx, s);
    }
    mx = block_reduce_max(mx, s_red);
    // Eq. 2
    float part = 0.f;
    for (int j = tid; j < Ck; j += SEL_THREADS) {
        const int c = cnt[j];
        const float w = (c > 0) ? (float)c * expf(s_P[j] - mx) : 0.f;
        s_P[j] = w;
        part += w;
    }
    const float den = block_reduce_sum(part, s_red);
    const float inv_den = den > 0.f ? 1.0f / den : 0.f;
    for (int j = tid; j < Ck; j += SEL_THREADS) {
        const float p = s_P[j] * inv_den;
        s_P[j] = p;
        if (p_est) p_est[((size_t)h * Cq + i) * Ck + j] = p;
    }
    __syncthreads();

    const bool empty_row = counts_q && counts_q[(size_t)h * Cq + i] == 0;
    if (empty_row) {
        for (int j = tid; j < Ck; j += SEL_THREADS) s_flag[j] = 0;
    } else if (top_p >= 1.0f) {
        for (int j = tid; j < Ck; j += SEL_THREADS) s_flag[j] = cnt[j] > 0;
    } else {
        // sort keys: larger P' first, then smaller j.  P' >= 0, so its bit
        // pattern orders like the value.
        for (int j = tid; j < npow2; j += SEL_THREADS) {
            unsigned long long key = ~0ull;
            if (j < Ck) key = ((unsigned long long)(0xFFFFFFFFu - __float_as_uint(s_P[j])) << 32) | (unsigned)j;
            s_key[j] = key;
        }
        __syncthreads();
        for (int k = 2; k <= npow2; k <<= 1) {
            for (int jj = k >> 1; jj > 0; jj >>= 1) {
                for (int t = tid; t < npow2; t += SEL_THREADS) {
                    const int partner = t ^ jj;
                    if (partner > t) {
                        const unsigned long long a = s_key[t], b = s_key[partner];
                        const bool up = (t & k) == 0;
                        if ((a > b) == up) { s_key[t] = b; s_key[partner] = a; }
                    }
                }
                __syncthreads();
            }
        }
        // exclusive prefix sum of P' in sorted order; thread t owns a contiguous slice
        const int per = (Ck + SEL_THREADS - 1) / SEL_THREADS;
        const int t0 = min(Ck, tid * per), t1 = min(Ck, t0 + per);
        float sum = 0.f;
        for (int t = t0; t < t1; ++t) sum += s_P[(int)(s_key[t] & 0xFFFFFFFFu)];
        float total;
        float run = block_exclusive_scan<float>(sum, s_scan_f, &total);
        for (int j = tid; j < Ck; j += SEL_THREADS) s_flag[j] = 0;
        __syncthreads();
        for (int t = t0; t < t1; ++t) {
            const int j = (int)(s_key[t] & 0xFFFFFFFFu);
            if (run < top_p && cnt[j] > 0) s_flag[j] = 1;
            run += s_P[j];
        }
    }
    __syncthreads();

    // kept clusters in ascending j
    const int per = (Ck + SEL_THREADS - 1) / SEL_THREADS;
    const int j0 = min(Ck, tid * per), j1 = min(Ck, j0 + per);
    int nk = 0, keys = 0;
    for (int j = j0; j < j1; ++j)
        if (s_flag[j]) { nk += 1; keys += cnt[j]; }
    int total_n;
    int pos = block_exclusive_scan<int32_t>(nk, s_scan_i, &total_n);
    int32_t *list = lists + ((size_t)h * Cq + i) * Ck;
    for (int j = j0; j < j1; ++j)
        if (s_flag[j]) list[pos++] = j;
    int total_keys;
    (void)block_exclusive_scan<int32_t>(keys, s_scan_i, &total_keys);
    if (tid == 0) {
        row_len[(size_t)h * Cq + i] = total_n;
        row_keys[(size_t)h * Cq + i] = total_keys;
    }
}

__global__ __launch_bounds__(SEL_THREADS) void select_compact_kernel(
    const int32_t *__restrict__ lists, const int32_t *__restrict__ row_len, const int32_t *__restrict__ row_keys,
    const int32_t *__restrict__ counts_q, const int32_t *__restrict__ counts_k, int Cq, int Ck,
    int32_t *__restrict__ row_ptr, int32_t *__restrict__ col_idx, float *__restrict__ density)
{
    extern __shared__ int32_t s_ptr[];                 // [Cq + 1]
    __shared__ int32_t s_scan_i[SEL_THREADS];
    __shared__ double s_red[SEL_THREADS / 64];
    const int h = blockIdx.x, tid = threadIdx.x;
    const int32_t *len = row_len + (size_t)h * Cq;
    const int per = (Cq + SEL_THREADS - 1) / SEL_THREADS;
    const int i0 = min(Cq, tid * per), i1 = min(Cq, i0 + per);
    int sum = 0;
    for (int i = i0; i < i1; ++i) sum += len[i];
    int total;
    int run = block_exclusive_scan<int32_t>(sum, s_scan_i, &total);
    for (int i = i0; i < i1; ++i) { s_ptr[i] = run; run += len[i]; }
    if (tid == 0) s_ptr[Cq] = total;
    __syncthreads();
    int32_t *rp = row_ptr + (size_t)h * (Cq + 1);
    for (int i = tid; i <= Cq; i += SEL_THREADS) rp[i] = s_ptr[i];
    int32_t *ci = col_idx + (size_t)h * Cq * Ck;
    for (int i = 0; i < Cq; ++i) {
        const int32_t *list = lists + ((size_t)h * Cq + i) * Ck;
        const int n = s_ptr[i + 1] - s_ptr[i];
        for (int e = tid; e < n; e += SEL_THREADS) ci[s_ptr[i] + e] = list[e];
    }
    if (density) {
        // work = sum_i |Q_i| * (keys selected for i): integers below 2^53, exact in double
        double w = 0.0, nq = 0.0, nk = 0.0;
        for (int i = tid; i < Cq; i += SEL_THREADS) {
            const int c = counts_q[(size_t)h * Cq + i];
            w += (double)c * (double)row_keys[(size_t)h * Cq + i];
            nq += (double)c;
        }
        for (int j = tid; j < Ck; j += SEL_THREADS) nk += (double)counts_k[(size_t)h * Ck + j];
        w = block_reduce_sum_f64(w, s_red);
        nq = block_reduce_sum_f64(nq, s_red);
        nk = block_reduce_sum_f64(nk, s_red);
        if (tid == 0) density[h] = (nq > 0.0 && nk > 0.0) ? (float)(w / (nq * nk)) : 0.f;
    }
}

static int next_pow2(int x)
{
    int p = 1;
    while (p < x) p <<= 1;
    return p;
}

size_t select_ws_bytes(int H, int Cq, int Ck)
{
    Carver c(nullptr);
    c.take<int32_t>((size_t)H * Cq * Ck);   // per-row lists
    c.take<int32_t>((size_t)H * Cq);        // row lengths
    c.take<int32_t>((size_t)H * Cq);        // keys selected per row
    return c.used;
}

static size_t select_lds_bytes(int Ck, int d)
{
    return (size_t)next_pow2(Ck) * (sizeof(unsigned long long) + sizeof(float)) + (size_t)d * sizeof(float) +
           (size_t)Ck * sizeof(int32_t);
}

int select_prepare() { return set_dynamic_lds(reinterpret_cast<const void *>(select_row_kernel), select_lds_bytes(SVG2_MAX_CLUSTERS, 128)); }

int select_launch(const float *cq, const float *ck, const int32_t *counts_q, const int32_t *counts_k,
                  int H, int Cq, int Ck, int d, float top_p, int32_t *row_ptr, int32_t *col_idx,
                  float *p_est, float *density, void *ws, hipStream_t st)
{
    Carver c(ws);
    int32_t *lists = c.take<int32_t>((size_t)H * Cq * Ck);
    int32_t *row_len = c.take<int32_t>((size_t)H * Cq);
    int32_t *row_keys = c.take<int32_t>((size_t)H * Cq);
    const int np2 = next_pow2(Ck);
    const size_t lds = select_lds_bytes(Ck, d);
    hipLaunchKernelGGL(select_row_kernel, dim3(Cq, H), dim3(SEL_THREADS), lds, st, cq, ck, counts_q, counts_k, Cq, Ck,
                       d, np2, top_p, p_est, lists, row_len, row_keys);
    hipLaunchKernelGGL(select_compact_kernel, dim3(H), dim3(SEL_THREADS), (size_t)(Cq + 1) * sizeof(int32_t), st,
                       lists, row_len, row_keys, counts_q, counts_k, Cq, Ck, row_ptr, col_idx, density);
    SVG2_HIP_CHECK(hipGetLastError());
    return SVG2_OK;
}

}  // namespace svg2
