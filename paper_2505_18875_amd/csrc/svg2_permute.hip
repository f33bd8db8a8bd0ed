// Semantic-aware permutation (paper Section 4.1) as a stable counting sort of
// token ids by cluster label, plus the row gather that applies it.
//
//   hist     per (head, chunk): histogram of labels              (LDS atomics)
//   scan     per head: totals -> offsets (exclusive scan over clusters) and
//            the first output slot of every (chunk, cluster)
//   scatter  per (head, chunk): one wavefront walks its chunk in token order,
//            ranking equal labels inside each group of 64 with ballots, so the
//            order inside a cluster stays the original token order
//   gather   dst[r,:] = src[perm[r],:], 16 bytes per lane, rows coalesced on
//            the write side
//
// Everything is integer work: results are unique and reproducible bit for bit.
#include <algorithm>
#include <mutex>

#include "svg2_common.h"

namespace svg2 {

static constexpr int PERM_CHUNK = 1024;     // tokens per chunk (one wavefront in scatter)

// Scratch of svg2_permute_noalloc: the per-(head, chunk, cluster) histogram of the counting sort lives in this
// file-scope array instead of a caller's workspace.  Every GPU the library runs on holds its own copy until the
// process ends.  In host code the name is only a handle: the device address is looked up once per device
// (hipGetSymbolAddress) and that pointer is what kernels get.
static __device__ __align__(256) unsigned char scratch[SVG2_PERMUTE_NOALLOC_SCRATCH_BYTES];

// Every kernel of the sort takes up to two independent problems ("sides": the Q tokens and the K tokens of a
// layer, which share H and N but not C) and picks its side with blockIdx.z, so that both sorts of a layer -- or of
// a k-means iteration -- cost one launch per step instead of two.
__global__ __launch_bounds__(256) void permute_hist_kernel(SortArgs a, int N, int nchunks)
{
    extern __shared__ int32_t s_hist[];
    const SortSide S = blockIdx.z ? a.s[1] : a.s[0];      // (a select of scalars, not an indexed copy)
    const int chunk = blockIdx.x, h = blockIdx.y, C = S.C;
    for (int c = threadIdx.x; c < C; c += blockDim.x) s_hist[c] = 0;
    __syncthreads();
    const int n0 = chunk * PERM_CHUNK;
    const int n1 = min(N, n0 + PERM_CHUNK);
    const int32_t *lab = S.labels + (size_t)h * N;
    for (int n = n0 + threadIdx.x; n < n1; n += blockDim.x) atomicAdd(&s_hist[lab[n]], 1);
    __syncthreads();
    int32_t *out = S.hist + ((size_t)h * nchunks + chunk) * C;
    for (int c = threadIdx.x; c < C; c += blockDim.x) out[c] = s_hist[c];
}

// One workgroup per head and side.  hist[h][k][c] becomes the first sorted row that
// chunk k writes for cluster c.  The loads of a cluster's column are issued SCAN_UB at a time before they are
// used, so the kernel waits for a few round trips to memory instead of one per chunk.
// If the side asks for it (S.pieces), the kernel also cuts every cluster into pieces of at most S.seg sorted rows
// (never crossing a cluster boundary) for the segmented sum of the k-means update step: pieces[h][first_piece[c] + t]
// = (cluster, first row, rows, 0), first_piece[h][C] = n_pieces[h] = number of pieces of the head.
static constexpr int SCAN_UB = 16;

__global__ __launch_bounds__(256) void permute_scan_kernel(SortArgs a, int N, int nchunks)
{
    extern __shared__ int32_t s_tot[];                 // [C] totals, then exclusive offsets
    __shared__ int32_t s_part[256];
    __shared__ int32_t s_wave[4];
    __shared__ int32_t s_carry;
    const SortSide S = blockIdx.z ? a.s[1] : a.s[0];      // (a select of scalars, not an indexed copy)
    const int h = blockIdx.x, tid = threadIdx.x, C = S.C;
    int32_t *hh = S.hist + (size_t)h * nchunks * C;
    for (int c = tid; c < C; c += 256) {
        int run = 0;
        for (int k0 = 0; k0 < nchunks; k0 += SCAN_UB) {
            int v[SCAN_UB];
#pragma unroll
            for (int u = 0; u < SCAN_UB; ++u) v[u] = (k0 + u < nchunks) ? hh[(size_t)(k0 + u) * C + c] : 0;
#pragma unroll
            for (int u = 0; u < SCAN_UB; ++u) run += v[u];
        }
        s_tot[c] = run;
    }
    __syncthreads();
    // exclusive scan of s_tot over c: each thread owns a contiguous slice
    const int per = (C + 255) / 256;
    const int c0 = min(C, tid * per), c1 = min(C, c0 + per);
    int sum = 0;
    for (int c = c0; c < c1; ++c) sum += s_tot[c];
    s_part[tid] = sum;
    __syncthreads();
    if (tid == 0) {
        int run = 0;
        for (int t = 0; t < 256; ++t) { int v = s_part[t]; s_part[t] = run; run += v; }
    }
    __syncthreads();
    int run = s_part[tid];
    for (int c = c0; c < c1; ++c) { int v = s_tot[c]; s_tot[c] = run; run += v; }
    __syncthreads();
    int32_t *off = S.offsets + (size_t)h * (C + 1);
    for (int c = tid; c < C; c += 256) {
        int pos = s_tot[c];
        off[c] = pos;
        for (int k0 = 0; k0 < nchunks; k0 += SCAN_UB) {
            int v[SCAN_UB];
#pragma unroll
            for (int u = 0; u < SCAN_UB; ++u) v[u] = (k0 + u < nchunks) ? hh[(size_t)(k0 + u) * C + c] : 0;
#pragma unroll
            for (int u = 0; u < SCAN_UB; ++u) {
                if (k0 + u < nchunks) hh[(size_t)(k0 + u) * C + c] = pos;
                pos += v[u];
            }
        }
    }
    if (tid == 0) off[C] = N;
    if (S.pieces == nullptr) return;

    // pieces of the segmented sum: running count over the clusters, 256 clusters per pass
    const int seg = S.seg, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) s_carry = 0;
    __syncthreads();
    for (int cb = 0; cb < C; cb += 256) {
        const int c = cb + tid;
        const int start = (c < C) ? s_tot[c] : 0;
        const int size = (c < C) ? ((c + 1 < C) ? s_tot[c + 1] : N) - start : 0;
        const int np = (size + seg - 1) / seg;
        int incl = np;
        for (int o = 1; o < 64; o <<= 1) {
            const int v = __shfl_up(incl, o);
            if (lane >= o) incl += v;
        }
        if (lane == 63) s_wave[wave] = incl;
        __syncthreads();
        int base = s_carry;
        for (int w = 0; w < wave; ++w) base += s_wave[w];
        const int first = base + incl - np;
        if (c < C) S.first_piece[(size_t)h * (C + 1) + c] = first;
        for (int t = 0; t < np; ++t)
            S.pieces[(size_t)h * S.max_pieces + first + t] = make_int4(c, start + t * seg, min(seg, size - t * seg), 0);
        __syncthreads();
        if (tid == 255) s_carry = base + incl;
        __syncthreads();
    }
    if (tid == 0) {
        S.first_piece[(size_t)h * (C + 1) + C] = s_carry;
        S.n_pieces[h] = s_carry;
    }
}

__global__ __launch_bounds__(64) void permute_scatter_kernel(SortArgs a, int N, int nchunks)
{
    extern __shared__ int32_t s_cur[];                 // [C] next free sorted row per cluster
    const SortSide S = blockIdx.z ? a.s[1] : a.s[0];      // (a select of scalars, not an indexed copy)
    const int chunk = blockIdx.x, h = blockIdx.y, lane = threadIdx.x, C = S.C, nbits = S.nbits;
    const int32_t *base = S.hist + ((size_t)h * nchunks + chunk) * C;
    for (int c = lane; c < C; c += 64) s_cur[c] = base[c];
    __syncthreads();
    const int32_t *lab = S.labels + (size_t)h * N;
    int32_t *pm = S.perm + (size_t)h * N;
    int32_t *ip = S.inv_perm ? S.inv_perm + (size_t)h * N : nullptr;
    const int n0 = chunk * PERM_CHUNK;
    const int n1 = min(N, n0 + PERM_CHUNK);
    const unsigned long long lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
    // all labels of the chunk are requested up front (one memory round trip instead of one per group of 64)
    constexpr int NG = PERM_CHUNK / 64;
    int lr[NG];
#pragma unroll
    for (int i = 0; i < NG; ++i) {
        const int n = n0 + i * 64 + lane;
        lr[i] = (n < n1) ? lab[n] : 0;
    }
#pragma unroll
    for (int i = 0; i < NG; ++i) {
        const int g = n0 + i * 64;
        if (g >= n1) break;
        const int n = g + lane;
        const bool valid = n < n1;
        const int l = lr[i];
        // lanes holding the same label as this one
        unsigned long long peers = __ballot(valid);
        for (int b = 0; b < nbits; ++b) {
            const bool bit = (l >> b) & 1;
            const unsigned long long m = __ballot(bit);
            peers &= bit ? m : ~m;
        }
        int pos = 0;
        if (valid) {
            pos = s_cur[l] + __popcll(peers & lt_mask);
            pm[pos] = n;
            if (ip) ip[n] = pos;
        }
        __syncthreads();
        // the first lane of every peer group advances that cluster's cursor
        if (valid && (peers & lt_mask) == 0) s_cur[l] += __popcll(peers);
        __syncthreads();
    }
}

// dst[h, r, :] = src[h, perm[h, r], :] for up to two tensors; a row is
// `lanes_per_row` lanes of 16 bytes.
struct GatherPtrs {
    const uint4 *src[2];
    uint4 *dst[2];
};

__global__ __launch_bounds__(256) void permute_gather_kernel(GatherPtrs p, const int32_t *__restrict__ perm, int N,
                                                             int lanes_per_row, int rows_per_block)
{
    const int h = blockIdx.y, t = blockIdx.z;
    const uint4 *src = p.src[t] + (size_t)h * N * lanes_per_row;
    uint4 *dst = p.dst[t] + (size_t)h * N * lanes_per_row;
    const int32_t *pm = perm + (size_t)h * N;
    const int r0 = blockIdx.x * rows_per_block;
    const int r1 = min(N, r0 + rows_per_block);
    const int rows_per_pass = 256 / lanes_per_row;
    const int sub = threadIdx.x / lanes_per_row, part = threadIdx.x % lanes_per_row;
    for (int r = r0 + sub; r < r1; r += rows_per_pass) {
        const int s = pm[r];
        dst[(size_t)r * lanes_per_row + part] = src[(size_t)s * lanes_per_row + part];
    }
}

size_t permute_ws_bytes(int H, int N, int C)
{
    const int nchunks = cdiv(N, PERM_CHUNK);
    return align256((size_t)H * nchunks * C * sizeof(int32_t));
}

// The counting sort of one or two sides (labels -> offsets, perm, inv_perm; pieces if asked for): three launches.
// The caller fills labels, C, hist, offsets, perm, inv_perm and the piece fields of every side; nbits is set here.
int sort_launch(SortArgs a, int nsides, int H, int N, hipStream_t st)
{
    const int nchunks = cdiv(N, PERM_CHUNK);
    int cmax = 0;
    for (int s = 0; s < nsides; ++s) {
        int nbits = 0;
        while ((1 << nbits) < a.s[s].C) ++nbits;
        a.s[s].nbits = nbits;
        cmax = std::max(cmax, a.s[s].C);
    }
    const size_t lds = (size_t)cmax * sizeof(int32_t);
    hipLaunchKernelGGL(permute_hist_kernel, dim3(nchunks, H, nsides), dim3(256), lds, st, a, N, nchunks);
    hipLaunchKernelGGL(permute_scan_kernel, dim3(H, 1, nsides), dim3(256), lds, st, a, N, nchunks);
    hipLaunchKernelGGL(permute_scatter_kernel, dim3(nchunks, H, nsides), dim3(64), lds, st, a, N, nchunks);
    SVG2_HIP_CHECK(hipGetLastError());
    return SVG2_OK;
}

static void gather_launch(const int32_t *perm, int H, int N, int n_tensors, const void *const *src, void *const *dst,
                          int dtype, int d, hipStream_t st)
{
    GatherPtrs p = {};
    for (int t = 0; t < n_tensors; ++t) {
        p.src[t] = static_cast<const uint4 *>(src[t]);
        p.dst[t] = static_cast<uint4 *>(dst[t]);
    }
    const int row_bytes = d * (dtype == SVG2_BF16 ? 2 : 4);
    const int lanes_per_row = row_bytes / 16;
    const int rows_per_block = 256;
    hipLaunchKernelGGL(permute_gather_kernel, dim3(cdiv(N, rows_per_block), H, n_tensors), dim3(256), 0, st, p,
                       perm, N, lanes_per_row, rows_per_block);
}

int permute_launch(const int32_t *labels, int H, int N, int C, int32_t *offsets, int32_t *perm,
                   int32_t *inv_perm, int n_tensors, const void *const *src, void *const *dst,
                   int dtype, int d, void *ws, hipStream_t st)
{
    SortArgs a = {};
    a.s[0].labels = labels;
    a.s[0].C = C;
    a.s[0].hist = static_cast<int32_t *>(ws);
    a.s[0].offsets = offsets;
    a.s[0].perm = perm;
    a.s[0].inv_perm = inv_perm;
    {
        ProfileSpan sp(SVG2_K_PERMUTE_SORT, st);
        SVG2_TRY(sort_launch(a, 1, H, N, st));
    }
    if (n_tensors > 0) {
        ProfileSpan sp(SVG2_K_PERMUTE_GATHER, st);
        gather_launch(perm, H, N, n_tensors, src, dst, dtype, d, st);
    }
    SVG2_HIP_CHECK(hipGetLastError());
    return SVG2_OK;
}

// Both permutations of a layer (Section 4.1: pi_q for Q, pi_k shared by K and V) with one launch per sort step.
// ws holds the histograms of both sides (permute_ws_bytes for each, Q first).  copy = false: index vectors only.
int permute_pair_launch(const int32_t *labels_q, const int32_t *labels_k, int H, int N, int Cq, int Ck,
                        int32_t *offsets_q, int32_t *offsets_k, int32_t *perm_q, int32_t *perm_k, bool copy,
                        const void *Q, const void *K, const void *V, void *Qp, void *Kp, void *Vp, int dtype, int d,
                        void *ws, hipStream_t st)
{
    SortArgs a = {};
    a.s[0].labels = labels_q;
    a.s[0].C = Cq;
    a.s[0].hist = static_cast<int32_t *>(ws);
    a.s[0].offsets = offsets_q;
    a.s[0].perm = perm_q;
    a.s[1].labels = labels_k;
    a.s[1].C = Ck;
    a.s[1].hist = reinterpret_cast<int32_t *>(static_cast<char *>(ws) + permute_ws_bytes(H, N, Cq));
    a.s[1].offsets = offsets_k;
    a.s[1].perm = perm_k;
    {
        ProfileSpan sp(SVG2_K_PERMUTE_SORT, st);
        SVG2_TRY(sort_launch(a, 2, H, N, st));
    }
    if (copy) {
        ProfileSpan sp(SVG2_K_PERMUTE_GATHER, st);
        const void *src_q[1] = {Q};
        void *dst_q[1] = {Qp};
        gather_launch(perm_q, H, N, 1, src_q, dst_q, dtype, d, st);
        const void *src_k[2] = {K, V};
        void *dst_k[2] = {Kp, Vp};
        gather_launch(perm_k, H, N, 2, src_k, dst_k, dtype, d, st);
    }
    SVG2_HIP_CHECK(hipGetLastError());
    return SVG2_OK;
}

// Device address of `scratch` on the current device (looked up on the first call per device, then kept).
static constexpr int PERM_MAX_DEVICES = 64;
static std::mutex g_scratch_mu;
static void *g_scratch_ptr[PERM_MAX_DEVICES] = {};

int permute_static_scratch(void **out)
{
    int dev = -1;
    SVG2_HIP_CHECK(hipGetDevice(&dev));
    SVG2_REQUIRE(dev >= 0 && dev < PERM_MAX_DEVICES, SVG2_INVALID_ARG, "device ordinal %d is outside 0..%d", dev,
                 PERM_MAX_DEVICES - 1);
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        SVG2_HIP_CHECK(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        SVG2_REQUIRE(p != nullptr, SVG2_HIP_ERROR, "hipGetSymbolAddress returned a null address for the scratch array");
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return SVG2_OK;
}

}  // namespace svg2
