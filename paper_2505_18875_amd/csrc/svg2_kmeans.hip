// Per-head Lloyd k-means (paper Section 4.1), batched over heads.
//
// One iteration = assign, update, finalize:
//   assign    token x centroid contraction with a fused argmin.
//             bf16 input: MFMA 32x32x16 bf16 with the centroid tile as the A
//             operand (rows) and the tokens as the B operand (columns), so a
//             lane's 16 accumulators are 16 centroids of ONE token and the
//             running argmin stays in registers.  dist = ||c||^2 - 2 x.c.
//             fp32 input: a plain FMA kernel (one token per thread).
//   update    segmented sum over the label-sorted token order: the counting sort
//             of the permutation stage gives offsets and the sorted token ids;
//             every cluster is cut into pieces of at most KM_SEG rows, one
//             wavefront sums one piece in registers (4 rows of 256 bytes per
//             load instruction) and writes a partial sum.  No atomics: the
//             partials of a cluster are added in a fixed order, so the
//             centroids are reproducible bit for bit, and the cost does not
//             depend on how skewed the cluster sizes are.
//   finalize  mean = sum / count (an empty cluster keeps its centroid), the
//             bf16 copy of the centroids the next assign reads, and ||c||^2.
//
// For bf16 input the assign step sees the centroids rounded to bf16 (both in
// x.c and in ||c||^2); the centroids handed back stay fp32 means.
#include <type_traits>

#include "svg2_common.h"

namespace svg2 {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

static constexpr int KM_CMAX = 512;    // centroids resident in LDS at a time (bf16 kernel)
static constexpr int KM_NW = 8;        // wavefronts per workgroup (bf16 kernel)
static constexpr int KM_TB = 2;        // 32-token blocks per wavefront (bf16 kernel)
static constexpr int KM_WG_TOKENS = KM_NW * KM_TB * 32;
static constexpr int KM_IB = 8;        // token blocks per work item (bf16 kernel)
static constexpr int KM_UB = 4;        // load instructions in flight per wavefront in the segmented sum
static constexpr int KM_SEG = 256;     // rows per piece of the segmented sum
static constexpr int KM_FULL_FIRST = 1; // iterations whose update step sums every cluster afresh ...
static constexpr int KM_FULL_EVERY = 16; // ... and again every so many iterations (bounds the rounding drift of the delta update)

// ---------------------------------------------------------------- finalize
// grid (C, H), block d.  mode 0: centroids <- init (first call).  mode 1: cluster sum = sum of the cluster's
// pieces (pieces first_piece[j] .. first_piece[j+1] of the head).  mode 2 (delta update): cluster sum = previous
// cluster sum + the pieces of the tokens that joined the cluster (new sort order) - the pieces of the tokens that
// left it (previous sort order).  The sums are kept in csum between iterations; an empty cluster keeps its
// centroid and gets the sum 0.  All additions happen in a fixed order: reproducible bit for bit.
template <bool BF16>
__global__ void kmeans_finalize_kernel(const float *__restrict__ init, float *__restrict__ centroids,
                                       const float *__restrict__ psum, const int32_t *__restrict__ first_piece,
                                       const int32_t *__restrict__ offsets, int max_pieces, int C, int d,
                                       bf16_t *__restrict__ cb, float *__restrict__ cn,
                                       int32_t *__restrict__ counts_out, int mode, float *__restrict__ csum,
                                       const float *__restrict__ psum_old, const int32_t *__restrict__ first_piece_old)
{
    __shared__ float s_red[2];
    const int j = blockIdx.x, h = blockIdx.y, k = threadIdx.x;
    const size_t idx = ((size_t)h * C + j) * d + k;
    float c;
    if (mode != 0) {
        const int cnt = offsets[(size_t)h * (C + 1) + j + 1] - offsets[(size_t)h * (C + 1) + j];
        const int p0 = first_piece[(size_t)h * (C + 1) + j], p1 = first_piece[(size_t)h * (C + 1) + j + 1];
        float s = (mode == 2) ? csum[idx] : 0.f;
        // the pieces are added in their order, one after the other (the result does not depend on how the loop is
        // unrolled); unrolled, the loads of 8 pieces are in flight together -- the largest cluster of a head has
        // dozens of pieces and its block decides how long the launch takes
#pragma unroll 8
        for (int q = p0; q < p1; ++q) s += psum[((size_t)h * max_pieces + q) * d + k];
        if (mode == 2) {
            const int o0 = first_piece_old[(size_t)h * (C + 1) + j], o1 = first_piece_old[(size_t)h * (C + 1) + j + 1];
#pragma unroll 8
            for (int q = o0; q < o1; ++q) s -= psum_old[((size_t)h * max_pieces + q) * d + k];
        }
        if (cnt > 0) {
            c = s / (float)cnt;
        } else {
            s = 0.f;
            c = centroids[idx];
        }
        csum[idx] = s;
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
// grid (items, H), block 64 * KM_NW, one workgroup per CU.  A work item is KM_IB blocks of
// KM_WG_TOKENS tokens of one head; the head's centroids (up to KM_CMAX at a time) stay in LDS
// for the whole item.  argmin_j ||c_j||^2 - 2 x.c_j is taken as argmax_j x.c_j - ||c_j||^2 / 2:
// the accumulators of the contraction start at -||c_j||^2 / 2 (the C operand of the first
// matrix instruction), so no vector instruction is spent on forming the distance.  With more
// than KM_CMAX centroids the running best of a token goes through `best_ws` between chunks.
template <int D, bool OBJ>
__global__ __launch_bounds__(64 * KM_NW, 1) void kmeans_assign_bf16_kernel(
    const bf16_t *__restrict__ X, const bf16_t *__restrict__ cb, const float *__restrict__ cn, int N, int C,
    int32_t *__restrict__ labels, float *__restrict__ best_ws, float *__restrict__ objective, int obj_stride)
{
    constexpr int KS = D / 16;              // MFMA k-steps
    constexpr int ROW = D + 8;              // LDS row stride in elements (16 bytes of padding)
    extern __shared__ __align__(16) unsigned char s_raw[];
    bf16_t *s_c = reinterpret_cast<bf16_t *>(s_raw);                           // [KM_CMAX][ROW]
    float *s_hcn = reinterpret_cast<float *>(s_raw + (size_t)KM_CMAX * ROW * 2);   // [KM_CMAX]: -||c||^2 / 2

    const int h = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, col = lane & 31;
    const bf16_t *Xh = X + (size_t)h * N * D;
    const bf16_t *cbh = cb + (size_t)h * C * D;
    const float *cnh = cn + (size_t)h * C;
    const int nchunk = (C + KM_CMAX - 1) / KM_CMAX;
    float obj = 0.f;

    for (int chunk = 0; chunk < nchunk; ++chunk) {
        const int c0 = chunk * KM_CMAX;
        const int cc = min(KM_CMAX, C - c0), ccp = (cc + 31) & ~31;
        __syncthreads();
        // stage the chunk (rows past the last centroid are zero and can never win)
        for (int e = tid; e < ccp * (D / 8); e += 64 * KM_NW) {
            const int r = e / (D / 8), part = e % (D / 8);
            uint4 v = make_uint4(0, 0, 0, 0);
            if (r < cc) v = reinterpret_cast<const uint4 *>(cbh + (size_t)(c0 + r) * D)[part];
            *reinterpret_cast<uint4 *>(&s_c[r * ROW + part * 8]) = v;
        }
        for (int t = tid; t < ccp; t += 64 * KM_NW) s_hcn[t] = (t < cc) ? -0.5f * cnh[c0 + t] : -INFINITY;
        __syncthreads();

        // Token blocks of the item, two register buffers: the tokens of block b + 1 are requested
        // from global memory before block b is computed.
        // tokens as the B operand: lane (col, half) holds elements 16 s + 8 half .. + 8 of token `col`
        bf16x8 xb[2][KM_TB][KS];
        const int blk0 = blockIdx.x * KM_IB;
        auto load_x = [&](auto buf_tag, int b) {
            constexpr int BUF = decltype(buf_tag)::value;
            const int tok0 = (blk0 + b) * KM_WG_TOKENS + wave * (KM_TB * 32);
#pragma unroll
            for (int tb = 0; tb < KM_TB; ++tb) {
                const int n = min(N - 1, tok0 + tb * 32 + col);
                const uint4 *src = reinterpret_cast<const uint4 *>(Xh + (size_t)n * D + 8 * half);
#pragma unroll
                for (int s = 0; s < KS; ++s) {
                    const uint4 v = src[2 * s];
                    __builtin_memcpy(&xb[BUF][tb][s], &v, 16);
                }
            }
        };
        // One step = one 32-centroid row block against the wavefront's KM_TB token blocks: KS * KM_TB
        // matrix instructions back to back, then the argmax of their accumulators on the vector ALU
        // while the other wavefront of the SIMD has the matrix cores.  The operands of the next step
        // (centroid rows, -||c||^2 / 2) are requested from LDS before the argmax.  argmax of a step:
        // m = max of the 16 accumulators (max3 chain), the offset of the first accumulator equal to m,
        // then one compare with the running best.
        auto compute = [&](auto buf_tag, int b) {
            constexpr int BUF = decltype(buf_tag)::value;
            const int tok0 = (blk0 + b) * KM_WG_TOKENS + wave * (KM_TB * 32);
            float best[KM_TB];
            int bidx[KM_TB];
#pragma unroll
            for (int tb = 0; tb < KM_TB; ++tb) {
                if (chunk == 0) {
                    best[tb] = -INFINITY;
                    bidx[tb] = 0;
                } else {
                    const int n = min(N - 1, tok0 + tb * 32 + col);
                    best[tb] = best_ws[(size_t)h * N + n];
                    bidx[tb] = labels[(size_t)h * N + n];
                }
            }
            const int nrb = ccp / 32;
            bf16x8 a[KS];
            f32x16 cinit;
            auto fetch = [&](int rb) {          // accumulator i is centroid 8 (i/4) + 4 half + i%4 of the row block
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const float4 v = *reinterpret_cast<const float4 *>(&s_hcn[rb * 32 + 8 * g + 4 * half]);
                    cinit[4 * g] = v.x; cinit[4 * g + 1] = v.y; cinit[4 * g + 2] = v.z; cinit[4 * g + 3] = v.w;
                }
                const bf16_t *arow = &s_c[(rb * 32 + col) * ROW + 8 * half];
#pragma unroll
                for (int s = 0; s < KS; ++s) {
                    const uint4 v = *reinterpret_cast<const uint4 *>(arow + 16 * s);
                    __builtin_memcpy(&a[s], &v, 16);
                }
            };
            fetch(0);
#pragma unroll 1
            for (int rb = 0; rb < nrb; ++rb) {
                f32x16 acc[KM_TB];
#pragma unroll
                for (int s = 0; s < KS; ++s)
#pragma unroll
                    for (int q = 0; q < KM_TB; ++q)
                        acc[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[s], xb[BUF][q][s], s == 0 ? cinit : acc[q], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                if (rb + 1 < nrb) fetch(rb + 1);
                __builtin_amdgcn_sched_barrier(0);
                const int rbase = c0 + rb * 32 + 4 * half;
#pragma unroll
                for (int q = 0; q < KM_TB; ++q) {
                    float m = fmaxf(fmaxf(acc[q][0], acc[q][1]), acc[q][2]);
#pragma unroll
                    for (int c = 1; c < 7; ++c) m = fmaxf(fmaxf(m, acc[q][2 * c + 1]), acc[q][2 * c + 2]);
                    m = fmaxf(m, acc[q][15]);
                    int off = 0;
#pragma unroll
                    for (int i = 15; i >= 0; --i)               // descending: a tie keeps the lower centroid
                        off = (acc[q][i] == m) ? 8 * (i >> 2) + (i & 3) : off;
                    const bool upd = m > best[q];                 // strict: a tie keeps the earlier row block
                    best[q] = upd ? m : best[q];
                    bidx[q] = upd ? rbase + off : bidx[q];
                    // the values have to exist here: keeps the argmax in front of the next contraction
                    asm volatile("" : "+v"(best[q]), "+v"(bidx[q]));
                }
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int tb = 0; tb < KM_TB; ++tb) {
                const float ob = __shfl_xor(best[tb], 32);
                const int oi = __shfl_xor(bidx[tb], 32);
                if (ob > best[tb] || (ob == best[tb] && oi < bidx[tb])) { best[tb] = ob; bidx[tb] = oi; }
                const int n = tok0 + tb * 32 + col;
                if (half == 0 && n < N) {
                    labels[(size_t)h * N + n] = bidx[tb];
                    if (chunk + 1 < nchunk) best_ws[(size_t)h * N + n] = best[tb];
                }
                if (OBJ && chunk + 1 == nchunk) {
                    float x2 = 0.f;                               // ||x||^2 of this lane's half of the token
#pragma unroll
                    for (int s = 0; s < KS; ++s)
#pragma unroll
                        for (int k = 0; k < 8; ++k) {
                            const float xv = (float)xb[BUF][tb][s][k];
                            x2 = fmaf(xv, xv, x2);
                        }
                    x2 += __shfl_xor(x2, 32);
                    if (half == 0 && n < N) obj += x2 - 2.f * best[tb];
                }
            }
        };
        // blocks of this item that hold tokens (wavefront-uniform)
        const int nblk = min(KM_IB, (N - blk0 * KM_WG_TOKENS + KM_WG_TOKENS - 1) / KM_WG_TOKENS);
        if (nblk > 0) load_x(std::integral_constant<int, 0>{}, 0);
#pragma unroll 1
        for (int b = 0; b < nblk; b += 2) {
            if (b + 1 < nblk) load_x(std::integral_constant<int, 1>{}, b + 1);
            compute(std::integral_constant<int, 0>{}, b);
            if (b + 1 < nblk) {
                if (b + 2 < nblk) load_x(std::integral_constant<int, 0>{}, b + 2);
                compute(std::integral_constant<int, 1>{}, b + 1);
            }
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
// Pieces of at most KM_SEG sorted rows, never crossing a cluster boundary.
// grid (H), block 256.
__global__ __launch_bounds__(256) void kmeans_pieces_kernel(const int32_t *__restrict__ offsets, int C,
                                                            int max_pieces, int4 *__restrict__ pieces,
                                                            int32_t *__restrict__ first_piece,
                                                            int32_t *__restrict__ n_pieces)
{
    __shared__ int32_t s_wave[4];
    __shared__ int32_t s_carry;
    const int h = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int32_t *off = offsets + (size_t)h * (C + 1);
    if (tid == 0) s_carry = 0;
    __syncthreads();
    for (int c0 = 0; c0 < C; c0 += 256) {
        const int c = c0 + tid;
        const int start = (c < C) ? off[c] : 0;
        const int size = (c < C) ? off[c + 1] - start : 0;
        const int np = (size + KM_SEG - 1) / KM_SEG;
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
        if (c < C) first_piece[(size_t)h * (C + 1) + c] = first;
        for (int t = 0; t < np; ++t)
            pieces[(size_t)h * max_pieces + first + t] = make_int4(c, start + t * KM_SEG, min(KM_SEG, size - t * KM_SEG), 0);
        __syncthreads();
        if (tid == 255) s_carry = base + incl;
        __syncthreads();
    }
    if (tid == 0) {
        first_piece[(size_t)h * (C + 1) + C] = s_carry;
        n_pieces[h] = s_carry;
    }
}

// grid (ceil(max_pieces / 4), H), block 256: one wavefront per piece.  A row is
// LPR lanes of 16 bytes; 64 / LPR rows are read per instruction and KM_UB
// instructions are in flight before their values are added.
template <typename T, int D>
__global__ __launch_bounds__(256) void kmeans_segsum_kernel(const T *__restrict__ X, const int32_t *__restrict__ perm,
                                                            int N, int max_pieces, const int4 *__restrict__ pieces,
                                                            const int32_t *__restrict__ n_pieces,
                                                            float *__restrict__ psum)
{
    constexpr int EPL = 16 / sizeof(T);            // elements per lane
    constexpr int LPR = D / EPL;                   // lanes per row
    constexpr int RPI = 64 / LPR;                  // rows per instruction
    const int h = blockIdx.y, lane = threadIdx.x & 63;
    const int piece = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (piece >= n_pieces[h]) return;
    const int4 desc = pieces[(size_t)h * max_pieces + piece];
    const int row0 = desc.y, nrows = desc.z;
    const int sub = lane / LPR, part = lane % LPR;
    const T *Xh = X + (size_t)h * N * D;
    const int32_t *pm = perm + (size_t)h * N;
    float acc[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] = 0.f;
    for (int r = 0; r < nrows; r += RPI * KM_UB) {
        uint4 v[KM_UB];
        bool ok[KM_UB];
#pragma unroll
        for (int u = 0; u < KM_UB; ++u) {
            const int rr = r + u * RPI + sub;
            ok[u] = rr < nrows;
            const int src = pm[row0 + min(rr, nrows - 1)];
            v[u] = reinterpret_cast<const uint4 *>(Xh + (size_t)src * D)[part];
        }
#pragma unroll
        for (int u = 0; u < KM_UB; ++u) {
            if (!ok[u]) continue;
            const unsigned w[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
            if (sizeof(T) == 2) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    acc[2 * q] += __uint_as_float(w[q] << 16);
                    acc[2 * q + 1] += __uint_as_float(w[q] & 0xFFFF0000u);
                }
            } else {
#pragma unroll
                for (int q = 0; q < 4; ++q) acc[q] += __uint_as_float(w[q]);
            }
        }
    }
    // lanes with the same `part` hold the same columns
#pragma unroll
    for (int o = LPR; o < 64; o <<= 1)
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[e] += __shfl_xor(acc[e], o);
    if (sub == 0) {
        float *out = psum + ((size_t)h * max_pieces + piece) * D + part * EPL;
#pragma unroll
        for (int e = 0; e < EPL; e += 4)
            *reinterpret_cast<float4 *>(out + e) = make_float4(acc[e], acc[e + 1], acc[e + 2], acc[e + 3]);
    }
}

// The same over the rows of a piece whose label in `other` differs from the piece's cluster: with `other` = the
// previous labels and the new sort order these are the tokens that JOINED the cluster in this iteration, with
// `other` = the new labels and the previous sort order the tokens that LEFT it.  A wavefront first scans its piece
// one row per lane and packs the rows that qualify into a list (in sorted order, so the sum keeps a fixed order),
// then reads only those rows of X.
template <typename T, int D>
__global__ __launch_bounds__(256) void kmeans_segsum_delta_kernel(const T *__restrict__ X,
                                                                  const int32_t *__restrict__ perm,
                                                                  const int32_t *__restrict__ other, int N,
                                                                  int max_pieces, const int4 *__restrict__ pieces,
                                                                  const int32_t *__restrict__ n_pieces,
                                                                  float *__restrict__ psum)
{
    constexpr int EPL = 16 / sizeof(T);
    constexpr int LPR = D / EPL;
    constexpr int RPI = 64 / LPR;
    __shared__ int32_t s_list[4][KM_SEG];
    const int h = blockIdx.y, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int piece = blockIdx.x * 4 + wave;
    if (piece >= n_pieces[h]) return;
    const int4 desc = pieces[(size_t)h * max_pieces + piece];
    const int cl = desc.x, row0 = desc.y, nrows = desc.z;
    const int sub = lane / LPR, part = lane % LPR;
    const T *Xh = X + (size_t)h * N * D;
    const int32_t *pm = perm + (size_t)h * N;
    const int32_t *ot = other + (size_t)h * N;
    int32_t *list = s_list[wave];
    const unsigned long long lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
    int cnt = 0;
    // the rows of the piece and then their other labels are requested together: two memory round trips for the
    // piece instead of two per 64 rows
    constexpr int NG = KM_SEG / 64;
    int srcs[NG], oth[NG];
#pragma unroll
    for (int i = 0; i < NG; ++i) {
        const int rr = i * 64 + lane;
        srcs[i] = (rr < nrows) ? pm[row0 + rr] : 0;
    }
#pragma unroll
    for (int i = 0; i < NG; ++i) oth[i] = ot[srcs[i]];
#pragma unroll
    for (int i = 0; i < NG; ++i) {
        if (i * 64 >= nrows) break;
        const bool take = i * 64 + lane < nrows && oth[i] != cl;
        const unsigned long long m = __ballot(take);
        if (take) list[cnt + __popcll(m & lt_mask)] = srcs[i];
        cnt += __popcll(m);
    }
    float acc[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] = 0.f;
    for (int r = 0; r < cnt; r += RPI * KM_UB) {
        uint4 v[KM_UB];
        bool ok[KM_UB];
#pragma unroll
        for (int u = 0; u < KM_UB; ++u) {
            const int rr = r + u * RPI + sub;
            ok[u] = rr < cnt;
            const int src = list[min(rr, cnt - 1)];
            v[u] = reinterpret_cast<const uint4 *>(Xh + (size_t)src * D)[part];
        }
#pragma unroll
        for (int u = 0; u < KM_UB; ++u) {
            if (!ok[u]) continue;
            const unsigned w[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
            if (sizeof(T) == 2) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    acc[2 * q] += __uint_as_float(w[q] << 16);
                    acc[2 * q + 1] += __uint_as_float(w[q] & 0xFFFF0000u);
                }
            } else {
#pragma unroll
                for (int q = 0; q < 4; ++q) acc[q] += __uint_as_float(w[q]);
            }
        }
    }
#pragma unroll
    for (int o = LPR; o < 64; o <<= 1)
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[e] += __shfl_xor(acc[e], o);
    if (sub == 0) {
        float *out = psum + ((size_t)h * max_pieces + piece) * D + part * EPL;
#pragma unroll
        for (int e = 0; e < EPL; e += 4)
            *reinterpret_cast<float4 *>(out + e) = make_float4(acc[e], acc[e + 1], acc[e + 2], acc[e + 3]);
    }
}

__global__ void kmeans_zero_kernel(float *p, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0.f;
}

// ---------------------------------------------------------------- host side
struct KmeansWs {
    bf16_t *cb;
    float *cn;
    // two sets of the label-sorted order and its pieces: iteration t uses set t % 2, so the previous iteration's
    // order is still there for the delta update
    int32_t *offsets[2], *perm[2], *first_piece[2], *n_pieces[2];
    int4 *pieces[2];
    float *psum[2], *best, *csum;
    int32_t *labels_prev;
    void *sort_ws;
    int max_pieces;
    size_t total;
};

static KmeansWs kmeans_carve(void *ws, int H, int N, int d, int C)
{
    KmeansWs k;
    k.max_pieces = cdiv(N, KM_SEG) + C;
    Carver c(ws);
    k.cb = c.take<bf16_t>((size_t)H * C * d);
    k.cn = c.take<float>((size_t)H * C);
    for (int s = 0; s < 2; ++s) {
        k.offsets[s] = c.take<int32_t>((size_t)H * (C + 1));
        k.perm[s] = c.take<int32_t>((size_t)H * N);
        k.first_piece[s] = c.take<int32_t>((size_t)H * (C + 1));
        k.n_pieces[s] = c.take<int32_t>((size_t)H);
        k.pieces[s] = c.take<int4>((size_t)H * k.max_pieces);
        k.psum[s] = c.take<float>((size_t)H * k.max_pieces * d);
    }
    k.csum = c.take<float>((size_t)H * C * d);
    k.labels_prev = c.take<int32_t>((size_t)H * N);
    k.best = c.take<float>(C > KM_CMAX ? (size_t)H * N : 0);
    k.sort_ws = c.take<char>(permute_ws_bytes(H, N, C));
    k.total = c.used;
    return k;
}

size_t kmeans_ws_bytes(int dtype, int H, int N, int d, int C)
{
    (void)dtype;
    return kmeans_carve(nullptr, H, N, d, C).total;
}

template <typename T, int D, bool BF16>
static int kmeans_run(const T *X, int H, int N, int C, int iters, const float *init, float *centroids,
                      int32_t *labels, int32_t *counts, float *objective, void *ws, hipStream_t st)
{
    const KmeansWs k = kmeans_carve(ws, H, N, D, C);
    if (objective)
        hipLaunchKernelGGL(kmeans_zero_kernel, dim3(cdiv(H * iters, 256)), dim3(256), 0, st, objective, H * iters);
    hipLaunchKernelGGL((kmeans_finalize_kernel<BF16>), dim3(C, H), dim3(D), 0, st, init, centroids, k.psum[0],
                       k.first_piece[0], k.offsets[0], k.max_pieces, C, D, k.cb, k.cn, (int32_t *)nullptr, 0, k.csum,
                       (const float *)nullptr, (const int32_t *)nullptr);
    for (int t = 0; t < iters; ++t) {
        float *obj = objective ? objective + t : nullptr;
        // Update step: the first KM_FULL_FIRST iterations, and every KM_FULL_EVERY-th after that, sum every
        // cluster afresh; the others only move the tokens whose label changed (a quarter in the second
        // iteration, a few per cent from the third on) between the cluster sums, which reads a fraction of X.
        const bool full = t < KM_FULL_FIRST || t % KM_FULL_EVERY == 0;
        const int s = t & 1;
        // the labels of iteration t go to the caller's buffer when iters - 1 - t is even, else to the scratch
        // buffer: the last iteration lands in the caller's buffer and the previous labels are always the other one
        int32_t *lab = ((iters - 1 - t) & 1) ? k.labels_prev : labels;
        const int32_t *lab_prev = ((iters - 1 - t) & 1) ? labels : k.labels_prev;
        if (BF16) {
            const dim3 grid(cdiv(cdiv(N, KM_WG_TOKENS), KM_IB), H);
            const bf16_t *Xb = reinterpret_cast<const bf16_t *>(X);
            const size_t lds = (size_t)KM_CMAX * (D + 8) * sizeof(bf16_t) + KM_CMAX * sizeof(float);
            auto kern = obj ? kmeans_assign_bf16_kernel<D, true> : kmeans_assign_bf16_kernel<D, false>;
            SVG2_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
            hipLaunchKernelGGL(kern, grid, dim3(64 * KM_NW), lds, st, Xb, k.cb, k.cn, N, C, lab, k.best, obj, iters);
        } else {
            const dim3 grid(cdiv(N, 128), H);
            const float *Xf = reinterpret_cast<const float *>(X);
            if (obj)
                hipLaunchKernelGGL((kmeans_assign_f32_kernel<D, true>), grid, dim3(128), 0, st, Xf, centroids, k.cn, N,
                                   C, lab, obj, iters);
            else
                hipLaunchKernelGGL((kmeans_assign_f32_kernel<D, false>), grid, dim3(128), 0, st, Xf, centroids, k.cn, N,
                                   C, lab, obj, iters);
        }
        // label-sorted order of the tokens, then the segmented sum over it
        const int rc = permute_launch(lab, H, N, C, k.offsets[s], k.perm[s], nullptr, 0, nullptr, nullptr, 0, 0,
                                      k.sort_ws, st);
        if (rc != SVG2_OK) return rc;
        hipLaunchKernelGGL(kmeans_pieces_kernel, dim3(H), dim3(256), 0, st, k.offsets[s], C, k.max_pieces, k.pieces[s],
                           k.first_piece[s], k.n_pieces[s]);
        const dim3 sgrid(cdiv(k.max_pieces, 4), H);
        if (full) {
            hipLaunchKernelGGL((kmeans_segsum_kernel<T, D>), sgrid, dim3(256), 0, st, X, k.perm[s], N, k.max_pieces,
                               k.pieces[s], k.n_pieces[s], k.psum[s]);
            hipLaunchKernelGGL((kmeans_finalize_kernel<BF16>), dim3(C, H), dim3(D), 0, st, (const float *)nullptr,
                               centroids, k.psum[s], k.first_piece[s], k.offsets[s], k.max_pieces, C, D, k.cb, k.cn,
                               counts, 1, k.csum, (const float *)nullptr, (const int32_t *)nullptr);
        } else {
            // tokens that joined a cluster: new order, previous labels; tokens that left: previous order, new labels
            hipLaunchKernelGGL((kmeans_segsum_delta_kernel<T, D>), sgrid, dim3(256), 0, st, X, k.perm[s],
                               lab_prev, N, k.max_pieces, k.pieces[s], k.n_pieces[s], k.psum[s]);
            hipLaunchKernelGGL((kmeans_segsum_delta_kernel<T, D>), sgrid, dim3(256), 0, st, X, k.perm[1 - s], lab, N,
                               k.max_pieces, k.pieces[1 - s], k.n_pieces[1 - s], k.psum[1 - s]);
            hipLaunchKernelGGL((kmeans_finalize_kernel<BF16>), dim3(C, H), dim3(D), 0, st, (const float *)nullptr,
                               centroids, k.psum[s], k.first_piece[s], k.offsets[s], k.max_pieces, C, D, k.cb, k.cn,
                               counts, 2, k.csum, k.psum[1 - s], k.first_piece[1 - s]);
        }
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
