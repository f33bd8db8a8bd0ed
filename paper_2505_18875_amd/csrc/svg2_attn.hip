// Block-sparse attention over variable-size clusters (paper Section 4.3).
//
// A work item is (head, tile of up to BM consecutive rows of ONE query
// cluster).  Its keys are the rows of the key clusters selected for that query
// cluster (one CSR row), taken as one virtual concatenated sequence that is
// consumed 64 keys at a time: a 64-key tile may straddle cluster boundaries,
// so short key clusters cost no padding; only the last tile of a work item is
// ragged and masked.  This plays the role of the per-token sparse load the
// paper describes, re-thought for LDS staging.
//
//   attn_plan_kernel   per head: tile descriptors (cluster, first row, rows)
//                      and, for every CSR entry, (first key row, keys before
//                      it in its CSR row).
//   attn_bf16_kernel   MFMA 32x32x16 bf16, FlashAttention-style online softmax
//                      in fp32.  Scores are computed transposed (S^T = K Q^T):
//                      a lane then holds 32 keys of ONE query, so row max / row
//                      sum stay in registers, and the probabilities are
//                      already laid out as the B operand of O^T += V^T P^T.
//                      V^T comes out of LDS through the transposing 64-bit
//                      read (ds_read_b64_tr_b16).
//   attn_f32_kernel    fp32 storage: plain FMA kernel, one query per thread.
//
// The result of sorted row r is stored at row perm_q[r] (Section 4.1: the
// inverse query permutation restores the original order).
#include "svg2_common.h"

namespace svg2 {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

static constexpr int ATT_BN = 64;          // keys per tile
static constexpr int ATT_GROUP = 8;        // consecutive tiles handed to one XCD

// ---------------------------------------------------------------- plan
// grid (H), block 256.
__global__ __launch_bounds__(256) void attn_plan_kernel(const int32_t *__restrict__ offsets_q,
                                                        const int32_t *__restrict__ offsets_k,
                                                        const int32_t *__restrict__ row_ptr,
                                                        const int32_t *__restrict__ col_idx, int Cq, int Ck, int BM,
                                                        int max_tiles, int4 *__restrict__ tiles,
                                                        int32_t *__restrict__ n_tiles, int2 *__restrict__ runs,
                                                        int32_t *__restrict__ row_keys)
{
    __shared__ int32_t s_wave[4];
    __shared__ int32_t s_carry;
    const int h = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int32_t *oq = offsets_q + (size_t)h * (Cq + 1);
    const int32_t *ok = offsets_k + (size_t)h * (Ck + 1);
    const int32_t *rp = row_ptr + (size_t)h * (Cq + 1);
    const int32_t *ci = col_idx + (size_t)h * Cq * Ck;
    int2 *rn = runs + (size_t)h * Cq * Ck;

    // tiles: running count over clusters, 256 clusters per pass
    if (tid == 0) s_carry = 0;
    __syncthreads();
    for (int c0 = 0; c0 < Cq; c0 += 256) {
        const int c = c0 + tid;
        const int start = (c < Cq) ? oq[c] : 0;
        const int size = (c < Cq) ? oq[c + 1] - start : 0;
        const int nt = (size + BM - 1) / BM;
        int incl = nt;
        for (int o = 1; o < 64; o <<= 1) {
            const int v = __shfl_up(incl, o);
            if (lane >= o) incl += v;
        }
        if (lane == 63) s_wave[wave] = incl;
        __syncthreads();
        int base = s_carry;
        for (int w = 0; w < wave; ++w) base += s_wave[w];
        const int first = base + incl - nt;
        for (int t = 0; t < nt; ++t)
            tiles[(size_t)h * max_tiles + first + t] = make_int4(c, start + t * BM, min(BM, size - t * BM), 0);
        __syncthreads();
        if (tid == 255) s_carry = base + incl;
        __syncthreads();
    }
    if (tid == 0) n_tiles[h] = s_carry;

    // runs: one wavefront per CSR row, 64 entries per pass
    for (int i = wave; i < Cq; i += 4) {
        const int e0 = rp[i], e1 = rp[i + 1];
        int carry = 0;
        for (int e = e0; e < e1; e += 64) {
            const int idx = e + lane;
            int start = 0, len = 0;
            if (idx < e1) {
                const int j = ci[idx];
                start = ok[j];
                len = ok[j + 1] - start;
            }
            int incl = len;
            for (int o = 1; o < 64; o <<= 1) {
                const int v = __shfl_up(incl, o);
                if (lane >= o) incl += v;
            }
            if (idx < e1) rn[idx] = make_int2(start, carry + incl - len);
            carry += __shfl(incl, 63);
        }
        if (lane == 0) row_keys[(size_t)h * Cq + i] = carry;
    }
}

// tile_base[h] = number of tiles of heads < h; tile_base[H] = all tiles.  One workgroup.
__global__ __launch_bounds__(256) void attn_tile_base_kernel(const int32_t *__restrict__ n_tiles, int H,
                                                             int32_t *__restrict__ tile_base)
{
    __shared__ int32_t s_wave[4];
    __shared__ int32_t s_carry;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) s_carry = 0;
    __syncthreads();
    for (int h0 = 0; h0 < H; h0 += 256) {
        const int h = h0 + tid;
        const int n = (h < H) ? n_tiles[h] : 0;
        int incl = n;
        for (int o = 1; o < 64; o <<= 1) {
            const int v = __shfl_up(incl, o);
            if (lane >= o) incl += v;
        }
        if (lane == 63) s_wave[wave] = incl;
        __syncthreads();
        int base = s_carry;
        for (int w = 0; w < wave; ++w) base += s_wave[w];
        if (h < H) tile_base[h] = base + incl - n;
        __syncthreads();
        if (tid == 255) s_carry = base + incl;
        __syncthreads();
    }
    if (tid == 0) tile_base[H] = s_carry;
}

// ---------------------------------------------------------------- bf16 MFMA kernel
// LDS transposing read: the 16 lanes of a block each pass the address of 4
// consecutive 16-bit values (row r = lane % 16); lane L gets element L % 4 of
// rows L / 4, L / 4 + 4, L / 4 + 8, L / 4 + 12.
__device__ __forceinline__ s16x4 lds_read_tr16(const bf16_t *p)
{
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (__attribute__((address_space(3))) s16x4 *)(uintptr_t)(const void *)p);
}

// Row of the permuted K / V that holds key number kk of the virtual key
// sequence; `cur` is a cursor into the run table that only moves forward.
__device__ __forceinline__ int run_lookup(const int2 *s_run, int &cur, int kk)
{
    int c = cur;
    while (kk >= s_run[c + 1].y) ++c;
    cur = c;
    const int2 rs = s_run[c];
    return rs.x + kk - rs.y;
}

template <int D, int QB>
__global__ __launch_bounds__(256, 2) void attn_bf16_kernel(
    const bf16_t *__restrict__ Q, const bf16_t *__restrict__ K, const bf16_t *__restrict__ V, int H, int N, int Cq,
    int Ck, const int32_t *__restrict__ row_ptr, const int32_t *__restrict__ perm_q,
    const int4 *__restrict__ tiles, const int32_t *__restrict__ tile_base, int max_tiles,
    const int2 *__restrict__ runs, const int32_t *__restrict__ row_keys, float scale_log2,
    bf16_t *__restrict__ O, float *__restrict__ lse)
{
    constexpr int KS = D / 16;                 // k-steps of QK^T
    constexpr int DVB = D / 32;                // 32-row blocks of O^T
    constexpr int ROWK = D + 8;                // LDS row strides (elements), chosen so that the 16 rows one
    constexpr int ROWV = D + 32;               // b128 pass / the 4 rows one transposing pass touch differ in banks
    constexpr int CPR = D / 8;                 // 16-byte chunks per row
    constexpr int LPASS = 256 / CPR;           // rows loaded per pass
    constexpr int NPASS = ATT_BN / LPASS;      // passes per 64-key tile

    extern __shared__ __align__(16) unsigned char s_raw[];
    bf16_t *sK = reinterpret_cast<bf16_t *>(s_raw);                 // [2][64][ROWK]
    bf16_t *sV = sK + 2 * ATT_BN * ROWK;                            // [2][64][ROWV]
    int32_t *s_rows = reinterpret_cast<int32_t *>(sV + 2 * ATT_BN * ROWV);   // [2][64]
    int2 *s_run = reinterpret_cast<int2 *>(s_rows + 2 * ATT_BN);    // [nnz + 1]

    // ---- which work item.  All tiles of all heads form one list (head-major, so
    // neighbours share keys).  Consecutive workgroup ids go round-robin over the 8
    // XCDs, each with its own L2: hand out the list in groups of ATT_GROUP
    // consecutive tiles per XCD, so tiles that share keys share an L2 and every XCD
    // gets the same amount of work whatever the per-head densities are.
    const int xcd = blockIdx.x % 8, slot = blockIdx.x / 8;
    const int v = (slot / ATT_GROUP) * (8 * ATT_GROUP) + xcd * ATT_GROUP + slot % ATT_GROUP;
    if (v >= tile_base[H]) return;
    int h = 0;
    for (int step = 1 << 15; step > 0; step >>= 1)
        if (h + step < H && tile_base[h + step] <= v) h += step;
    const int t = v - tile_base[h];
    const int4 desc = tiles[(size_t)h * max_tiles + t];
    const int ci = desc.x, row0 = desc.y, nrows = desc.z;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, col = lane & 31;

    const int e0 = row_ptr[(size_t)h * (Cq + 1) + ci];
    const int nnz = row_ptr[(size_t)h * (Cq + 1) + ci + 1] - e0;
    const int L = row_keys[(size_t)h * Cq + ci];
    const int2 *rn = runs + (size_t)h * Cq * Ck + e0;
    for (int e = tid; e < nnz; e += 256) s_run[e] = rn[e];
    if (tid == 0) s_run[nnz] = make_int2(0, L);

    const bf16_t *Qh = Q + (size_t)h * N * D;
    const bf16_t *Kh = K + (size_t)h * N * D;
    const bf16_t *Vh = V + (size_t)h * N * D;

    // ---- queries as the B operand of S^T = K Q^T
    bf16x8 qreg[QB][KS];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const int r = row0 + min(nrows - 1, (wave * QB + qb) * 32 + col);
        const uint4 *src = reinterpret_cast<const uint4 *>(Qh + (size_t)r * D + 8 * half);
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            const uint4 w = src[2 * s];
            __builtin_memcpy(&qreg[qb][s], &w, 16);
        }
    }
    const bool wave_active = (wave * QB) * 32 < nrows;

    f32x16 oacc[QB][DVB];
    float m_run[QB], l_run[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        m_run[qb] = -INFINITY;
        l_run[qb] = 0.f;
#pragma unroll
        for (int b = 0; b < DVB; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) oacc[qb][b][i] = 0.f;
    }

    // ---- loader.  The permuted K / V row of every key slot of a tile is looked up
    // by ONE wavefront (wave kt % 4, lane = slot) two tiles ahead and parked in
    // s_rows; every thread then copies chunk `lchunk` of slots lrow * NPASS + p.
    // The per-pass code is spelled out (ATT_FETCH) so the staging registers stay
    // in registers.
    const int lrow = tid / CPR, lchunk = tid % CPR;
    const char *Kb = reinterpret_cast<const char *>(Kh);
    const char *Vb = reinterpret_cast<const char *>(Vh);
    int cur = 0;
    uint4 kreg0, kreg1, kreg2, kreg3, vreg0, vreg1, vreg2, vreg3;
    kreg0 = kreg1 = kreg2 = kreg3 = vreg0 = vreg1 = vreg2 = vreg3 = make_uint4(0, 0, 0, 0);
    __syncthreads();                            // s_run visible

#define ATT_ROWS(KT)                                                                       \
    if (wave == ((KT) & 3)) {                                                              \
        const int kk = (KT) * ATT_BN + lane;                                               \
        s_rows[((KT) & 1) * ATT_BN + lane] = (kk < L) ? run_lookup(s_run, cur, kk) : 0;    \
    }
#define ATT_FETCH(P, KT)                                                                   \
    if (P < NPASS) {                                                                       \
        const unsigned off = (unsigned)s_rows[((KT) & 1) * ATT_BN + lrow * NPASS + P] * (unsigned)(D * 2) + lchunk * 16; \
        kreg##P = *reinterpret_cast<const uint4 *>(Kb + off);                              \
        vreg##P = *reinterpret_cast<const uint4 *>(Vb + off);                              \
    }
#define ATT_STAGE(P, BUF)                                                                  \
    if (P < NPASS) {                                                                       \
        const int r_ = (BUF) * ATT_BN + lrow * NPASS + P;                                  \
        *reinterpret_cast<uint4 *>(sK + r_ * ROWK + lchunk * 8) = kreg##P;                 \
        *reinterpret_cast<uint4 *>(sV + r_ * ROWV + lchunk * 8) = vreg##P;                 \
    }
#define ATT_FETCH_ALL(KT) ATT_FETCH(0, KT) ATT_FETCH(1, KT) ATT_FETCH(2, KT) ATT_FETCH(3, KT)
#define ATT_STAGE_ALL(BUF) ATT_STAGE(0, BUF) ATT_STAGE(1, BUF) ATT_STAGE(2, BUF) ATT_STAGE(3, BUF)

    const int ntile = (L + ATT_BN - 1) / ATT_BN;
    ATT_ROWS(0)
    ATT_ROWS(1)
    __syncthreads();
    if (ntile > 0) {
        ATT_FETCH_ALL(0)
        ATT_STAGE_ALL(0)
    }
    __syncthreads();

    // all global loads issued so far (queries, first tile) have landed: inside the loop
    // the only loads in flight are the prefetch of the next tile, which nothing in the
    // compute part has to wait for
    __builtin_amdgcn_s_waitcnt(0x0F70);         // vmcnt(0)
    for (int kt = 0; kt < ntile; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < ntile) { ATT_FETCH_ALL(kt + 1) }
        if (kt + 2 < ntile) { ATT_ROWS(kt + 2) }
        if (wave_active) {
            const bf16_t *bK = sK + buf * ATT_BN * ROWK;
            const bf16_t *bV = sV + buf * ATT_BN * ROWV;
            // ---- S^T block: rows = 64 keys (2 blocks of 32), columns = queries
            f32x16 sacc[2][QB];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int qb = 0; qb < QB; ++qb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) sacc[kb][qb][i] = 0.f;
#pragma unroll
            for (int s = 0; s < KS; ++s) {
#pragma unroll
                for (int kb = 0; kb < 2; ++kb) {
                    bf16x8 a;
                    const uint4 w = *reinterpret_cast<const uint4 *>(bK + (kb * 32 + col) * ROWK + 16 * s + 8 * half);
                    __builtin_memcpy(&a, &w, 16);
#pragma unroll
                    for (int qb = 0; qb < QB; ++qb)
                        sacc[kb][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[qb][s], sacc[kb][qb], 0, 0, 0);
                }
            }
            // ---- ragged end of the key sequence
            if (kt == ntile - 1 && (L % ATT_BN) != 0) {
                const int rem = L - kt * ATT_BN;
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int key = kb * 32 + 8 * (i >> 2) + 4 * half + (i & 3);
                        if (key >= rem)
#pragma unroll
                            for (int qb = 0; qb < QB; ++qb) sacc[kb][qb][i] = -INFINITY;
                    }
            }
            // ---- online softmax; accumulator i of block kb is key kb*32 + 8 (i/4) + 4 half + i%4
            bf16x8 pb[QB][4];
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) {
                float mx = sacc[0][qb][0];
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) mx = fmaxf(mx, sacc[kb][qb][i]);
                mx = fmaxf(mx, __shfl_xor(mx, 32));
                // the running maximum only moves when it would grow by more than 2^8: the
                // probabilities stay below 256 (fine in bf16 / fp32) and most tiles skip
                // the rescaling of the output accumulators
                const float mx_s = mx * scale_log2;
                const bool upd = mx_s > m_run[qb] + 8.0f;
                const float m_new = upd ? mx_s : m_run[qb];
                if (__any(upd)) {
                    const float alpha = __builtin_amdgcn_exp2f(m_run[qb] - m_new);
                    l_run[qb] *= alpha;
#pragma unroll
                    for (int b = 0; b < DVB; ++b)
#pragma unroll
                        for (int i = 0; i < 16; ++i) oacc[qb][b][i] *= alpha;
                }
                m_run[qb] = m_new;
                float psum = 0.f;
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int g = 0; g < 2; ++g) {
                        float p[8];
#pragma unroll
                        for (int j = 0; j < 8; ++j) {
                            p[j] = __builtin_amdgcn_exp2f(fmaf(sacc[kb][qb][8 * g + j], scale_log2, -m_new));
                            psum += p[j];
                        }
                        bf16x8 pk;
#pragma unroll
                        for (int j = 0; j < 8; ++j) pk[j] = (__bf16)p[j];
                        pb[qb][kb * 2 + g] = pk;
                    }
                l_run[qb] += psum;
            }
            // ---- O^T += V^T P^T
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
#pragma unroll
                for (int b = 0; b < DVB; ++b) {
                    const int r16 = lane & 15;
                    const int dv = b * 32 + ((lane >> 4) & 1) * 16 + 4 * (r16 & 3);
                    const int key0 = ks * 16 + 4 * half + (r16 >> 2);
                    const s16x4 lo = lds_read_tr16(bV + key0 * ROWV + dv);
                    const s16x4 hi = lds_read_tr16(bV + (key0 + 8) * ROWV + dv);
                    bf16x8 a;
                    __builtin_memcpy(&a, &lo, 8);
                    __builtin_memcpy(reinterpret_cast<char *>(&a) + 8, &hi, 8);
#pragma unroll
                    for (int qb = 0; qb < QB; ++qb)
                        oacc[qb][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb[qb][ks], oacc[qb][b], 0, 0, 0);
                }
            }
        }
        if (kt + 1 < ntile) { ATT_STAGE_ALL(buf ^ 1) }
        __syncthreads();
    }

#undef ATT_ROWS
#undef ATT_FETCH
#undef ATT_STAGE
#undef ATT_FETCH_ALL
#undef ATT_STAGE_ALL

    // ---- epilogue: normalise, store at the original row
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const int rl = (wave * QB + qb) * 32 + col;
        if (rl >= nrows) continue;
        const int r = row0 + rl;
        const size_t dst = (size_t)h * N + (perm_q ? perm_q[(size_t)h * N + r] : r);
        const float l_tot = l_run[qb] + __shfl_xor(l_run[qb], 32);
        const float inv = (l_tot > 0.f) ? 1.0f / l_tot : 0.f;
#pragma unroll
        for (int b = 0; b < DVB; ++b)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int dv0 = b * 32 + 8 * g + 4 * half;
                unsigned lo = (unsigned)f32_to_bf16(oacc[qb][b][4 * g + 0] * inv) |
                              ((unsigned)f32_to_bf16(oacc[qb][b][4 * g + 1] * inv) << 16);
                unsigned hi = (unsigned)f32_to_bf16(oacc[qb][b][4 * g + 2] * inv) |
                              ((unsigned)f32_to_bf16(oacc[qb][b][4 * g + 3] * inv) << 16);
                *reinterpret_cast<uint2 *>(O + dst * D + dv0) = make_uint2(lo, hi);
            }
        if (lse && half == 0)
            lse[dst] = (l_tot > 0.f) ? (m_run[qb] + log2f(l_tot)) * 0.6931471805599453f : -INFINITY;
    }
}

// ---------------------------------------------------------------- fp32 kernel
// grid (max_tiles, H), block 64: one query row per thread, 32 keys per LDS tile.
template <int D>
__global__ __launch_bounds__(64) void attn_f32_kernel(
    const float *__restrict__ Q, const float *__restrict__ K, const float *__restrict__ V, int N, int Cq, int Ck,
    const int32_t *__restrict__ row_ptr, const int32_t *__restrict__ perm_q, const int4 *__restrict__ tiles,
    const int32_t *__restrict__ n_tiles, int max_tiles, const int2 *__restrict__ runs,
    const int32_t *__restrict__ row_keys, float scale, float *__restrict__ O, float *__restrict__ lse)
{
    constexpr int TN = 32;
    __shared__ __align__(16) float sK[TN * D];
    __shared__ __align__(16) float sV[TN * D];
    const int h = blockIdx.y, t = blockIdx.x, tid = threadIdx.x;
    if (t >= n_tiles[h]) return;
    const int4 desc = tiles[(size_t)h * max_tiles + t];
    const int ci = desc.x, row0 = desc.y, nrows = desc.z;
    const int e0 = row_ptr[(size_t)h * (Cq + 1) + ci];
    const int nnz = row_ptr[(size_t)h * (Cq + 1) + ci + 1] - e0;
    const int L = row_keys[(size_t)h * Cq + ci];
    const int2 *rn = runs + (size_t)h * Cq * Ck + e0;
    const float *Kh = K + (size_t)h * N * D, *Vh = V + (size_t)h * N * D;

    const int r = row0 + min(tid, nrows - 1);
    float q[D], o[D];
#pragma unroll
    for (int k = 0; k < D / 4; ++k) {
        const float4 w = reinterpret_cast<const float4 *>(Q + ((size_t)h * N + r) * D)[k];
        q[4 * k] = w.x; q[4 * k + 1] = w.y; q[4 * k + 2] = w.z; q[4 * k + 3] = w.w;
    }
#pragma unroll
    for (int k = 0; k < D; ++k) o[k] = 0.f;
    float m = -INFINITY, l = 0.f;

    // loader: lanes 0..31 own key slot tid, lanes 32..63 the same slots (second half of the row)
    const int slot = tid & 31, hpart = tid >> 5;
    int cur = 0;
    for (int k0 = 0; k0 < L; k0 += TN) {
        __syncthreads();
        const int kk = k0 + slot;
        if (kk < L) {
            while (cur + 1 < nnz && kk >= rn[cur + 1].y) ++cur;
            const int2 rs = rn[cur];
            const size_t src = (size_t)(rs.x + kk - rs.y);
            const float4 *kp = reinterpret_cast<const float4 *>(Kh + src * D + hpart * (D / 2));
            const float4 *vp = reinterpret_cast<const float4 *>(Vh + src * D + hpart * (D / 2));
            float4 *dk = reinterpret_cast<float4 *>(sK + slot * D + hpart * (D / 2));
            float4 *dv = reinterpret_cast<float4 *>(sV + slot * D + hpart * (D / 2));
            for (int c = 0; c < D / 8; ++c) { dk[c] = kp[c]; dv[c] = vp[c]; }
        }
        __syncthreads();
        const int nk = min(TN, L - k0);
        float s[TN];
        float mx = -INFINITY;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            float acc = 0.f;
            if (j < nk) {
#pragma unroll
                for (int k = 0; k < D; ++k) acc = fmaf(q[k], sK[j * D + k], acc);
                acc *= scale;
                mx = fmaxf(mx, acc);
            }
            s[j] = acc;
        }
        const float m_new = fmaxf(m, mx);
        const float alpha = expf(m - m_new);
        m = m_new;
        l *= alpha;
#pragma unroll
        for (int k = 0; k < D; ++k) o[k] *= alpha;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            if (j < nk) {
                const float p = expf(s[j] - m_new);
                l += p;
#pragma unroll
                for (int k = 0; k < D; ++k) o[k] = fmaf(p, sV[j * D + k], o[k]);
            }
        }
    }
    if (tid < nrows) {
        const size_t dst = (size_t)h * N + (perm_q ? perm_q[(size_t)h * N + r] : r);
        const float inv = (l > 0.f) ? 1.0f / l : 0.f;
#pragma unroll
        for (int k = 0; k < D / 4; ++k)
            reinterpret_cast<float4 *>(O + dst * D)[k] =
                make_float4(o[4 * k] * inv, o[4 * k + 1] * inv, o[4 * k + 2] * inv, o[4 * k + 3] * inv);
        if (lse) lse[dst] = (l > 0.f) ? m + logf(l) : -INFINITY;
    }
}

// ---------------------------------------------------------------- host side
static constexpr int ATT_QB = 1;                 // 32-query blocks per wavefront (bf16 kernel)

static int attn_bm(int dtype) { return dtype == SVG2_BF16 ? 128 * ATT_QB : 64; }

size_t attn_ws_bytes(int dtype, int H, int N, int d, int Cq, int Ck)
{
    (void)d;
    const int max_tiles = cdiv(N, attn_bm(dtype)) + Cq;
    Carver c(nullptr);
    c.take<int4>((size_t)H * max_tiles);
    c.take<int32_t>((size_t)H);
    c.take<int32_t>((size_t)H + 1);
    c.take<int2>((size_t)H * Cq * Ck);
    c.take<int32_t>((size_t)H * Cq);
    return c.used;
}

struct AttnWs {
    int4 *tiles;
    int32_t *n_tiles, *tile_base;
    int2 *runs;
    int32_t *row_keys;
    int max_tiles;
};

static AttnWs attn_carve(void *ws, int dtype, int H, int N, int Cq, int Ck)
{
    AttnWs a;
    a.max_tiles = cdiv(N, attn_bm(dtype)) + Cq;
    Carver c(ws);
    a.tiles = c.take<int4>((size_t)H * a.max_tiles);
    a.n_tiles = c.take<int32_t>((size_t)H);
    a.tile_base = c.take<int32_t>((size_t)H + 1);
    a.runs = c.take<int2>((size_t)H * Cq * Ck);
    a.row_keys = c.take<int32_t>((size_t)H * Cq);
    return a;
}

int attn_plan_launch(int dtype, int H, int N, int Cq, int Ck, const int32_t *offsets_q, const int32_t *offsets_k,
                     const int32_t *row_ptr, const int32_t *col_idx, void *ws, hipStream_t st)
{
    const AttnWs a = attn_carve(ws, dtype, H, N, Cq, Ck);
    hipLaunchKernelGGL(attn_plan_kernel, dim3(H), dim3(256), 0, st, offsets_q, offsets_k, row_ptr, col_idx, Cq, Ck,
                       attn_bm(dtype), a.max_tiles, a.tiles, a.n_tiles, a.runs, a.row_keys);
    hipLaunchKernelGGL(attn_tile_base_kernel, dim3(1), dim3(256), 0, st, a.n_tiles, H, a.tile_base);
    SVG2_HIP_CHECK(hipGetLastError());
    return SVG2_OK;
}

int attn_main_launch(const void *Qp, const void *Kp, const void *Vp, int dtype, int H, int N, int d, int Cq, int Ck,
                     const int32_t *row_ptr, const int32_t *perm_q, float scale, void *O, float *lse, void *ws,
                     hipStream_t st)
{
    const AttnWs a = attn_carve(ws, dtype, H, N, Cq, Ck);
    const int max_tiles = a.max_tiles;
    int4 *tiles = a.tiles;
    int32_t *n_tiles = a.n_tiles;
    int32_t *tile_base = a.tile_base;
    int2 *runs = a.runs;
    int32_t *row_keys = a.row_keys;
    if (!(scale > 0.f)) scale = 1.0f / sqrtf((float)d);
    if (dtype == SVG2_BF16) {
        const int total = H * max_tiles;
        const int nwg = cdiv(total, 8 * ATT_GROUP) * 8 * ATT_GROUP;
        const float scale_log2 = scale * 1.4426950408889634f;
        const bf16_t *q = static_cast<const bf16_t *>(Qp), *k = static_cast<const bf16_t *>(Kp),
                     *v = static_cast<const bf16_t *>(Vp);
        bf16_t *o = static_cast<bf16_t *>(O);
        const size_t lds = (size_t)2 * ATT_BN * (2 * d + 40) * sizeof(bf16_t) + 2 * ATT_BN * sizeof(int32_t) +
                           (size_t)(Ck + 1) * sizeof(int2);
        if (d == 128) {
            auto kern = attn_bf16_kernel<128, ATT_QB>;
            SVG2_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
            hipLaunchKernelGGL(kern, dim3(nwg), dim3(256), lds, st, q, k, v, H, N, Cq, Ck, row_ptr, perm_q, tiles,
                               tile_base, max_tiles, runs, row_keys, scale_log2, o, lse);
        } else {
            auto kern = attn_bf16_kernel<64, ATT_QB>;
            SVG2_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
            hipLaunchKernelGGL(kern, dim3(nwg), dim3(256), lds, st, q, k, v, H, N, Cq, Ck, row_ptr, perm_q, tiles,
                               tile_base, max_tiles, runs, row_keys, scale_log2, o, lse);
        }
    } else {
        const float *q = static_cast<const float *>(Qp), *k = static_cast<const float *>(Kp),
                    *v = static_cast<const float *>(Vp);
        float *o = static_cast<float *>(O);
        if (d == 128)
            hipLaunchKernelGGL(attn_f32_kernel<128>, dim3(max_tiles, H), dim3(64), 0, st, q, k, v, N, Cq, Ck, row_ptr,
                               perm_q, tiles, n_tiles, max_tiles, runs, row_keys, scale, o, lse);
        else
            hipLaunchKernelGGL(attn_f32_kernel<64>, dim3(max_tiles, H), dim3(64), 0, st, q, k, v, N, Cq, Ck, row_ptr,
                               perm_q, tiles, n_tiles, max_tiles, runs, row_keys, scale, o, lse);
    }
    SVG2_HIP_CHECK(hipGetLastError());
    return SVG2_OK;
}

int attn_launch(const void *Qp, const void *Kp, const void *Vp, int dtype, int H, int N, int d, int Cq, int Ck,
                const int32_t *offsets_q, const int32_t *offsets_k, const int32_t *row_ptr,
                const int32_t *col_idx, const int32_t *perm_q, float scale, void *O, float *lse, void *ws,
                hipStream_t st)
{
    const int rc = attn_plan_launch(dtype, H, N, Cq, Ck, offsets_q, offsets_k, row_ptr, col_idx, ws, st);
    if (rc != SVG2_OK) return rc;
    return attn_main_launch(Qp, Kp, Vp, dtype, H, N, d, Cq, Ck, row_ptr, perm_q, scale, O, lse, ws, st);
}

}  // namespace svg2
