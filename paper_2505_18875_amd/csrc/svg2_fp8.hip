// FP8 storage of the attention operands (the "+ FP8" rows of the paper's Table 1).
//
// The paper gives no recipe, so this is a reading: Q, K and V are stored as OCP
// E4M3 (4 exponent bits, bias 7, 3 mantissa bits, largest value 448) with one
// scale per head and tensor (amax / 448); scores, the online softmax and all
// accumulators stay fp32; the probabilities go to the matrix cores as E4M3 too.
//
//   fp8_amax_kernel / fp8_quant_kernel   per-head amax (partial maxima, no atomics), then x * (448 / amax)
//                      rounded to nearest even by v_cvt_pk_fp8_f32.
//   attn_fp8_kernel    the block-sparse attention of Section 4.3 on E4M3
//                      operands: v_mfma_f32_32x32x64_f8f6f4 (the gfx950 instruction that
//                      runs E4M3 at twice the bf16 rate; the older 32x32x16 fp8 form runs
//                      at the bf16 rate), same work items, key tiles and transposed-score
//                      layout as the bf16 kernel, rows half as long.  What differs:
//                      * one instruction contracts 64 values: two per 32-key score block,
//                        and the second product is taken once per 64-key tile;
//                      * a probability is exp2(s - m) with the reference level m
//                        kept 2^6 BELOW the running maximum (re-levelled only when a
//                        score would exceed m by more than 2^8), so probabilities
//                        span (2^-9 .. 2^8] and the small ones of a flat row still
//                        land on normal E4M3 numbers;
//                      * the row sum is one more matrix instruction per tile (a V^T row
//                        of ones), so it is the sum of the ROUNDED probabilities, the
//                        same numbers that multiply V;
//                      * V^T comes out of LDS with the 8-bit transposing read
//                        (ds_read_b64_tr_b8).
//
// Two things the compiler does not take care of with these instructions (both seen as rare,
// run-to-run varying errors before they were handled): it places 18 wait states between a
// 32x32x64 f8f6f4 instruction and a vector instruction that touches its last result registers,
// the hardware needs 20 (measured); and it does not look into asm statements when it places
// the wait state a transcendental result needs before its first use.
#include <type_traits>

#include "svg2_attn_shared.h"

namespace svg2 {

typedef __attribute__((ext_vector_type(2))) int i32x2;
typedef __attribute__((ext_vector_type(8))) int i32x8;

static constexpr float E4M3_MAX = 448.0f;

// ---------------------------------------------------------------- quantisation
template <typename T> __device__ __forceinline__ void load8(const T *p, float *v);
template <> __device__ __forceinline__ void load8<float>(const float *p, float *v)
{
    const float4 a = reinterpret_cast<const float4 *>(p)[0], b = reinterpret_cast<const float4 *>(p)[1];
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}
template <> __device__ __forceinline__ void load8<bf16_t>(const bf16_t *p, float *v)
{
    const uint4 a = *reinterpret_cast<const uint4 *>(p);
    const unsigned w[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        v[2 * k] = __uint_as_float(w[k] << 16);
        v[2 * k + 1] = __uint_as_float(w[k] & 0xFFFF0000u);
    }
}

static constexpr int F8_AMAX_BLOCKS = 256;  // partial maxima per head

// max |x| over the 256 threads of a block (every thread gets it)
__device__ __forceinline__ float block_max_256(float m)
{
    __shared__ float s_m[4];
    for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
    __syncthreads();                            // s_m may still be read from an earlier call
    if ((threadIdx.x & 63) == 0) s_m[threadIdx.x >> 6] = m;
    __syncthreads();
    return fmaxf(fmaxf(s_m[0], s_m[1]), fmaxf(s_m[2], s_m[3]));
}

// grid (F8_AMAX_BLOCKS, H), block 256: partial[h][block] = max |x| over the block's share of the head
template <typename T>
__global__ __launch_bounds__(256) void fp8_amax_kernel(const T *__restrict__ X, size_t per_head,
                                                       float *__restrict__ partial)
{
    const int h = blockIdx.y;
    const T *xh = X + (size_t)h * per_head;
    float m = 0.f;
    // four independent 16-byte loads per thread and pass (8 values each), a block covers 8192 contiguous values
    constexpr int U = 4;
    for (size_t i0 = (size_t)blockIdx.x * (256 * 8 * U); i0 < per_head; i0 += (size_t)gridDim.x * (256 * 8 * U)) {
        float v[U][8];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const size_t i = i0 + ((size_t)u * 256 + threadIdx.x) * 8;
            if (i < per_head) load8<T>(xh + i, v[u]);
            else {
#pragma unroll
                for (int k = 0; k < 8; ++k) v[u][k] = 0.f;
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int k = 0; k < 8; ++k) m = fmaxf(m, fabsf(v[u][k]));
    }
    m = block_max_256(m);
    if (threadIdx.x == 0) partial[(size_t)h * F8_AMAX_BLOCKS + blockIdx.x] = m;
}

// four floats -> four E4M3 codes (round to nearest even), byte k = value k
__device__ __forceinline__ unsigned pack_e4m3x4(float a, float b, float c, float d)
{
    int w = 0;
    w = __builtin_amdgcn_cvt_pk_fp8_f32(a, b, w, false);
    w = __builtin_amdgcn_cvt_pk_fp8_f32(c, d, w, true);
    return (unsigned)w;
}

__device__ __forceinline__ float clamp_e4m3(float y) { return fminf(fmaxf(y, -E4M3_MAX), E4M3_MAX); }

// grid (blocks, H), block 256: 16 values per thread and pass
template <typename T>
__global__ __launch_bounds__(256) void fp8_quant_kernel(const T *__restrict__ X, size_t per_head,
                                                        const float *__restrict__ partial,
                                                        uint8_t *__restrict__ X8, float *__restrict__ scale)
{
    static_assert(F8_AMAX_BLOCKS == 256, "one partial maximum per thread");
    const int h = blockIdx.y;
    const float amax = block_max_256(partial[(size_t)h * F8_AMAX_BLOCKS + threadIdx.x]);
    const float inv = (amax > 0.f) ? E4M3_MAX / amax : 1.0f;
    if (blockIdx.x == 0 && threadIdx.x == 0) scale[h] = (amax > 0.f) ? amax / E4M3_MAX : 1.0f;
    const T *xh = X + (size_t)h * per_head;
    uint8_t *oh = X8 + (size_t)h * per_head;
    for (size_t i = ((size_t)blockIdx.x * 256 + threadIdx.x) * 16; i < per_head; i += (size_t)gridDim.x * 256 * 16) {
        float v[16];
        load8<T>(xh + i, v);
        load8<T>(xh + i + 8, v + 8);
        unsigned w[4];
#pragma unroll
        for (int k = 0; k < 4; ++k)
            w[k] = pack_e4m3x4(clamp_e4m3(v[4 * k] * inv), clamp_e4m3(v[4 * k + 1] * inv),
                               clamp_e4m3(v[4 * k + 2] * inv), clamp_e4m3(v[4 * k + 3] * inv));
        *reinterpret_cast<uint4 *>(oh + i) = make_uint4(w[0], w[1], w[2], w[3]);
    }
}

size_t fp8_quant_ws_bytes(int H) { return align256((size_t)H * F8_AMAX_BLOCKS * sizeof(float)); }

int fp8_quant_launch(const void *X, int dtype, int H, int N, int d, void *X8, float *scale, void *ws, hipStream_t st)
{
    float *partial = static_cast<float *>(ws);       // [H][F8_AMAX_BLOCKS] partial maxima
    const size_t per_head = (size_t)N * d;
    const int nb = (int)std::min<size_t>(1024, (per_head + 256 * 16 - 1) / (256 * 16));
    if (dtype == SVG2_BF16) {
        const bf16_t *x = static_cast<const bf16_t *>(X);
        hipLaunchKernelGGL(fp8_amax_kernel<bf16_t>, dim3(F8_AMAX_BLOCKS, H), dim3(256), 0, st, x, per_head, partial);
        hipLaunchKernelGGL(fp8_quant_kernel<bf16_t>, dim3(nb, H), dim3(256), 0, st, x, per_head, partial,
                           static_cast<uint8_t *>(X8), scale);
    } else {
        const float *x = static_cast<const float *>(X);
        hipLaunchKernelGGL(fp8_amax_kernel<float>, dim3(F8_AMAX_BLOCKS, H), dim3(256), 0, st, x, per_head, partial);
        hipLaunchKernelGGL(fp8_quant_kernel<float>, dim3(nb, H), dim3(256), 0, st, x, per_head, partial,
                           static_cast<uint8_t *>(X8), scale);
    }
    SVG2_HIP_CHECK(hipGetLastError());
    return SVG2_OK;
}

// ---------------------------------------------------------------- attention on E4M3 operands
// LDS transposing read for 8-bit data: the 16 lanes of a block each pass the address of 8
// consecutive bytes; with i < 8, lane i gets byte i of the rows of lanes 0, 2, .., 14 and lane
// 8 + i gets byte i of the rows of lanes 1, 3, .., 15.
__device__ __forceinline__ long lds_read_tr8(const lds_u8 *p)
{
    const i32x2 v = __builtin_amdgcn_ds_read_tr8_b64_v2i32((__attribute__((address_space(3))) i32x2 *)p);
    long r;
    __builtin_memcpy(&r, &v, 8);
    return r;
}

static constexpr int F8_NSTG = 2;           // K and V tile buffers in LDS (each).  A third one (tiles requested a tile
                                            // earlier) was measured slower on the Wan-like layer (8-head probe, ms sparse /
                                            // dense: 5.30 / 15.6 against 5.08 / 14.9); the tile loop is written for two
static constexpr float F8_HEADROOM = 8.0f;  // a score may exceed the reference level by 2^8 before it moves
static constexpr float F8_LEVEL = 6.0f;     // the reference level is put 2^6 below the block maximum

template <int D>
__global__ __launch_bounds__(64 * ATT_NW, 8 / ATT_NW) void attn_fp8_kernel(
    const uint8_t *__restrict__ Q, const uint8_t *__restrict__ K, const uint8_t *__restrict__ V,
    const float *__restrict__ scale_q, const float *__restrict__ scale_k, const float *__restrict__ scale_v, int H,
    int N, int Cq, int Ck, const int32_t *__restrict__ row_ptr, const int32_t *__restrict__ perm_q,
    const int32_t *__restrict__ perm_k, const int4 *__restrict__ tiles, const int32_t *__restrict__ tile_base,
    const int32_t *__restrict__ order, int max_tiles, const int2 *__restrict__ runs,
    const int32_t *__restrict__ row_keys, const int32_t *__restrict__ tile_run, int key_tiles, float scale_log2_base,
    int group, bf16_t *__restrict__ O, float *__restrict__ lse)
{
    static_assert(D == 128, "row = 128 bytes: the swizzles below are written for that");
    constexpr int KU = D / 64;                 // matrix instructions per score block (64 values of d each)
    constexpr int DVB = D / 32;                // 32-row blocks of O^T
    constexpr int RB = D;                      // bytes per K / V row
    constexpr int CPR = RB / 16;               // 16-byte chunks per row
    constexpr int RPI = 1024 / RB;             // rows one direct-to-LDS load instruction fills
    constexpr int NW = ATT_NW, NSTG = F8_NSTG;
    constexpr int NPASS = ATT_BN / (NW * RPI);
    static_assert(NPASS >= 1, "a tile needs at least one load instruction per wavefront");
    constexpr int TILE_B = ATT_BN * RB;

    // LDS: K tiles [NSTG][64][128 B], V tiles likewise, rows unpadded; 16-byte chunk c of row r
    // sits at position c ^ swz(r):
    //   K  swz = (r / 2) % 8                 the 16 rows of one ds_read_b128 pass cover all banks
    //   V  swz = 2 * (bit 1 of r + 2 * bit 3 of r)   the 8 rows (x 32 bytes) of half a transposing read differ
    extern __shared__ __align__(16) unsigned char s_raw[];
    unsigned char *sK = s_raw;
    unsigned char *sV = s_raw + NSTG * TILE_B;
    int32_t *s_rows = reinterpret_cast<int32_t *>(s_raw + 2 * NSTG * TILE_B);   // [2][64]
    int2 *s_run = reinterpret_cast<int2 *>(s_rows + 2 * ATT_BN);    // [nnz + 1]

    // work item: as in the bf16 kernel (one list of all tiles, ATT_GROUP consecutive tiles per XCD)
    const int xcd = blockIdx.x % 8, slot = blockIdx.x / 8;
    const int pos = (slot / group) * (8 * group) + xcd * group + slot % group;
    if (pos >= tile_base[H]) return;
    const int v = order[pos];                   // longest work items first
    int h = 0;
    for (int step = 1 << 15; step > 0; step >>= 1)
        if (h + step < H && tile_base[h + step] <= v) h += step;
    const int t = v - tile_base[h];
    const int4 desc = tiles[(size_t)h * max_tiles + t];
    const int ci = desc.x, row0 = desc.y, nrows = desc.z;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int half = lane >> 5, col = lane & 31;

    const int e0 = row_ptr[(size_t)h * (Cq + 1) + ci];
    const int nnz = row_ptr[(size_t)h * (Cq + 1) + ci + 1] - e0;
    const int L = row_keys[(size_t)h * Cq + ci];
    const int2 *rn = runs + (size_t)h * Cq * Ck + e0;
    const int32_t *trh = tile_run + ((size_t)h * Cq + ci) * key_tiles;      // run in which each key tile starts
    for (int e = tid; e < nnz; e += 64 * NW) s_run[e] = rn[e];
    if (tid == 0) s_run[nnz] = make_int2(0, L);

    const float scale_log2 = scale_log2_base * scale_q[h] * scale_k[h];
    const uint8_t *Qh = Q + (size_t)h * N * D;
    const char *Kb = reinterpret_cast<const char *>(K + (size_t)h * N * D);
    const char *Vb = reinterpret_cast<const char *>(V + (size_t)h * N * D);

    // ---- queries as the B operand of S^T = K Q^T.  One matrix instruction contracts 64 values of d,
    // 32 per lane half: half hf takes bytes 64 u + 32 hf .. + 32 of its row for instruction u, and
    // the K operand below is cut the same way (the instruction pairs byte j of the A lane with
    // byte j of the B lane of the same half, so any common order of the contraction index works).
    i32x8 qreg[KU];
    {
        int r = row0 + min(nrows - 1, wave * 32 + col);
        if (perm_k) r = perm_q[(size_t)h * N + r];
        const uint4 *src = reinterpret_cast<const uint4 *>(Qh + (size_t)r * D + 32 * half);
#pragma unroll
        for (int u = 0; u < KU; ++u) {
            const uint4 w0 = src[4 * u], w1 = src[4 * u + 1];
            __builtin_memcpy(&qreg[u], &w0, 16);
            __builtin_memcpy(reinterpret_cast<char *>(&qreg[u]) + 16, &w1, 16);
        }
    }
    const bool wave_active = wave * 32 < nrows;

    f32x16 oacc[DVB];
    float m_run = -INFINITY, l_run = 0.f;
#pragma unroll
    for (int b = 0; b < DVB; ++b)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[b][i] = 0.f;

    // ---- loader: as in the bf16 kernel (rows looked up by one wavefront, global -> LDS directly)
    const int32_t *pkh = perm_k ? perm_k + (size_t)h * N : nullptr;
    int cur = 0, row_pend = 0;
    int lk_hint = -1;                           // run in which the tile looked up next starts (-1: not known)
    const int ld_row = lane / CPR;
    const int ld_r = wave * RPI + ld_row;       // tile row modulo 32 (load pass p adds 32 p)
    const unsigned ld_koff = (unsigned)(((lane % CPR) ^ ((ld_r >> 1) & 7)) * 16);
    const unsigned ld_voff = (unsigned)(((lane % CPR) ^ (2 * (((ld_r >> 1) & 1) + 2 * ((ld_r >> 3) & 1)))) * 16);
    __syncthreads();                            // s_run visible

#define ATT_ROWS(KT)                                                                       \
    if (wave == ((KT) & (NW - 1))) {                                                       \
        const int kk = (KT) * ATT_BN + lane;                                               \
        int row_ = (kk < L) ? run_lookup(s_run, cur, kk) : 0;                              \
        if (perm_k) row_ = pkh[row_];                                                      \
        s_rows[((KT) & 1) * ATT_BN + lane] = row_ * RB;                                    \
    }
// The same in two steps, for the tile loop.  ISSUE, once a tile's fetches are on their way: the look-up of a later
// tile's rows and, gather-free, the load of the token index -- an ordinary load, so the compiler tracks it, with a
// whole tile of arithmetic to land in.  COMMIT, at the top of the next tile, behind the wait for all outstanding
// loads and the barrier that open it: the value has landed, and every wavefront has finished reading the half of
// s_rows that it goes to.
#define ATT_ROWS_ISSUE(KT)                                                                 \
    if (wave == ((KT) & (NW - 1))) {                                                       \
        const int kk = (KT) * ATT_BN + lane;                                               \
        cur = max(cur, lk_hint);                /* start at the tile's first run (from the plan) */ \
        row_pend = (kk < L) ? run_lookup(s_run, cur, kk) : 0;                              \
        if (perm_k) row_pend = pkh[row_pend];                                              \
    }
#define ATT_ROWS_COMMIT(KT)                                                                \
    if (wave == ((KT) & (NW - 1))) s_rows[((KT) & 1) * ATT_BN + lane] = row_pend * RB;
#define ATT_OFFS(KT, OFF)                                                                  \
    _Pragma("unroll") for (int p_ = 0; p_ < NPASS; ++p_)                                   \
        OFF[p_] = (unsigned)s_rows[((KT) & 1) * ATT_BN + (NW * p_ + wave) * RPI + ld_row];
#define ATT_FETCH(OFF, SRC, LOFF, DST)                                                     \
    _Pragma("unroll") for (int p_ = 0; p_ < NPASS; ++p_)                                   \
        load_to_lds_16(SRC, OFF[p_] + LOFF, DST + ((NW * p_ + wave) * RPI) * RB);

    const int ntile = (L + ATT_BN - 1) / ATT_BN;
    unsigned off_nx[NPASS];
    ATT_ROWS(0)
    ATT_ROWS(1)
    __syncthreads();
    if (ntile > 0) {
        ATT_OFFS(0, off_nx)
        ATT_FETCH(off_nx, Kb, ld_koff, sK)
        ATT_FETCH(off_nx, Vb, ld_voff, sV)
    }
    if (ntile > 1) {
        ATT_OFFS(1, off_nx)
        ATT_FETCH(off_nx, Kb, ld_koff, sK + TILE_B)
    }
    __syncthreads();                            // everyone has read the rows of tiles 0 and 1
    if (ntile > 2) { ATT_ROWS(2) }
    // tile 3 is looked up here and parked at the top of tile 0; the start of tile 4 is requested for the look-up at
    // the top of tile 0
    if (ntile > 3) {
        if (3 < key_tiles && wave == (3 & (NW - 1))) lk_hint = trh[3];
        ATT_ROWS_ISSUE(3)
    }
    lk_hint = -1;
    if (ntile > 4 && 4 < key_tiles && wave == (4 & (NW - 1))) lk_hint = trh[4];
    // off_nx stays live: the rows of tile NSTG - 1, whose V is requested at the top of tile 0

    // per-lane LDS read addresses (buffer 0): the two 16-byte halves of K operand u, V^T operand of column block b
    int koff[2 * KU], voff[DVB];
    {
        const int kz = (col >> 1) & 7;
#pragma unroll
        for (int c = 0; c < 2 * KU; ++c) koff[c] = col * RB + (((4 * (c >> 1) + 2 * half + (c & 1)) ^ kz) * 16);
        // V^T: lane r16 of a 16-lane block passes key i = r16 / 2 of the 8 keys this lane half has in a group of
        // 16 keys (byte j = 8 t + i of the operand <-> key 16 t + 8 (i / 4) + 4 half + i % 4 of the tile, the
        // order the probabilities come in) and the 8 output columns 32 b + 16 g16 + 8 (r16 % 2) ..; the read
        // hands lane l the column 32 b + l % 32.
        const int r16 = lane & 15, g16 = (lane >> 4) & 1, i = r16 >> 1;
        const int krow = 8 * (i >> 2) + 4 * half + (i & 3);
        const int vz = 2 * (((krow >> 1) & 1) + 2 * ((krow >> 3) & 1));
#pragma unroll
        for (int b = 0; b < DVB; ++b) voff[b] = krow * RB + ((((2 * b) ^ vz) + g16) * 16) + (r16 & 1) * 8;
        const int lds_base = (int)(unsigned)(size_t)(const lds_u8 *)s_raw;
#pragma unroll
        for (int c = 0; c < 2 * KU; ++c) { koff[c] += lds_base; asm volatile("" : "+v"(koff[c])); }
#pragma unroll
        for (int b = 0; b < DVB; ++b) { voff[b] += lds_base; asm volatile("" : "+v"(voff[b])); }
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);         // vmcnt(0)
    __syncthreads();

    // ---- schedule.  Scores and probabilities are handled in blocks of 32 keys (two per tile), the second
    // product once per 64-key tile (its contraction index is the whole tile).  Per tile t, with s0 = scores of
    // its block 0 already there and the reference level m decided for them:
    //   A:  s1 = K_{t,1} Q^T          (2 matrix instructions)  ||  pw[0..3] = exp2(s0 - m), LDS reads of V_t^T, K_{t+1,0}
    //   B:  maximum of s1, decision about m.  If m moved (rare), pw[0..3] is recomputed under the new m, so that
    //       both halves of the tile share one level.
    //   C:  s0 = K_{t+1,0} Q^T        (2)                      ||  pw[4..7] = exp2(s1 - m), LDS reads of V_t^T, K_{t+1,1}
    //   D:  accumulators brought to the level m if it moved since the last tile (rare);
    //       O^T += V_t^T P^T (4), l += 1^T P^T (1, last)       ||  maximum of the new s0, decision about m
    // Accumulator i of a score block is key 8 (i/4) + 4 half + i%4 of the block; word e of a block's probabilities
    // holds accumulators 4 e .. 4 e + 3; the B operand of the second product is pw[0..7].
#define ATT_FENCE __builtin_amdgcn_sched_barrier(0);
#define ATT_PIN(X) asm volatile("" : "+v"(X));
    constexpr int NOPS = 40;                    // vector operations of one block's probabilities
    const lds_u8 *lds = (const lds_u8 *)0;
    i32x8 ones;
#pragma unroll
    for (int i = 0; i < 8; ++i) ones[i] = 0x38383838;          // E4M3 1.0
    f32x16 s0, s1;
    int pw[8];                                  // probabilities of the tile: words 0..3 block 0, 4..7 block 1
    i32x8 ka[KU], va[DVB];                      // K operands of the next score block, V^T operands of this tile
    float m_acc = 0.f, t0 = 0.f, t1 = 0.f, t2 = 0.f, t3 = 0.f;
    for (int i = 0; i < 8; ++i) pw[i] = 0;
    f32x16 lt;                                  // row sums of the tile just accumulated (every element the same)
#pragma unroll
    for (int i = 0; i < 16; ++i) lt[i] = 0.f;
    bool any_upd = false;

    auto exp_op = [&](const f32x16 &S, auto w0_tag, int op) {
        const int e = op / 10, k = op % 10, w = decltype(w0_tag)::value + e;
        if (k == 0) { t0 = fmaf(S[4 * e], scale_log2, -m_run); ATT_PIN(t0) }
        else if (k == 1) { t1 = fmaf(S[4 * e + 1], scale_log2, -m_run); ATT_PIN(t1) }
        else if (k == 2) { t2 = fmaf(S[4 * e + 2], scale_log2, -m_run); ATT_PIN(t2) }
        else if (k == 3) { t3 = fmaf(S[4 * e + 3], scale_log2, -m_run); ATT_PIN(t3) }
        else if (k == 4) { t0 = __builtin_amdgcn_exp2f(t0); ATT_PIN(t0) }
        else if (k == 5) { t1 = __builtin_amdgcn_exp2f(t1); ATT_PIN(t1) }
        else if (k == 6) { t2 = __builtin_amdgcn_exp2f(t2); ATT_PIN(t2) }
        else if (k == 7) { t3 = __builtin_amdgcn_exp2f(t3); ATT_PIN(t3) }
        else if (k == 8) { pw[w] = __builtin_amdgcn_cvt_pk_fp8_f32(t0, t1, pw[w], false); ATT_PIN(pw[w]) }
        else { pw[w] = __builtin_amdgcn_cvt_pk_fp8_f32(t2, t3, pw[w], true); ATT_PIN(pw[w]) }
    };
    auto mask_block = [&](f32x16 &S, int base, int rem) {
#pragma unroll
        for (int i = 0; i < 16; ++i)
            if (base + 8 * (i >> 2) + 4 * half + (i & 3) >= rem) S[i] = -INFINITY;
    };
    auto decide = [&](float mx) {
        const float mx_s = max_xor32(mx) * scale_log2;
        const bool upd = mx_s > m_run + F8_HEADROOM;
        any_upd = __any(upd);
        m_run = upd ? mx_s - F8_LEVEL : m_run;
        ATT_PIN(m_run)
    };
    // The accumulators are expressed under the level m_acc; bring them to m_run.  Called once per tile, right
    // before the tile is accumulated (both decisions since the last tile are folded into one factor).  Ordinary
    // multiplications: the compiler sees every reader and writer of the accumulators and places the wait states
    // itself.  The matrix instructions of the previous tile have all completed here (its row sum, the last of
    // them, was read at the end of that tile).
    auto rescale_if_needed = [&]() {
        if (__any(m_acc != m_run)) {
            const float alpha = __builtin_amdgcn_exp2f(m_acc - m_run);
            m_acc = m_run;
            l_run *= alpha;
#pragma unroll
            for (int b = 0; b < DVB; ++b)
#pragma unroll
                for (int i = 0; i < 16; ++i) oacc[b][i] *= alpha;
        }
    };
    // 16-byte half c (0 .. 2 KU - 1) of the K operands of a score block whose first row is at KBYTE
    auto load_k = [&](auto kbyte_tag, int c) {
        constexpr int KBYTE = decltype(kbyte_tag)::value;
        const u32x4 w = lds_read_b128((lds + koff[c]) + KBYTE);
        __builtin_memcpy(reinterpret_cast<char *>(&ka[c >> 1]) + 16 * (c & 1), &w, 16);
    };
    // 8-byte piece idx (0 .. 4 DVB - 1) of the V^T operands of the tile at VBYTE: column block b = idx / 4 (kept in
    // va[b % 2]), key group idx % 4
    auto load_v = [&](auto vbyte_tag, int idx) {
        constexpr int VBYTE = decltype(vbyte_tag)::value;
        const int b = idx / 4, t = idx % 4;
        const long w = lds_read_tr8((lds + voff[b]) + (VBYTE + (t * 16) * RB));
        __builtin_memcpy(reinterpret_cast<char *>(&va[b]) + 8 * t, &w, 8);
    };
    // phases A and C: Sacc = K Q^T from ka (if DO_S)  ||  pw = exp2(Sexp - m); pieces V0 .. V0 + 3 of V^T;
    // each ka[u] is refilled with the operand of the block at KBYTE once its instruction has been issued (if DO_K)
    auto phase_s = [&](auto do_s_tag, auto do_k_tag, auto vbyte_tag, auto v0_tag, auto kbyte_tag, f32x16 &Sacc,
                       const f32x16 &Sexp, auto w0_tag) {
        constexpr bool DO_S = decltype(do_s_tag)::value;
        constexpr bool DO_K = decltype(do_k_tag)::value;
        constexpr int V0 = decltype(v0_tag)::value;
#pragma unroll
        for (int u = 0; u < KU; ++u) {
            if (DO_S) {
                const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                Sacc = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(ka[u], qreg[u], u == 0 ? zero : Sacc, 0, 0, 0, 0, 0,
                                                                       0);
            }
            ATT_FENCE
#pragma unroll
            for (int idx = V0 + (8 * u) / KU; idx < V0 + (8 * (u + 1)) / KU; ++idx) load_v(vbyte_tag, idx);
            if (DO_K) {
#pragma unroll
                for (int c = 2 * u; c < 2 * u + 2; ++c) load_k(kbyte_tag, c);
            }
#pragma unroll
            for (int op = (NOPS * u) / KU; op < (NOPS * (u + 1)) / KU; ++op) exp_op(Sexp, w0_tag, op);
            ATT_FENCE
        }
    };
    auto block_max = [&](const f32x16 &S) {
        float mx = max2_raw(fmaxf(S[0], S[1]), S[2]);
#pragma unroll
        for (int c = 1; c < 7; ++c) mx = max3_raw(mx, S[2 * c + 1], S[2 * c + 2]);
        return max2_raw(mx, S[15]);
    };
    // phase D: O^T += V^T P^T, l += 1^T P^T  ||  maximum of Snext and the decision (if DO_MAX).  The V^T operands
    // of column blocks 0 and 1 are there; those of blocks 2 and 3 are read into the same registers once the
    // instructions that use them have been issued.  The row-sum instruction goes LAST and its result is read at
    // the end of the phase: matrix instructions complete in order, so once that read is allowed every accumulator
    // of the tile has been written.  (Without it, the register copies the compiler places on the way out of the
    // tile loop read an accumulator that the last instruction is still writing: the wait states the compiler
    // inserts for that cover one basic block, not the branches out of the loop.)
    auto phase_pv = [&](auto do_max_tag, auto vbyte_tag, const f32x16 &Snext) {
        constexpr bool DO_MAX = decltype(do_max_tag)::value;
        static_assert(DVB == 4, "two operand registers serve four column blocks");
        float mx = -INFINITY;
        rescale_if_needed();
        const i32x8 pb = {pw[0], pw[1], pw[2], pw[3], pw[4], pw[5], pw[6], pw[7]};
#pragma unroll
        for (int b = 0; b < DVB; ++b) {
            oacc[b] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(va[b], pb, oacc[b], 0, 0, 0, 0, 0, 0);
            if (b == DVB - 1) {                 // every accumulator = the tile's row sum of this lane's query
                const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                lt = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(ones, pb, zero, 0, 0, 0, 0, 0, 0);
            }
            ATT_FENCE
            if (DO_MAX && b >= 2) {             // in the shadow of the last three instructions
#pragma unroll
                for (int c = 4 * (b - 2); c < 4 * (b - 1); ++c) {
                    if (c == 0) mx = max2_raw(fmaxf(Snext[0], Snext[1]), Snext[2]);
                    else if (c < 7) mx = max3_raw(mx, Snext[2 * c + 1], Snext[2 * c + 2]);
                    else mx = max2_raw(mx, Snext[15]);
                    ATT_PIN(mx)
                }
                if (b == DVB - 1) decide(mx);
            }
            ATT_FENCE
        }
        l_run += lt[0];
        // The compiler's wait states for this 16-pass instruction are two short of what the hardware needs before
        // the LAST result registers may be touched (measured: 20, inserted: 18), so nothing may read an
        // accumulator, or reuse a register of lt, right at that limit: four more wait states here, and lt stays
        // claimed until the next tile has started (see the tile loop).
        asm volatile("s_nop 3" : "+v"(lt));
    };
    using T = std::true_type;
    using F = std::false_type;

    // ---- prologue: scores of block 0 of tile 0 and their level, K operands of block 1
    if (wave_active && ntile > 0) {
#pragma unroll
        for (int c = 0; c < 2 * KU; ++c) load_k(std::integral_constant<int, 0>{}, c);
#pragma unroll
        for (int u = 0; u < KU; ++u) {
            const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            s0 = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(ka[u], qreg[u], u == 0 ? zero : s0, 0, 0, 0, 0, 0, 0);
        }
#pragma unroll
        for (int c = 0; c < 2 * KU; ++c) load_k(std::integral_constant<int, 32 * RB>{}, c);
        if (L < 32) mask_block(s0, 0, L);
        float mx = fmaxf(fmaxf(s0[0], s0[1]), s0[2]);
#pragma unroll
        for (int i = 3; i < 16; ++i) mx = fmaxf(mx, s0[i]);
        decide(mx);                             // key 0 exists: the maximum is finite
        m_acc = m_run;                          // the accumulators are zero: nothing to rescale
    }

#define ATT_TILE(BUF, HAS_NEXT)                                                            \
    {                                                                                      \
        /* the fetches issued NSTG - 1 tiles ago (V of this tile, K of the next) must have landed */ \
        __builtin_amdgcn_s_waitcnt(0x0F70);         /* vmcnt(0) */                         \
        __syncthreads();                                                                   \
        if (HAS_NEXT) {                                                                    \
            if (kt + NSTG + 1 < ntile) { ATT_ROWS_COMMIT(kt + NSTG + 1) }                  \
            if (kt + NSTG - 1 < ntile) { ATT_FETCH(off_nx, Vb, ld_voff, sV + ((BUF + NSTG - 1) % NSTG) * TILE_B) } \
            if (kt + NSTG < ntile) {                                                       \
                ATT_OFFS(kt + NSTG, off_nx)                                                \
                ATT_FETCH(off_nx, Kb, ld_koff, sK + BUF * TILE_B)                          \
            }                                                                              \
            /* rows of tile kt + NSTG + 2, parked at the top of the next tile (its start was requested a tile ago) */ \
            if (kt + NSTG + 2 < ntile) { ATT_ROWS_ISSUE(kt + NSTG + 2) }                   \
        }                                                                                  \
        if (wave_active) {                                                                 \
            asm volatile("" : "+v"(lt));            /* the registers of the last row sum are free from here on */ \
            using HN = std::integral_constant<bool, HAS_NEXT>;                             \
            constexpr int KB_ = ((BUF + 1) % NSTG) * TILE_B, VB_ = NSTG * TILE_B + BUF * TILE_B; \
            using VB = std::integral_constant<int, VB_>;                                   \
            phase_s(T{}, HN{}, VB{}, std::integral_constant<int, 0>{}, std::integral_constant<int, KB_>{}, s1, s0, \
                    std::integral_constant<int, 0>{});                                     \
            if (!HAS_NEXT) mask_block(s1, 32, L - kt * ATT_BN);                            \
            decide(block_max(s1));                                                         \
            if (any_upd) {                      /* rare: block 0 again, under the level both blocks share */ \
                _Pragma("unroll") for (int op = 0; op < NOPS; ++op) exp_op(s0, std::integral_constant<int, 0>{}, op); \
            }                                                                              \
            phase_s(HN{}, HN{}, VB{}, std::integral_constant<int, 8>{},                    \
                    std::integral_constant<int, KB_ + 32 * RB>{}, s0, s1, std::integral_constant<int, 4>{}); \
            if (HAS_NEXT && kt + 2 == ntile && L - (kt + 1) * ATT_BN < 32)                 \
                mask_block(s0, 0, L - (kt + 1) * ATT_BN);                                  \
            phase_pv(HN{}, VB{}, s0);                                                      \
        }                                                                                  \
        {       /* where the tile looked up at the top of the next tile starts: requested here */ \
            const int tn_ = kt + NSTG + 3;                                                 \
            lk_hint = -1;                                                                  \
            if (HAS_NEXT && tn_ < ntile && tn_ < key_tiles && wave == (tn_ & (NW - 1))) lk_hint = trh[tn_]; \
        }                                                                                  \
        ++kt;                                                                              \
    }
    static_assert(NSTG == 2, "the row look-up is parked behind the vmcnt(0) that opens a tile: written for two buffers");
    int kt = 0;
    while (kt < ntile - 1) {
        ATT_TILE(0, true)
        if (kt >= ntile - 1) break;
        ATT_TILE(1, true)
    }
    if (ntile > 0) {
        const int bl = kt % NSTG;
        if (bl == 0) ATT_TILE(0, false)
        else ATT_TILE(1, false)
    }
#undef ATT_TILE
#undef ATT_FENCE
#undef ATT_PIN
#undef ATT_ROWS
#undef ATT_ROWS_ISSUE
#undef ATT_ROWS_COMMIT
#undef ATT_OFFS
#undef ATT_FETCH

    // ---- epilogue: l_run is the whole row sum of this lane's query (both lane halves hold it)
    asm volatile("s_nop 7" : "+v"(lt));         // (see phase D: margin before the accumulators are read)
    {
        const int rl = wave * 32 + col;
        if (rl < nrows) {
            const int r = row0 + rl;
            const size_t dst = (size_t)h * N + (perm_q ? perm_q[(size_t)h * N + r] : r);
            const float l_tot = l_run;
            const float inv = (l_tot > 0.f) ? scale_v[h] / l_tot : 0.f;
#pragma unroll
            for (int b = 0; b < DVB; ++b)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int dv0 = b * 32 + 8 * g + 4 * half;
                    unsigned lo = (unsigned)f32_to_bf16(oacc[b][4 * g + 0] * inv) |
                                  ((unsigned)f32_to_bf16(oacc[b][4 * g + 1] * inv) << 16);
                    unsigned hi = (unsigned)f32_to_bf16(oacc[b][4 * g + 2] * inv) |
                                  ((unsigned)f32_to_bf16(oacc[b][4 * g + 3] * inv) << 16);
                    *reinterpret_cast<uint2 *>(O + dst * D + dv0) = make_uint2(lo, hi);
                }
            if (lse && half == 0)
                lse[dst] = (l_tot > 0.f) ? (m_run + log2f(l_tot)) * 0.6931471805599453f : -INFINITY;
        }
    }
}

static size_t attn_fp8_lds_bytes(int d, int Ck)
{
    return (size_t)2 * F8_NSTG * ATT_BN * d + 2 * ATT_BN * sizeof(int32_t) + (size_t)(Ck + 1) * sizeof(int2);
}

int attn_fp8_prepare()
{
    return set_dynamic_lds(reinterpret_cast<const void *>(attn_fp8_kernel<128>), attn_fp8_lds_bytes(128, SVG2_MAX_CLUSTERS));
}

int attn_fp8_main_launch(const void *Q8, const void *K8, const void *V8, const float *scale_q, const float *scale_k,
                         const float *scale_v, int H, int N, int d, int Cq, int Ck, const int32_t *row_ptr,
                         const int32_t *perm_q, const int32_t *perm_k, float scale, void *O, float *lse, void *ws,
                         hipStream_t st)
{
    const AttnWs a = attn_carve(ws, SVG2_BF16, H, N, Cq, Ck);   // same work items as the bf16 kernel
    if (!(scale > 0.f)) scale = 1.0f / sqrtf((float)d);
    const int total = H * a.max_tiles;
    const int group = ATT_GROUP;
    const int nwg = cdiv(total, 8 * group) * 8 * group;
    const float scale_log2 = scale * 1.4426950408889634f;
    const size_t lds = attn_fp8_lds_bytes(d, Ck);
    auto kern = attn_fp8_kernel<128>;
    hipLaunchKernelGGL(kern, dim3(nwg), dim3(64 * ATT_NW), lds, st, static_cast<const uint8_t *>(Q8),
                       static_cast<const uint8_t *>(K8), static_cast<const uint8_t *>(V8), scale_q, scale_k, scale_v, H,
                       N, Cq, Ck, row_ptr, perm_q, perm_k, a.tiles, a.tile_base, a.order, a.max_tiles, a.runs, a.row_keys,
                       a.tile_run, a.key_tiles, scale_log2, group, static_cast<bf16_t *>(O), lse);
    SVG2_HIP_CHECK(hipGetLastError());
    return SVG2_OK;
}

}  // namespace svg2
