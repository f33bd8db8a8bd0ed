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
#include <type_traits>

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
typedef __attribute__((address_space(3))) unsigned char lds_u8;      // byte in LDS (32-bit address)

__device__ __forceinline__ s16x4 lds_read_tr16(const lds_u8 *p)
{
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)p);
}

typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

__device__ __forceinline__ u32x4 lds_read_b128(const lds_u8 *p)
{
    return *reinterpret_cast<const __attribute__((address_space(3))) u32x4 *>(p);
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

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;

// two floats -> two bf16 (round to nearest even) in one word, low half first
__device__ __forceinline__ unsigned pack_bf16x2(float a, float b)
{
    const f32x2 f = {a, b};
    const bf16x2 h = __builtin_convertvector(f, bf16x2);
    unsigned w;
    __builtin_memcpy(&w, &h, 4);
    return w;
}

// max / sum of a value with the one held by lane ^ 32 (v_permlane32_swap: no LDS round trip)
__device__ __forceinline__ float max_xor32(float x)
{
    const unsigned u = __float_as_uint(x);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float sum_xor32(float x)
{
    const unsigned u = __float_as_uint(x);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// acc + both bf16 halves of w (v_dot2c_f32_bf16 with a vector of ones): the row sum is taken
// over the rounded probabilities, the same values the matrix cores multiply with V
__device__ __forceinline__ float add_bf16x2(unsigned w, float acc)
{
    bf16x2 x;
    __builtin_memcpy(&x, &w, 4);
    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
    return __builtin_amdgcn_fdot2_f32_bf16(x, ones, acc, false);
}

// words 4 k .. 4 k + 3 of the packed probabilities as an MFMA operand
__device__ __forceinline__ bf16x8 pb_operand(const unsigned *pw, int k)
{
    bf16x8 r;
    __builtin_memcpy(&r, pw + 4 * k, 16);
    return r;
}

template <int D>
__global__ __launch_bounds__(256, 2) void attn_bf16_kernel(
    const bf16_t *__restrict__ Q, const bf16_t *__restrict__ K, const bf16_t *__restrict__ V, int H, int N, int Cq,
    int Ck, const int32_t *__restrict__ row_ptr, const int32_t *__restrict__ perm_q,
    const int4 *__restrict__ tiles, const int32_t *__restrict__ tile_base, int max_tiles,
    const int2 *__restrict__ runs, const int32_t *__restrict__ row_keys, float scale_log2, int group,
    bf16_t *__restrict__ O, float *__restrict__ lse)
{
    constexpr int KS = D / 16;                 // k-steps of QK^T
    constexpr int DVB = D / 32;                // 32-row blocks of O^T
    constexpr int RB = 2 * D;                  // bytes per K / V row
    constexpr int CPR = D / 8;                 // 16-byte chunks per row
    constexpr int RPI = 1024 / RB;             // rows one direct-to-LDS load instruction fills (64 lanes x 16 B)
    constexpr int NPASS = ATT_BN / (4 * RPI);  // such instructions per wavefront, tile and tensor
    constexpr int TILE_B = ATT_BN * RB;        // bytes of one K or V tile in LDS

    // LDS: K tiles [2][64][D] and V tiles [2][64][D], rows unpadded (the direct loads
    // fill 1024 contiguous bytes per instruction); bank conflicts are avoided by
    // storing 16-byte chunk c of row r at position c ^ swz(r):
    //   K  swz = (r / (256 / RB)) % CPR        the 16 rows of one ds_read_b128 pass differ
    //   V  swz = 4 * ((r / (256 / RB)) % (CPR / 4))   the 4 rows of one transposing pass differ
    extern __shared__ __align__(16) unsigned char s_raw[];
    unsigned char *sK = s_raw;                                      // [2][TILE_B]
    unsigned char *sV = s_raw + 2 * TILE_B;                         // [2][TILE_B]
    int32_t *s_rows = reinterpret_cast<int32_t *>(s_raw + 4 * TILE_B);   // [2][64]
    int2 *s_run = reinterpret_cast<int2 *>(s_rows + 2 * ATT_BN);    // [nnz + 1]

    // ---- which work item.  All tiles of all heads form one list (head-major, so
    // neighbours share keys).  Consecutive workgroup ids go round-robin over the 8
    // XCDs, each with its own L2: hand out the list in groups of ATT_GROUP
    // consecutive tiles per XCD, so tiles that share keys share an L2 and every XCD
    // gets the same amount of work whatever the per-head densities are.
    const int xcd = blockIdx.x % 8, slot = blockIdx.x / 8;
    const int v = (slot / group) * (8 * group) + xcd * group + slot % group;
    if (v >= tile_base[H]) return;
    int h = 0;
    for (int step = 1 << 15; step > 0; step >>= 1)
        if (h + step < H && tile_base[h + step] <= v) h += step;
    const int t = v - tile_base[h];
    const int4 desc = tiles[(size_t)h * max_tiles + t];
    const int ci = desc.x, row0 = desc.y, nrows = desc.z;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // wavefront-uniform: lives in a scalar register
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

    // ---- queries as the B operand of S^T = K Q^T: this wavefront owns 32 rows of the tile
    bf16x8 qreg[KS];
    {
        const int r = row0 + min(nrows - 1, wave * 32 + col);
        const uint4 *src = reinterpret_cast<const uint4 *>(Qh + (size_t)r * D + 8 * half);
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            const uint4 w = src[2 * s];
            __builtin_memcpy(&qreg[s], &w, 16);
        }
    }
    const bool wave_active = wave * 32 < nrows;

    f32x16 oacc[DVB];
    float m_run = -INFINITY, l_run = 0.f;
#pragma unroll
    for (int b = 0; b < DVB; ++b)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[b][i] = 0.f;

    // ---- loader.  The permuted K / V row of every key slot of a tile is looked up by
    // ONE wavefront (wave kt % 4, lane = slot) two tiles ahead and parked in s_rows.
    // The rows then go from global memory straight into LDS (no staging registers):
    // load instruction (wave, p) fills LDS rows (4 p + wave) * RPI .. + RPI of the tile,
    // lane l the chunk position l % CPR of row l / CPR, so it fetches the global chunk
    // that the swizzle puts there.
    const char *Kb = reinterpret_cast<const char *>(Kh);
    const char *Vb = reinterpret_cast<const char *>(Vh);
    int cur = 0;
    const int ld_row = lane / CPR;                                  // row inside the instruction's group
    const int ld_swz = ((wave * RPI + ld_row) / (256 / RB));
    const unsigned ld_koff = (unsigned)(((lane % CPR) ^ (ld_swz % CPR)) * 16);
    const unsigned ld_voff = (unsigned)(((lane % CPR) ^ (4 * (ld_swz % (CPR / 4)))) * 16);
    __syncthreads();                            // s_run visible

#define ATT_ROWS(KT)                                                                       \
    if (wave == ((KT) & 3)) {                                                              \
        const int kk = (KT) * ATT_BN + lane;                                               \
        s_rows[((KT) & 1) * ATT_BN + lane] = (kk < L) ? run_lookup(s_run, cur, kk) : 0;    \
    }
#define ATT_FETCH(P, KT, BUF)                                                              \
    if (P < NPASS) {                                                                       \
        const int grp_ = (4 * P + wave) * RPI;                                             \
        const unsigned off_ = (unsigned)s_rows[((KT) & 1) * ATT_BN + grp_ + ld_row] * (unsigned)RB;        \
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(Kb + (off_ + ld_koff)), \
                                         (__attribute__((address_space(3))) void *)(sK + (BUF) * TILE_B + grp_ * RB), 16, 0, 0); \
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(Vb + (off_ + ld_voff)), \
                                         (__attribute__((address_space(3))) void *)(sV + (BUF) * TILE_B + grp_ * RB), 16, 0, 0); \
    }
// Online-softmax bookkeeping for one block of 32 scores per query (16 per lane, the
// other 16 in lane ^ 32).  The running maximum only moves when it would grow by
// more than 2^8, so probabilities stay below 256 and the rescaling of the output
// accumulators is rare.  FIX_PB: block 0's probabilities (pw[0..7]) are already
// computed but not yet accumulated, so they are rescaled too.
#define ATT_NEW_MAX(S, FIX_PB)                                                             \
    {                                                                                      \
        float mx = fmaxf(fmaxf(S[0], S[1]), S[2]);                                         \
        _Pragma("unroll") for (int i = 3; i < 16; ++i) mx = fmaxf(mx, S[i]);               \
        mx = max_xor32(mx);                                                                \
        const float mx_s = mx * scale_log2;                                                \
        const bool upd = mx_s > m_run + 8.0f;                                              \
        if (__any(upd)) {                                                                  \
            const float m_new = upd ? mx_s : m_run;                                        \
            const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);                     \
            m_run = m_new;                                                                 \
            l_run *= alpha;                                                                \
            _Pragma("unroll") for (int b = 0; b < DVB; ++b)                                \
                _Pragma("unroll") for (int i = 0; i < 16; ++i) oacc[b][i] *= alpha;        \
            if (FIX_PB) {                                                                  \
                _Pragma("unroll") for (int j = 0; j < 8; ++j)                              \
                    pw[j] = pack_bf16x2(__uint_as_float(pw[j] << 16) * alpha,              \
                                        __uint_as_float(pw[j] & 0xFFFF0000u) * alpha);     \
            }                                                                              \
        }                                                                                  \
    }
#define ATT_FETCH_ALL(KT, BUF) ATT_FETCH(0, KT, BUF) ATT_FETCH(1, KT, BUF) ATT_FETCH(2, KT, BUF) ATT_FETCH(3, KT, BUF)

    const int ntile = (L + ATT_BN - 1) / ATT_BN;
    ATT_ROWS(0)
    ATT_ROWS(1)
    __syncthreads();
    if (ntile > 0) { ATT_FETCH_ALL(0, 0) }
    // per-lane LDS read offsets (bytes, buffer 0): K operand of k-step s, V^T operand of column block b
    int koff[KS], voff[DVB];
    {
        const int kz = (col / (256 / RB)) % CPR;
#pragma unroll
        for (int s = 0; s < KS; ++s) koff[s] = col * RB + (((2 * s + half) ^ kz) * 16);
        const int r16 = lane & 15;
        const int kr0 = 4 * half + (r16 >> 2);
        const int vz = 4 * ((kr0 / (256 / RB)) % (CPR / 4));
        const int cl = 2 * ((lane >> 4) & 1) + ((r16 & 3) >> 1);
#pragma unroll
        for (int b = 0; b < DVB; ++b) voff[b] = kr0 * RB + ((((4 * b) ^ vz) + cl) * 16) + (r16 & 1) * 8;
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);         // vmcnt(0): queries and the first tile have landed
    __syncthreads();

    // One 64-key tile of this wavefront's 32 queries, from LDS buffer `buf`.  RAGGED: keys
    // past `rem` do not exist (end of the key sequence) and get a score of -inf.
    //
    // The tile is two blocks of 32 keys, each with its own online-softmax step, and the
    // instruction stream is laid out by hand (ATT_FENCE keeps the compiler from moving
    // code across chunk boundaries): every matrix instruction of the second score block
    // is followed by the vector work (exp2, row sum, bf16 packing) of 16 / KS scores of
    // the first block, and every matrix instruction that accumulates the first block
    // into the output by the vector work of the second block.  One matrix instruction
    // keeps the cores busy for 32 cycles, about what 7 vector instructions take.
    // Accumulator i of a block is key 8 (i/4) + 4 half + i%4 of that block.
#define ATT_FENCE __builtin_amdgcn_sched_barrier(0);
    auto compute_tile = [&](auto ragged_tag, auto buf_tag, int rem) {
        constexpr bool RAGGED = decltype(ragged_tag)::value;
        constexpr int BUF = decltype(buf_tag)::value;
        constexpr int EPC = 16 / KS;               // scores handled per chunk of score-block work
        constexpr int NPV = 2 * DVB;               // matrix instructions per block in O^T += V^T P^T
        constexpr int EPV = 16 / NPV;              // scores handled per chunk there
        // LDS addresses are a per-lane 32-bit base plus a compile-time constant, which the
        // DS instructions take as their immediate offset
        const lds_u8 *lds = (const lds_u8 *)s_raw;
        constexpr int KB = BUF * TILE_B, VB = 2 * TILE_B + BUF * TILE_B;
        // V^T operand of matrix instruction idx (ks = idx / DVB: 16 keys, b = idx % DVB: 32 output columns)
        auto load_v = [&](int idx) {
            const int ks = idx / DVB, b = idx % DVB;
            const s16x4 lo = lds_read_tr16((lds + voff[b]) + (VB + (ks * 16) * RB));
            const s16x4 hi = lds_read_tr16((lds + voff[b]) + (VB + (ks * 16 + 8) * RB));
            bf16x8 a;
            __builtin_memcpy(&a, &lo, 8);
            __builtin_memcpy(reinterpret_cast<char *>(&a) + 8, &hi, 8);
            return a;
        };
        f32x16 s0, s1;
        unsigned pw[16];                            // probabilities, two bf16 per word; 4 words = one B operand
        bf16x8 ka[KS];
        // ---- scores of block 0
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            const u32x4 w = lds_read_b128((lds + koff[s]) + KB);
            __builtin_memcpy(&ka[s], &w, 16);
        }
#pragma unroll
        for (int i = 0; i < 16; ++i) s0[i] = 0.f;
#pragma unroll
        for (int s = 0; s < KS; ++s) s0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[s], qreg[s], s0, 0, 0, 0);
        ATT_FENCE
        // operands of block 1 are fetched while the maximum of block 0 is worked out
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            const u32x4 w = lds_read_b128((lds + koff[s]) + (KB + 32 * RB));
            __builtin_memcpy(&ka[s], &w, 16);
        }
        if (RAGGED) {
#pragma unroll
            for (int i = 0; i < 16; ++i)
                if (8 * (i >> 2) + 4 * half + (i & 3) >= rem) s0[i] = -INFINITY;
        }
        ATT_NEW_MAX(s0, false)
        // ---- scores of block 1 (matrix cores)  ||  probabilities of block 0 (vector ALU)
#pragma unroll
        for (int i = 0; i < 16; ++i) s1[i] = 0.f;
        float psum = 0.f;
        ATT_FENCE
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            s1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[s], qreg[s], s1, 0, 0, 0);
            ATT_FENCE
#pragma unroll
            for (int e = EPC * s; e < EPC * s + EPC; e += 2) {
                const float p0 = __builtin_amdgcn_exp2f(fmaf(s0[e], scale_log2, -m_run));
                const float p1 = __builtin_amdgcn_exp2f(fmaf(s0[e + 1], scale_log2, -m_run));
                pw[e >> 1] = pack_bf16x2(p0, p1);
                psum = add_bf16x2(pw[e >> 1], psum);
            }
            ATT_FENCE
        }
        l_run += psum;
        bf16x8 vop[2];                              // V^T operands, alternating so no copies are needed
        vop[0] = load_v(0);
        if (RAGGED) {
#pragma unroll
            for (int i = 0; i < 16; ++i)
                if (32 + 8 * (i >> 2) + 4 * half + (i & 3) >= rem) s1[i] = -INFINITY;
        }
        ATT_NEW_MAX(s1, true)
        // ---- O^T += V^T P^T for block 0 (matrix cores)  ||  probabilities of block 1 (vector ALU)
        psum = 0.f;
        ATT_FENCE
#pragma unroll
        for (int idx = 0; idx < NPV; ++idx) {
            vop[(idx + 1) & 1] = load_v(idx + 1);   // idx + 1 = NPV is the first operand of block 1
            oacc[idx % DVB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vop[idx & 1], pb_operand(pw, idx / DVB),
                                                                      oacc[idx % DVB], 0, 0, 0);
            ATT_FENCE
#pragma unroll
            for (int e = EPV * idx; e < EPV * idx + EPV; e += 2) {
                const float p0 = __builtin_amdgcn_exp2f(fmaf(s1[e], scale_log2, -m_run));
                const float p1 = __builtin_amdgcn_exp2f(fmaf(s1[e + 1], scale_log2, -m_run));
                pw[8 + (e >> 1)] = pack_bf16x2(p0, p1);
                psum = add_bf16x2(pw[8 + (e >> 1)], psum);
            }
            ATT_FENCE
        }
        l_run += psum;
        // ---- O^T += V^T P^T for block 1
#pragma unroll
        for (int idx = NPV; idx < 2 * NPV; ++idx) {
            if (idx + 1 < 2 * NPV) vop[(idx + 1) & 1] = load_v(idx + 1);
            oacc[idx % DVB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vop[idx & 1], pb_operand(pw, idx / DVB),
                                                                      oacc[idx % DVB], 0, 0, 0);
        }
    };
#undef ATT_FENCE


    // Main loop, unrolled by two so that the LDS buffer index is a compile-time constant
    // (every LDS address is then a per-lane base plus an immediate).  While tile kt is
    // computed from buffer kt % 2, tile kt + 1 streams into the other buffer.
#define ATT_STEP(BUFC)                                                                     \
    {                                                                                      \
        ATT_FETCH_ALL(kt + 1, 1 - BUFC)                                                    \
        if (kt + 2 < ntile) { ATT_ROWS(kt + 2) }                                           \
        if (wave_active) compute_tile(std::false_type{}, std::integral_constant<int, BUFC>{}, ATT_BN); \
        __builtin_amdgcn_s_waitcnt(0x0F70);     /* vmcnt(0): the next tile is in LDS */    \
        __syncthreads();                                                                   \
        ++kt;                                                                              \
    }
    int kt = 0;
    while (kt < ntile - 1) {                    // every tile but the last: full, and a next one to fetch
        ATT_STEP(0)
        if (kt >= ntile - 1) break;
        ATT_STEP(1)
    }
    // the last tile (kept out of the loop so the loop body has a single path): maybe ragged
    if (ntile > 0 && wave_active) {
        const int rem = L - kt * ATT_BN;
        if (kt & 1) {
            if (rem < ATT_BN) compute_tile(std::true_type{}, std::integral_constant<int, 1>{}, rem);
            else compute_tile(std::false_type{}, std::integral_constant<int, 1>{}, ATT_BN);
        } else {
            if (rem < ATT_BN) compute_tile(std::true_type{}, std::integral_constant<int, 0>{}, rem);
            else compute_tile(std::false_type{}, std::integral_constant<int, 0>{}, ATT_BN);
        }
    }
#undef ATT_STEP

#undef ATT_NEW_MAX
#undef ATT_ROWS
#undef ATT_FETCH
#undef ATT_FETCH_ALL

    // ---- epilogue: normalise, store at the original row
    {
        const int rl = wave * 32 + col;
        if (rl < nrows) {
            const int r = row0 + rl;
            const size_t dst = (size_t)h * N + (perm_q ? perm_q[(size_t)h * N + r] : r);
            const float l_tot = sum_xor32(l_run);
            const float inv = (l_tot > 0.f) ? 1.0f / l_tot : 0.f;
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
static int attn_bm(int dtype) { return dtype == SVG2_BF16 ? 128 : 64; }   // rows per tile

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
        const int group = ATT_GROUP;
        const int nwg = cdiv(total, 8 * group) * 8 * group;
        const float scale_log2 = scale * 1.4426950408889634f;
        const bf16_t *q = static_cast<const bf16_t *>(Qp), *k = static_cast<const bf16_t *>(Kp),
                     *v = static_cast<const bf16_t *>(Vp);
        bf16_t *o = static_cast<bf16_t *>(O);
        const size_t lds = (size_t)4 * ATT_BN * d * sizeof(bf16_t) + 2 * ATT_BN * sizeof(int32_t) +
                           (size_t)(Ck + 1) * sizeof(int2);
        if (d == 128) {
            auto kern = attn_bf16_kernel<128>;
            SVG2_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
            hipLaunchKernelGGL(kern, dim3(nwg), dim3(256), lds, st, q, k, v, H, N, Cq, Ck, row_ptr, perm_q, tiles,
                               tile_base, max_tiles, runs, row_keys, scale_log2, group, o, lse);
        } else {
            auto kern = attn_bf16_kernel<64>;
            SVG2_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
            hipLaunchKernelGGL(kern, dim3(nwg), dim3(256), lds, st, q, k, v, H, N, Cq, Ck, row_ptr, perm_q, tiles,
                               tile_base, max_tiles, runs, row_keys, scale_log2, group, o, lse);
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
