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
//
// Gather-free variant (perm_k given): Q, K and V stay in token order and the
// kernels go through perm_q / perm_k when they fetch a row -- the per-token
// sparse load of Section 4.3 -- so no permuted copies are needed.
#include <algorithm>
#include <type_traits>

#include "svg2_attn_shared.h"

namespace svg2 {


// Launch shape of the bf16 kernel.  Measured on the Wan-like layer (8-head probe, ms sparse / dense):
// 4 wavefronts, 2 buffers, 2 workgroups per CU 7.76 / 24.5;  8 wavefronts, 3 buffers, 1 workgroup per CU
// (half the L2 -> LDS traffic, but 8 wavefronts behind one barrier) 8.17 / 25.7.
static constexpr int ATT_NSTG = 2;         // K and V tile buffers in LDS (each); the schedule is written for two
static constexpr int ATT_RUN_LDS = 1920;     // runs of a work item kept in LDS (15 KB: two workgroups of 80 KB still fit a CU)
static constexpr int ATT_OPS_B = 0;        // vector operations of a block's probabilities done early (see phase B)

// ---------------------------------------------------------------- plan
// grid (H), block 256.
__global__ __launch_bounds__(256) void attn_plan_kernel(const int32_t *__restrict__ offsets_q,
                                                        const int32_t *__restrict__ offsets_k,
                                                        const int32_t *__restrict__ row_ptr,
                                                        const int32_t *__restrict__ col_idx, int Cq, int Ck, int BM,
                                                        int max_tiles, int4 *__restrict__ tiles,
                                                        int32_t *__restrict__ n_tiles, int2 *__restrict__ runs,
                                                        int32_t *__restrict__ row_keys,
                                                        int32_t *__restrict__ cl_first, int key_tiles,
                                                        int32_t *__restrict__ tile_run)
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
        if (c < Cq) cl_first[(size_t)h * Cq + c] = first;
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
            if (idx < e1) {
                const int before = carry + incl - len;          // keys of the row in front of this run
                rn[idx] = make_int2(start, before);
                // the 64-key tiles whose first key lies in this run start their row look-up here
                int32_t *tr = tile_run + ((size_t)h * Cq + i) * key_tiles;
                for (int t = (before + ATT_BN - 1) / ATT_BN; t * ATT_BN < before + len && t < key_tiles; ++t) tr[t] = idx - e0;
            }
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

// order[0 .. all tiles): the work items sorted by decreasing number of key tiles (longest first), so that the
// last workgroups of a launch are short ones.  The tiles of one query cluster stay together (they read the
// same keys); among clusters of equal length the order is whatever the atomics give -- it only decides when a
// work item runs, never what it computes.  One workgroup; with more clusters than ORD_MAX_CLUSTERS the list
// keeps its head-major order.
static constexpr int ORD_BUCKETS = 2048;
static constexpr int ORD_MAX_CLUSTERS = 1 << 20;

__global__ __launch_bounds__(1024) void attn_order_kernel(const int32_t *__restrict__ offsets_q,
                                                          const int32_t *__restrict__ tile_base,
                                                          const int32_t *__restrict__ row_keys,
                                                          const int32_t *__restrict__ cl_first, int H, int Cq, int BM,
                                                          int32_t *__restrict__ order)
{
    __shared__ int32_t s_cnt[ORD_BUCKETS];
    __shared__ int32_t s_part[1024];
    const int tid = threadIdx.x;
    const long long ncl = (long long)H * Cq;
    if (ncl > ORD_MAX_CLUSTERS) {
        const int total = tile_base[H];
        for (int v = tid; v < total; v += 1024) order[v] = v;
        return;
    }
    for (int b = tid; b < ORD_BUCKETS; b += 1024) s_cnt[b] = 0;
    __syncthreads();
    auto bucket_of = [&](int i) {               // longest first: bucket 0 holds the clusters with the most key tiles
        const int kt = (row_keys[i] + ATT_BN - 1) / ATT_BN;
        return ORD_BUCKETS - 1 - min(kt, ORD_BUCKETS - 1);
    };
    auto tiles_of = [&](int i) {
        const int h = i / Cq, c = i - h * Cq;
        const int32_t *oq = offsets_q + (size_t)h * (Cq + 1);
        return (oq[c + 1] - oq[c] + BM - 1) / BM;
    };
    for (int i = tid; i < (int)ncl; i += 1024) {
        const int nt = tiles_of(i);
        if (nt > 0) atomicAdd(&s_cnt[bucket_of(i)], nt);
    }
    __syncthreads();
    // exclusive scan over the buckets: two per thread
    const int a0 = s_cnt[2 * tid], a1 = s_cnt[2 * tid + 1];
    s_part[tid] = a0 + a1;
    __syncthreads();
    for (int o = 1; o < 1024; o <<= 1) {
        const int v = (tid >= o) ? s_part[tid - o] : 0;
        __syncthreads();
        s_part[tid] += v;
        __syncthreads();
    }
    const int excl = s_part[tid] - (a0 + a1);
    s_cnt[2 * tid] = excl;
    s_cnt[2 * tid + 1] = excl + a0;
    __syncthreads();
    for (int i = tid; i < (int)ncl; i += 1024) {
        const int nt = tiles_of(i);
        if (nt > 0) {
            const int h = i / Cq;
            const int pos = atomicAdd(&s_cnt[bucket_of(i)], nt);
            const int v0 = tile_base[h] + cl_first[i];
            for (int t = 0; t < nt; ++t) order[pos + t] = v0 + t;
        }
    }
}

// ---------------------------------------------------------------- bf16 MFMA kernel

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

// RUN_CAP: the launch was sized for at most ATT_RUN_LDS runs in LDS (more than that many key clusters); a work item
// with more runs then reads them from global memory.  Without it the table always fits and that path does not exist.
template <int D, bool RUN_CAP>
__global__ __launch_bounds__(64 * ATT_NW, 8 / ATT_NW) void attn_bf16_kernel(
    const bf16_t *__restrict__ Q, const bf16_t *__restrict__ K, const bf16_t *__restrict__ V, int H, int N, int Cq,
    int Ck, const int32_t *__restrict__ row_ptr, const int32_t *__restrict__ perm_q,
    const int32_t *__restrict__ perm_k, const int4 *__restrict__ tiles, const int32_t *__restrict__ tile_base,
    const int32_t *__restrict__ order, int max_tiles,
    const int2 *__restrict__ runs, const int32_t *__restrict__ row_keys, const int32_t *__restrict__ tile_run,
    int key_tiles, float scale_log2, int group, bf16_t *__restrict__ O, float *__restrict__ lse)
{
    constexpr int KS = D / 16;                 // k-steps of QK^T
    constexpr int DVB = D / 32;                // 32-row blocks of O^T
    constexpr int RB = 2 * D;                  // bytes per K / V row
    constexpr int CPR = D / 8;                 // 16-byte chunks per row
    constexpr int RPI = 1024 / RB;             // rows one direct-to-LDS load instruction fills (64 lanes x 16 B)
    constexpr int NW = ATT_NW, NSTG = ATT_NSTG;
    constexpr int NPASS = ATT_BN / (NW * RPI); // such instructions per wavefront, tile and tensor
    static_assert(NPASS >= 1, "a tile needs at least one load instruction per wavefront");
    constexpr int TILE_B = ATT_BN * RB;        // bytes of one K or V tile in LDS

    // LDS: K tiles [NSTG][64][D] and V tiles [NSTG][64][D], rows unpadded (the direct loads
    // fill 1024 contiguous bytes per instruction); bank conflicts are avoided by
    // storing 16-byte chunk c of row r at position c ^ swz(r):
    //   K  swz = (r / (256 / RB)) % CPR        the 16 rows of one ds_read_b128 pass differ
    //   V  swz = 4 * ((r / (256 / RB)) % (CPR / 4))   the 4 rows of one transposing pass differ
    extern __shared__ __align__(16) unsigned char s_raw[];
    unsigned char *sK = s_raw;                                      // [NSTG][TILE_B]
    unsigned char *sV = s_raw + NSTG * TILE_B;                      // [NSTG][TILE_B]
    int32_t *s_rows = reinterpret_cast<int32_t *>(s_raw + 2 * NSTG * TILE_B);   // [2][64]
    int2 *s_run = reinterpret_cast<int2 *>(s_rows + 2 * ATT_BN);    // [nnz + 1]

    // ---- which work item.  All tiles of all heads form one list (head-major, so
    // neighbours share keys).  Consecutive workgroup ids go round-robin over the 8
    // XCDs, each with its own L2: hand out the list in groups of ATT_GROUP
    // consecutive tiles per XCD, so tiles that share keys share an L2 and every XCD
    // gets the same amount of work whatever the per-head densities are.
    const int xcd = blockIdx.x % 8, slot = blockIdx.x / 8;
    const int pos = (slot / group) * (8 * group) + xcd * group + slot % group;
    if (pos >= tile_base[H]) return;
    const int v = order[pos];                   // longest work items first (attn_order_kernel)
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
    const int32_t *trh = tile_run + ((size_t)h * Cq + ci) * key_tiles;      // run in which each key tile starts
    // The run table of the work item (nnz entries + a closing one) is staged in LDS when it fits the share of LDS
    // that still lets two workgroups run on a CU; a query cluster that selects more key clusters than that reads
    // its runs from global memory (slow look-ups, same result).
    const bool runs_in_lds = !RUN_CAP || nnz + 1 <= ATT_RUN_LDS;
    if (runs_in_lds) {
        for (int e = tid; e < nnz; e += 64 * NW) s_run[e] = rn[e];
        if (tid == 0) s_run[nnz] = make_int2(0, L);
    }
    auto run_at = [&](int c) -> int2 {
        if (!RUN_CAP || runs_in_lds) return s_run[c];
        return c < nnz ? rn[c] : make_int2(0, L);
    };

    const bf16_t *Qh = Q + (size_t)h * N * D;
    const bf16_t *Kh = K + (size_t)h * N * D;
    const bf16_t *Vh = V + (size_t)h * N * D;

    // ---- queries as the B operand of S^T = K Q^T: this wavefront owns 32 rows of the tile
    bf16x8 qreg[KS];
    {
        int r = row0 + min(nrows - 1, wave * 32 + col);
        if (perm_k) r = perm_q[(size_t)h * N + r];      // gather-free: Q is in token order
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
    // ONE wavefront (wave kt % NW, lane = slot) ahead of time and parked in s_rows.  The
    // rows then go from global memory straight into LDS (no staging registers): load
    // instruction (wave, p) fills LDS rows (NW p + wave) * RPI .. + RPI of the tile, lane l
    // the chunk position l % CPR of row l / CPR, so it fetches the global chunk that the
    // swizzle puts there.  K tiles are fetched two tiles ahead of their use and V tiles
    // one tile ahead (see the schedule below), so the byte offsets of a tile's rows are
    // kept in registers from its K fetch to its V fetch.
    const char *Kb = reinterpret_cast<const char *>(Kh);
    const char *Vb = reinterpret_cast<const char *>(Vh);
    const int32_t *pkh = perm_k ? perm_k + (size_t)h * N : nullptr;
    int cur = 0;                                // per-lane cursor into the run table, only moves forward
    int lk_hint = -1;                           // run in which the tile looked up next starts (-1: not known)
    const int ld_row = lane / CPR;                                  // row inside the instruction's group
    const int ld_swz = ((wave * RPI + ld_row) / (256 / RB));
    const unsigned ld_koff = (unsigned)(((lane % CPR) ^ (ld_swz % CPR)) * 16);
    const unsigned ld_voff = (unsigned)(((lane % CPR) ^ (4 * (ld_swz % (CPR / 4)))) * 16);
    __syncthreads();                            // s_run visible

#define ATT_ROWS(KT)                                                                       \
    if (wave == ((KT) & (NW - 1))) {                                                       \
        const int kk = (KT) * ATT_BN + lane;                                               \
        int row_ = 0;                                                                      \
        if (kk < L) {                                                                      \
            while (kk >= run_at(cur + 1).y) ++cur;                                         \
            const int2 rs_ = run_at(cur);                                                  \
            row_ = rs_.x + kk - rs_.y;                                                     \
        }                                                                                  \
        if (perm_k) {                           /* gather-free: sorted row -> token */     \
            row_ = pkh[row_];                                                              \
            asm volatile("" : "+v"(row_));      /* the wait for this load stays inside the branch */ \
        }                                                                                  \
        s_rows[((KT) & 1) * ATT_BN + lane] = row_ * RB;     /* byte offset of the row */   \
    }
// second and third step of the look-up of a tile's rows (first step: lk_rs_ = s_run[cur], lk_nb_ = start of the next run)
#define ATT_LOOKUP_FINISH(KT)                                                              \
    {                                                                                      \
        const int kk = (KT) * ATT_BN + lane;                                               \
        if (kk < L) {                                                                      \
            while (kk >= lk_nb_) {                                                         \
                ++cur;                                                                     \
                lk_rs_ = run_at(cur);                                                      \
                lk_nb_ = run_at(cur + 1).y;                                                \
            }                                                                              \
            lk_row_ = lk_rs_.x + kk - lk_rs_.y;                                            \
        }                                                                                  \
        if (perm_k) lk_row_ = pkh[lk_row_];     /* gather-free: sorted row -> token */     \
    }
#define ATT_LOOKUP_STORE(KT)                                                               \
    {                                                                                      \
        asm volatile("" : "+v"(lk_row_));       /* the value is first touched here, so the wait for it comes here */ \
        s_rows[((KT) & 1) * ATT_BN + lane] = lk_row_ * RB;                                 \
    }
#define ATT_OFFS(KT, OFF)                                                                  \
    _Pragma("unroll") for (int p_ = 0; p_ < NPASS; ++p_)                                   \
        OFF[p_] = (unsigned)s_rows[((KT) & 1) * ATT_BN + (NW * p_ + wave) * RPI + ld_row];
#define ATT_FETCH(OFF, SRC, LOFF, DST)                                                     \
    _Pragma("unroll") for (int p_ = 0; p_ < NPASS; ++p_)                                   \
        load_to_lds_16(SRC, OFF[p_] + LOFF, DST + ((NW * p_ + wave) * RPI) * RB);

// one load instruction (pass P) of a tile: DSTB = byte offset of the tile's buffer in LDS
#define ATT_FETCH1(P, OFF, SRC, LOFF, DSTB)                                                \
    load_to_lds_16(SRC, OFF[P] + LOFF, s_raw + (DSTB) + ((NW * (P) + wave) * RPI) * RB);

    const int ntile = (L + ATT_BN - 1) / ATT_BN;
    unsigned off_nx[NPASS];                     // row offsets of the tile whose V is fetched next
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
    if (ntile > 3 && 3 < key_tiles && wave == (3 & (NW - 1))) lk_hint = trh[3];      // tile 3 is looked up during tile 0
    // off_nx stays live: it holds the rows of tile 1, whose V is requested during tile 0
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
        // fold the address of the LDS buffer in once and make the sums opaque: otherwise the compiler re-adds the
        // (link-time constant) base in front of every LDS read
        const int lds_base = (int)(unsigned)(size_t)(const lds_u8 *)s_raw;
#pragma unroll
        for (int s = 0; s < KS; ++s) { koff[s] += lds_base; asm volatile("" : "+v"(koff[s])); }
#pragma unroll
        for (int b = 0; b < DVB; ++b) { voff[b] += lds_base; asm volatile("" : "+v"(voff[b])); }
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);         // vmcnt(0): queries and the first tiles have landed
    __syncthreads();

    // ---- schedule.  The key sequence is consumed in blocks of 32 keys (two per 64-key
    // tile).  Per block j the work is S_j = K_j Q^T (KS matrix instructions), the running
    // maximum, P_j = exp2(S_j - m) (vector ALU, 6 operations per pair of scores: two fma,
    // two exp2, one pack to bf16, one row-sum dot) and O^T += V_j^T P_j^T (NPV matrix
    // instructions).  The blocks are software-pipelined so that every matrix instruction
    // has about the same amount of independent vector work in its shadow:
    //
    //   phase A(j):  S_{j+1} = K_{j+1} Q^T   ||  last two thirds of P_j, LDS reads of V_j^T
    //   phase B(j):  O^T += V_j^T P_j^T      ||  maximum of S_{j+1} and the decision about the
    //                                            running maximum (first half), first third of
    //                                            P_{j+1} (second half), LDS reads of K_{j+2}
    //
    // The instruction stream is laid out by hand (ATT_FENCE keeps the compiler from moving
    // code across chunk boundaries).  The running maximum only moves when it would grow by
    // more than 2^8 (probabilities stay below 256), so rescaling the output accumulators is
    // rare; it is applied at the end of phase B, when block j has been accumulated under the
    // old maximum.  Accumulator i of a block is key 8 (i/4) + 4 half + i%4.
    //
    // Tile t lives in K buffer t % 2 and V buffer t % 2.  One barrier per tile: at the top of
    // tile t every wavefront has finished tile t - 1 and all fetches issued during tile t - 1
    // have landed.  V_{t+1} and K_{t+2} are requested during tile t (K is read one and a half
    // blocks ahead of V, so it is fetched a tile earlier): the V loads one by one after every
    // other matrix instruction of the first phase A, the K loads likewise in the first phase B.
    // Issued in one burst at the top of the tile, the load instructions of all wavefronts of a
    // CU queue up behind each other (a CU accepts one 1 KB load per ~17 cycles) while no matrix
    // instruction is in flight.  The rows of tile t + 3 are looked up by one wavefront in three
    // steps between the phases (request the run, resolve it, park the row offsets in s_rows), so
    // that neither the LDS latency nor the latency of the gathered index is waited for.
#define ATT_FENCE __builtin_amdgcn_sched_barrier(0);
// An empty volatile asm that "modifies" a value: the value has to exist at this point of the
// program, so optimisation passes that work above the instruction scheduler cannot sink the
// vector work out of the chunk it was written in.
#define ATT_PIN(X) asm volatile("" : "+v"(X));
    constexpr int NPV = 2 * DVB;
    constexpr int NOPS = 48;                    // vector operations of one block's probabilities
    constexpr int OPS_B = ATT_OPS_B;            // of which phase B (of the block before) does the first OPS_B
    const lds_u8 *lds = (const lds_u8 *)0;      // koff / voff are complete LDS addresses
    f32x16 s0, s1;                              // scores of block 0 / block 1 of a tile
    unsigned pw0[8], pw1[8];                    // probabilities of block 0 / block 1, two bf16 per word
    bf16x8 ka[KS], va[NPV];                     // K operands of the next score block, V^T operands of this one
    float psum = 0.f, m_acc = 0.f, t0 = 0.f, t1 = 0.f;    // m_acc: the maximum the accumulators are expressed under
    bool any_upd = false;

    // operation `op` (0..47) of the probabilities of one block: S -> pw
    auto exp_op = [&](const f32x16 &S, unsigned *pw, int op) {
        const int e = op / 6, k = op % 6;
        if (k == 0) { t0 = fmaf(S[2 * e], scale_log2, -m_run); ATT_PIN(t0) }
        else if (k == 1) { t1 = fmaf(S[2 * e + 1], scale_log2, -m_run); ATT_PIN(t1) }
        else if (k == 2) { t0 = __builtin_amdgcn_exp2f(t0); ATT_PIN(t0) }
        else if (k == 3) { t1 = __builtin_amdgcn_exp2f(t1); ATT_PIN(t1) }
        else if (k == 4) { pw[e] = pack_bf16x2(t0, t1); ATT_PIN(pw[e]) }
        else { psum = add_bf16x2(pw[e], psum); ATT_PIN(psum) }
    };
    auto mask_block = [&](f32x16 &S, int base, int rem) {
#pragma unroll
        for (int i = 0; i < 16; ++i)
            if (base + 8 * (i >> 2) + 4 * half + (i & 3) >= rem) S[i] = -INFINITY;
    };
    // the decision about the running maximum, given the maximum mx of a new score block
    auto decide = [&](float mx) {
        const float mx_s = max_xor32(mx) * scale_log2;
        const bool upd = mx_s > m_run + 8.0f;
        any_upd = __any(upd);
        m_run = upd ? mx_s : m_run;
        ATT_PIN(m_run)
        psum = 0.f;
    };
    // K operands of a score block: KBYTE = byte offset of the block's first row in LDS
    auto load_k = [&](auto kbyte_tag, int s) {
        constexpr int KBYTE = decltype(kbyte_tag)::value;
        const u32x4 w = lds_read_b128((lds + koff[s]) + KBYTE);
        __builtin_memcpy(&ka[s], &w, 16);
    };
    // V^T operand idx of a block (ks = idx / DVB: 16 keys, b = idx % DVB: 32 output columns)
    auto load_v = [&](auto vbyte_tag, int idx) {
        constexpr int VBYTE = decltype(vbyte_tag)::value;
        const int ks = idx / DVB, b = idx % DVB;
        const s16x4 lo = lds_read_tr16((lds + voff[b]) + (VBYTE + (ks * 16) * RB));
        const s16x4 hi = lds_read_tr16((lds + voff[b]) + (VBYTE + (ks * 16 + 8) * RB));
        __builtin_memcpy(&va[idx], &lo, 8);
        __builtin_memcpy(reinterpret_cast<char *>(&va[idx]) + 8, &hi, 8);
    };
    // phase A: Sacc = K Q^T from ka[] (if DO_S)  ||  operations 16..47 of pw = exp2(Sexp - m), V^T operands from VBYTE
    auto phase_a = [&](auto do_s_tag, auto vbyte_tag, auto vfetch_tag, f32x16 &Sacc, const f32x16 &Sexp, unsigned *pw) {
        constexpr bool DO_S = decltype(do_s_tag)::value;
        constexpr int VFETCH = decltype(vfetch_tag)::value;     // >= 0: LDS byte offset of the V buffer to fill
        constexpr int KPF = KS / NPASS;                         // k-steps per load instruction
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            if (DO_S) {
                if (s == 0) {
#pragma unroll
                    for (int i = 0; i < 16; ++i) Sacc[i] = 0.f;
                }
                Sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[s], qreg[s], Sacc, 0, 0, 0);
            }
            ATT_FENCE
#pragma unroll
            for (int idx = (2 * NPV * s) / KS; idx < (2 * NPV * (s + 1)) / KS && idx < NPV; ++idx)
                load_v(vbyte_tag, idx);         // all issued in the first half, so they have landed by phase B
#pragma unroll
            for (int op = OPS_B + ((NOPS - OPS_B) * s) / KS; op < OPS_B + ((NOPS - OPS_B) * (s + 1)) / KS; ++op)
                exp_op(Sexp, pw, op);
            if constexpr (VFETCH >= 0) {
                if (s % KPF == KPF - 1) { ATT_FETCH1(s / KPF, off_nx, Vb, ld_voff, VFETCH) }
            }
            ATT_FENCE
        }
        l_run += psum;
    };
    // phase B: O^T += V^T P^T from va[] and pr[]  ||  maximum of Snext and the decision, then operations
    // 0..15 of pn = exp2(Snext - m) (if DO_MAX); K operands of the block after Snext from KBYTE (if DO_K)
    auto phase_b = [&](auto do_max_tag, auto do_k_tag, auto kbyte_tag, auto kfetch_tag, auto slot_tag, bool do_kfetch,
                       const unsigned *pr, const f32x16 &Snext, unsigned *pn) {
        constexpr bool DO_MAX = decltype(do_max_tag)::value;
        constexpr bool DO_K = decltype(do_k_tag)::value;
        constexpr int KFETCH = decltype(kfetch_tag)::value;     // >= 0: LDS byte offset of the K buffer to fill
        constexpr int SLOT = decltype(slot_tag)::value;         // which half of s_rows holds that tile's rows
        constexpr int KF0 = NPV / 4;                            // first matrix instruction followed by a load
        constexpr int HB = NPV / 2;
        float mx = -INFINITY;
#pragma unroll
        for (int idx = 0; idx < NPV; ++idx) {
            bf16x8 pb;
            __builtin_memcpy(&pb, pr + 4 * (idx / DVB), 16);
            oacc[idx % DVB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[idx], pb, oacc[idx % DVB], 0, 0, 0);
            ATT_FENCE
            if (DO_K) {
#pragma unroll
                for (int s = (KS * idx) / NPV; s < (KS * (idx + 1)) / NPV; ++s) load_k(kbyte_tag, s);
            }
            if (DO_MAX && idx < HB) {
#pragma unroll
                for (int c = (8 * idx) / HB; c < (8 * (idx + 1)) / HB; ++c) {
                    // the first read of the new scores is an ordinary fmaxf, so that the compiler puts the wait
                    // states between the matrix instructions and the vector read; the other reads come later
                    if (c == 0) mx = max2_raw(fmaxf(Snext[0], Snext[1]), Snext[2]);
                    else if (c < 7) mx = max3_raw(mx, Snext[2 * c + 1], Snext[2 * c + 2]);
                    else mx = max2_raw(mx, Snext[15]);
                    ATT_PIN(mx)
                }
                if (idx == HB - 1) decide(mx);
            }
            if (DO_MAX && idx >= HB) {
#pragma unroll
                for (int op = (OPS_B * (idx - HB)) / HB; op < (OPS_B * (idx - HB + 1)) / HB; ++op)
                    exp_op(Snext, pn, op);
            }
            if constexpr (KFETCH >= 0) {
                if (do_kfetch) {
                    if (idx == 0) {
#pragma unroll
                        for (int p_ = 0; p_ < NPASS; ++p_)
                            off_nx[p_] = (unsigned)s_rows[SLOT * ATT_BN + (NW * p_ + wave) * RPI + ld_row];
                    }
                    if (idx >= KF0 && idx < KF0 + NPASS) { ATT_FETCH1(idx - KF0, off_nx, Kb, ld_koff, KFETCH) }
                }
            }
            ATT_FENCE
        }
        if (DO_MAX && any_upd) {            // rare: the factor is only formed here
            const float alpha = __builtin_amdgcn_exp2f(m_acc - m_run);
            m_acc = m_run;
            l_run *= alpha;
#pragma unroll
            for (int b = 0; b < DVB; ++b)
#pragma unroll
                for (int i = 0; i < 16; ++i) oacc[b][i] *= alpha;
        }
    };
    using T = std::true_type;
    using F = std::false_type;

    // ---- prologue: S of block 0 of tile 0, its maximum, the first third of its probabilities,
    // K operands of block 1
    if (wave_active && ntile > 0) {
#pragma unroll
        for (int s = 0; s < KS; ++s) load_k(std::integral_constant<int, 0>{}, s);
#pragma unroll
        for (int i = 0; i < 16; ++i) s0[i] = 0.f;
#pragma unroll
        for (int s = 0; s < KS; ++s) s0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[s], qreg[s], s0, 0, 0, 0);
#pragma unroll
        for (int s = 0; s < KS; ++s) load_k(std::integral_constant<int, 32 * RB>{}, s);
        if (L < 32) mask_block(s0, 0, L);
        float mx = fmaxf(fmaxf(s0[0], s0[1]), s0[2]);
#pragma unroll
        for (int i = 3; i < 16; ++i) mx = fmaxf(mx, s0[i]);
        decide(mx);                             // key 0 exists, so the maximum is finite; nothing to rescale yet
        m_acc = m_run;
#pragma unroll
        for (int op = 0; op < OPS_B; ++op) exp_op(s0, pw0, op);
    }

    // One tile: tile kt sits in K / V buffer BUF = kt % NSTG.  HAS_NEXT: tile kt + 1 exists.
    // At the top, the fetches issued during the tile before (V of this tile, K of the next) must
    // have landed.
#define ATT_TILE(BUF, HAS_NEXT)                                                            \
    {                                                                                      \
        __builtin_amdgcn_s_waitcnt(0x0F70);     /* vmcnt(0) */                             \
        __syncthreads();                                                                   \
        /* fetches of this tile: V of the next tile (it exists: HAS_NEXT) into the other V buffer, K of the  \
           tile after it into this tile's K buffer; spread over the first two phases so that the load        \
           instructions of the wavefronts of a CU do not queue up behind each other at the top of a tile */  \
        constexpr int VF_ = HAS_NEXT ? NSTG * TILE_B + ((BUF + 1) % NSTG) * TILE_B : -1;   \
        constexpr int KF_ = HAS_NEXT ? BUF * TILE_B : -1;                                  \
        const bool do_kf_ = HAS_NEXT && kt + NSTG < ntile;                                 \
        /* rows of tile kt + 3 (needed by the K fetch of the next tile): one wavefront looks them up, in   \
           three steps between the phases so that the LDS and memory latencies are not waited for */     \
        const bool lk_ = HAS_NEXT && kt + NSTG + 1 < ntile && wave == ((kt + NSTG + 1) & (NW - 1)); \
        int2 lk_rs_ = make_int2(0, 0);                                                     \
        int lk_nb_ = 0, lk_row_ = 0;                                                       \
        if (lk_) {                                                                         \
            cur = max(cur, lk_hint);            /* start at the tile's first run, not where this lane was 4 tiles ago */ \
            lk_rs_ = run_at(cur);                                                          \
            lk_nb_ = run_at(cur + 1).y;                                                    \
        }                                                                                  \
        if (wave_active) {                                                                 \
            using HN = std::integral_constant<bool, HAS_NEXT>;                             \
            constexpr int KB_ = ((BUF + 1) % NSTG) * TILE_B, VB_ = NSTG * TILE_B + BUF * TILE_B; \
            phase_a(T{}, std::integral_constant<int, VB_>{}, std::integral_constant<int, VF_>{}, s1, s0, pw0); \
            if (!HAS_NEXT) mask_block(s1, 32, L - kt * ATT_BN);                            \
            if (lk_) { ATT_LOOKUP_FINISH(kt + NSTG + 1) }                                  \
            phase_b(T{}, HN{}, std::integral_constant<int, KB_>{}, std::integral_constant<int, KF_>{}, \
                    std::integral_constant<int, BUF>{}, do_kf_, pw0, s1, pw1);             \
            phase_a(HN{}, std::integral_constant<int, VB_ + 32 * RB>{}, std::integral_constant<int, -1>{}, s0, s1, pw1); \
            if (HAS_NEXT && kt + 2 == ntile && L - (kt + 1) * ATT_BN < 32)                 \
                mask_block(s0, 0, L - (kt + 1) * ATT_BN);                                  \
            phase_b(HN{}, HN{}, std::integral_constant<int, KB_ + 32 * RB>{}, std::integral_constant<int, -1>{}, \
                    std::integral_constant<int, 0>{}, false, pw1, s0, pw0);                \
            /* stored at the end of the tile: the wait for the gathered index (all loads: the compiler  \
               does not know which are outstanding) then falls together with the one at the top */      \
            if (lk_) { ATT_LOOKUP_STORE(kt + NSTG + 1) }                                   \
        } else if (HAS_NEXT) {      /* a wavefront without query rows still loads its share of the tiles */ \
            ATT_FETCH(off_nx, Vb, ld_voff, sV + ((BUF + NSTG - 1) % NSTG) * TILE_B)        \
            if (do_kf_) {                                                                  \
                ATT_OFFS(kt + NSTG, off_nx)                                                \
                ATT_FETCH(off_nx, Kb, ld_koff, sK + BUF * TILE_B)                          \
            }                                                                              \
            if (lk_) {                                                                     \
                ATT_LOOKUP_FINISH(kt + NSTG + 1)                                           \
                ATT_LOOKUP_STORE(kt + NSTG + 1)                                            \
            }                                                                              \
        }                                                                                  \
        /* where the tile that the next tile looks up starts (from the plan, global memory): requested here, \
           used behind the wait at the top of the next tile */                                              \
        {                                                                                  \
            const int tn_ = kt + NSTG + 2;                                                 \
            lk_hint = -1;                                                                  \
            if (HAS_NEXT && tn_ < ntile && tn_ < key_tiles && wave == (tn_ & (NW - 1))) lk_hint = trh[tn_]; \
        }                                                                                  \
        ++kt;                                                                              \
    }
    static_assert(NSTG == 2, "the fetch schedule below is written for two buffers");
    int kt = 0;
    while (kt < ntile - 1) {                    // every tile but the last
        ATT_TILE(0, true)
        if (kt >= ntile - 1) break;
        ATT_TILE(1, true)
    }
    if (ntile > 0) {                            // the last tile: nothing follows it, maybe ragged
        if (kt % NSTG == 0) ATT_TILE(0, false)
        else ATT_TILE(1, false)
    }
#undef ATT_TILE
#undef ATT_FENCE
#undef ATT_PIN
#undef ATT_ROWS
#undef ATT_OFFS
#undef ATT_LOOKUP_FINISH
#undef ATT_LOOKUP_STORE
#undef ATT_FETCH
#undef ATT_FETCH1

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
    const int32_t *__restrict__ row_ptr, const int32_t *__restrict__ perm_q, const int32_t *__restrict__ perm_k,
    const int4 *__restrict__ tiles, const int32_t *__restrict__ n_tiles, int max_tiles,
    const int2 *__restrict__ runs, const int32_t *__restrict__ row_keys, float scale, float *__restrict__ O,
    float *__restrict__ lse)
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
    const int qr = perm_k ? perm_q[(size_t)h * N + r] : r;      // gather-free: Q is in token order
    float q[D], o[D];
#pragma unroll
    for (int k = 0; k < D / 4; ++k) {
        const float4 w = reinterpret_cast<const float4 *>(Q + ((size_t)h * N + qr) * D)[k];
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
            size_t src = (size_t)(rs.x + kk - rs.y);
            if (perm_k) src = (size_t)perm_k[(size_t)h * N + src];  // gather-free: sorted row -> token
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

size_t attn_ws_bytes(int dtype, int H, int N, int d, int Cq, int Ck)
{
    (void)d;
    return attn_carve(nullptr, dtype, H, N, Cq, Ck).bytes;
}

static size_t attn_lds_bytes(int d, int Ck)
{
    return (size_t)2 * ATT_NSTG * ATT_BN * d * sizeof(bf16_t) + 2 * ATT_BN * sizeof(int32_t) +
           (size_t)std::min(Ck + 1, ATT_RUN_LDS) * sizeof(int2);
}

int attn_prepare(int dtype, int d)
{
    if (dtype != SVG2_BF16) return SVG2_OK;
    const size_t lds = attn_lds_bytes(d, SVG2_MAX_CLUSTERS);
    if (d == 128) {
        SVG2_TRY(set_dynamic_lds(reinterpret_cast<const void *>(attn_bf16_kernel<128, true>), lds));
        SVG2_TRY(set_dynamic_lds(reinterpret_cast<const void *>(attn_bf16_kernel<128, false>), lds));
    } else {
        SVG2_TRY(set_dynamic_lds(reinterpret_cast<const void *>(attn_bf16_kernel<64, true>), lds));
        SVG2_TRY(set_dynamic_lds(reinterpret_cast<const void *>(attn_bf16_kernel<64, false>), lds));
    }
    return SVG2_OK;
}

int attn_plan_launch(int dtype, int H, int N, int Cq, int Ck, const int32_t *offsets_q, const int32_t *offsets_k,
                     const int32_t *row_ptr, const int32_t *col_idx, void *ws, hipStream_t st)
{
    const AttnWs a = attn_carve(ws, dtype, H, N, Cq, Ck);
    hipLaunchKernelGGL(attn_plan_kernel, dim3(H), dim3(256), 0, st, offsets_q, offsets_k, row_ptr, col_idx, Cq, Ck,
                       attn_bm(dtype), a.max_tiles, a.tiles, a.n_tiles, a.runs, a.row_keys, a.cl_first, a.key_tiles,
                       a.tile_run);
    hipLaunchKernelGGL(attn_tile_base_kernel, dim3(1), dim3(256), 0, st, a.n_tiles, H, a.tile_base);
    if (dtype == SVG2_BF16)                     // the fp32 kernel is launched on a (tile, head) grid and needs no list
        hipLaunchKernelGGL(attn_order_kernel, dim3(1), dim3(1024), 0, st, offsets_q, a.tile_base, a.row_keys,
                           a.cl_first, H, Cq, attn_bm(dtype), a.order);
    SVG2_HIP_CHECK(hipGetLastError());
    return SVG2_OK;
}

int attn_main_launch(const void *Qp, const void *Kp, const void *Vp, int dtype, int H, int N, int d, int Cq, int Ck,
                     const int32_t *row_ptr, const int32_t *perm_q, const int32_t *perm_k, float scale, void *O,
                     float *lse, void *ws, hipStream_t st)
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
        const size_t lds = attn_lds_bytes(d, Ck);
        const bool cap = Ck + 1 > ATT_RUN_LDS;
        auto kern = d == 128 ? (cap ? attn_bf16_kernel<128, true> : attn_bf16_kernel<128, false>)
                             : (cap ? attn_bf16_kernel<64, true> : attn_bf16_kernel<64, false>);
        hipLaunchKernelGGL(kern, dim3(nwg), dim3(64 * ATT_NW), lds, st, q, k, v, H, N, Cq, Ck, row_ptr, perm_q, perm_k, tiles,
                           tile_base, a.order, max_tiles, runs, row_keys, a.tile_run, a.key_tiles, scale_log2, group, o, lse);
    } else {
        const float *q = static_cast<const float *>(Qp), *k = static_cast<const float *>(Kp),
                    *v = static_cast<const float *>(Vp);
        float *o = static_cast<float *>(O);
        if (d == 128)
            hipLaunchKernelGGL(attn_f32_kernel<128>, dim3(max_tiles, H), dim3(64), 0, st, q, k, v, N, Cq, Ck, row_ptr,
                               perm_q, perm_k, tiles, n_tiles, max_tiles, runs, row_keys, scale, o, lse);
        else
            hipLaunchKernelGGL(attn_f32_kernel<64>, dim3(max_tiles, H), dim3(64), 0, st, q, k, v, N, Cq, Ck, row_ptr,
                               perm_q, perm_k, tiles, n_tiles, max_tiles, runs, row_keys, scale, o, lse);
    }
    SVG2_HIP_CHECK(hipGetLastError());
    return SVG2_OK;
}

int attn_launch(const void *Qp, const void *Kp, const void *Vp, int dtype, int H, int N, int d, int Cq, int Ck,
                const int32_t *offsets_q, const int32_t *offsets_k, const int32_t *row_ptr,
                const int32_t *col_idx, const int32_t *perm_q, const int32_t *perm_k, float scale, void *O,
                float *lse, void *ws, hipStream_t st)
{
    const int rc = attn_plan_launch(dtype, H, N, Cq, Ck, offsets_q, offsets_k, row_ptr, col_idx, ws, st);
    if (rc != SVG2_OK) return rc;
    return attn_main_launch(Qp, Kp, Vp, dtype, H, N, d, Cq, Ck, row_ptr, perm_q, perm_k, scale, O, lse, ws, st);
}

}  // namespace svg2
