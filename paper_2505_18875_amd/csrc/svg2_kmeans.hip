// Per-head Lloyd k-means (paper Section 4.1), batched over heads and over the two sides of a layer (the Q tokens
// and the K tokens are clustered independently, Section 4.1; every kernel here takes both problems in one launch).
//
// One iteration = assign, settle near-ties, update:
//   assign    token x centroid contraction with a fused argmax.
//             bf16 input: MFMA 32x32x16 bf16 with the centroid tile as the A operand (rows) and the tokens as
//             the B operand (columns), so a lane's 16 accumulators are 16 centroids of ONE token.  The
//             accumulators start at -||c||^2 / 2, so argmin ||c||^2 - 2 x.c is the argmax of the accumulator.
//             Each accumulator gets its position written into its 4 lowest mantissa bits; the largest and the
//             second largest of these keys are tracked per token (max3 / med3 trees, no compare-and-select
//             chains), which gives the label and the gap to the runner-up.
//             fp32 input: a plain FMA kernel (one token per thread).
//   settle    (bf16) every token whose gap is within the error bound of the fp32 contraction is assigned
//             again in double precision, over all centroids, lowest index winning an exact tie.  Products of
//             two bf16 numbers are exact and their sums fit a double, so these labels are THE argmin of the
//             definition, not an approximation of it; a fraction of a per cent of the tokens take this path.
//   update    segmented sum over the label-sorted token order (counting sort, shared with the permutation
//             stage), in double precision: sums of bf16 values are exact in a double, so the cluster sums do
//             not depend on the order of the additions -- reproducible bit for bit, independent of how skewed
//             the cluster sizes are, and the delta update below never drifts.  From the second iteration on
//             only the tokens whose label changed are moved between the cluster sums.
//   finalize  mean = sum / count in double (an empty cluster keeps its centroid), the fp32 centroid that is
//             handed back, the bf16 copy the next assign reads (rounded from the DOUBLE mean, so it is the
//             correctly rounded bf16 of the mean), and ||c||^2 of that copy.
//
// For bf16 input the assign step sees the centroids rounded to bf16 (both in x.c and in ||c||^2); the
// centroids handed back stay fp32 means.
#include <algorithm>
#include <atomic>
#include <type_traits>

#include "svg2_common.h"

namespace svg2 {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(16))) float f32x16;

static constexpr int KM_CMAX = 512;    // centroids resident in LDS at a time (bf16 kernel)
static constexpr int KM_NW = 8;        // wavefronts per workgroup (bf16 kernel)
static constexpr int KM_TB = 2;        // 32-token blocks per wavefront (bf16 kernel)
static constexpr int KM_WG_TOKENS = KM_NW * KM_TB * 32;
static constexpr int KM_UB = 4;        // load instructions in flight per wavefront in the segmented sum
static constexpr int KM_SEG = 256;     // rows per piece of the segmented sum
static constexpr int KM_FULL_EVERY = 16; // iterations between updates that sum every cluster afresh (the others move the changed tokens)
static constexpr int KM_SETTLE_BLOCKS = 64;  // workgroups per head and side that walk the list of near-ties
// A token is settled in double precision when the gap between its two best keys is at most
//     KM_TIE_KEY * |best key|  +  KM_TIE_ACC * (||x||^2 / 2 + max_j ||c_j||^2).
// First term: the 4 mantissa bits given to the position move a key by less than 16 units in its last place,
// 2^-19 of its value; two keys of at most the best one's magnitude (the runner-up is within the gap of it).
// Second term: the fp32 accumulation of the contraction.  sum_k |x_k c_jk| + ||c_j||^2 / 2 is below the
// bracket; 8 chained matrix instructions with a few units in the last place of the partial sums each are taken
// to stay within 2^-21 of it per accumulator, two accumulators.  (An assumption about the matrix cores'
// internal rounding, which is not documented; the parity tests compare the labels of many heads with the
// double-precision definition and would show a violation as a label that differs away from a tie.)
static constexpr float KM_TIE_KEY = 3.814697265625e-06f;      // 2^-18
static constexpr float KM_TIE_ACC = 9.5367431640625e-07f;     // 2^-20
static constexpr float KM_PAD_HCN = -3.0e38f;   // -||c||^2 / 2 of the padding rows of a centroid block: never wins, stays finite

// One side of a k-means call: all heads of the Q tokens, or of the K tokens.
struct KmSide {
    const void *X;              // [H,N,d] tokens
    const float *init;          // [H,C,d]
    float *centroids;           // [H,C,d] out (may alias init)
    int32_t *labels;            // [H,N] out
    int32_t *counts;            // [H,C] out
    float *objective;           // [H,iters] or null
    int C;
    // workspace
    bf16_t *cb;                 // [H,C,d] centroids rounded to bf16 (bf16 input)
    bf16_t *cbT;                // [H,d/8,C,8] the same, 16-byte chunk-major: chunk q of consecutive centroids is contiguous
    float *hcn;                 // [H,C] -||c||^2 / 2 of the rounded centroids (bf16 input), ||c||^2 (fp32 input)
    double *cn64;               // [H,C] ||c||^2 of the rounded centroids
    double *cd;                 // [H,C,d] centroids in double (what an empty cluster keeps)
    double *csum;               // [H,C,d] cluster sums, kept between iterations
    float *best, *second;       // [H,N] running best / runner-up between centroid chunks (C > KM_CMAX only)
    int32_t *flag_cnt;          // [H] tokens to settle
    int32_t *flag_list;         // [H,N]
    int32_t *labels_alt;        // [H,N] the labels of consecutive iterations alternate between this and `labels`
    int32_t *hist;              // sort scratch
    // two sets of the label-sorted order and its pieces: iteration t uses set t % 2, so the previous
    // iteration's order is still there for the delta update
    int32_t *offsets[2], *perm[2], *first_piece[2], *n_pieces[2];
    int4 *pieces[2];
    double *psum[2];            // [H,max_pieces,d]
    int max_pieces;
};

struct KmArgs {
    KmSide s[2];
    int nsides, H, N, iters;
};

// labels written / read by iteration t
struct KmIter {
    int32_t *lab[2];
    const int32_t *lab_prev[2];
    int t, set;
};

// element `i` (0 or 1) of a two-element array inside a kernel argument: a select, so that the struct stays in
// scalar registers (indexing it with a run-time value would move it to scratch memory)
#define KM_SEL(arr, i) ((i) ? (arr)[1] : (arr)[0])

// v_max / v_min / v_max3 / v_med3 as they are (fmaxf and friends first canonicalise operands the compiler cannot
// prove quiet; the keys here are never NaN).  Not volatile: the scheduler may place them.
__device__ __forceinline__ float km_max(float a, float b)
{
    float r;
    asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}
__device__ __forceinline__ float km_min(float a, float b)
{
    float r;
    asm("v_min_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}
__device__ __forceinline__ float km_max3(float a, float b, float c)
{
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}
__device__ __forceinline__ float km_med3(float a, float b, float c)
{
    float r;
    asm("v_med3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

// the values lanes l and l + 32 hold of x: .x = the lower half's, .y = the upper half's, the same in both lanes (one
// vector instruction; a shuffle across the halves goes through the LDS crossbar and is waited for)
struct KmHalves { unsigned lo, hi; };
__device__ __forceinline__ KmHalves km_halves(unsigned x)
{
    const auto r = __builtin_amdgcn_permlane32_swap(x, x, false, false);
    return {r[0], r[1]};
}

// double -> bf16, round to nearest even, in ONE rounding: via float unless the float lands exactly on the midpoint
// of two bf16 values, where the side the double was on decides (and an exact midpoint goes to even).
__device__ __forceinline__ bf16_t f64_to_bf16(double m)
{
    const float f = (float)m;
    const unsigned u = __float_as_uint(f);
    if ((u & 0xFFFFu) != 0x8000u) return (bf16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
    const double fd = (double)f, am = fabs(m), af = fabs(fd);
    const bool up = am > af || (am == af && ((u >> 16) & 1u));
    return (bf16_t)((u >> 16) + (up ? 1u : 0u));
}

// ---------------------------------------------------------------- finalize
// grid (max C, H, sides), block d.  mode 0: centroids <- init (first call).  mode 1: cluster sum = sum of the
// cluster's pieces of set `set`.  mode 2 (delta update): cluster sum = previous cluster sum + the pieces of the
// tokens that joined the cluster (set `set`) - the pieces of the tokens that left it (the other set).  All sums
// are doubles of bf16 / fp32 values: exact, whatever the order.
template <bool BF16>
__global__ void kmeans_finalize_kernel(KmArgs a, int mode, int set)
{
    __shared__ double s_red[2];
    const KmSide S = blockIdx.z ? a.s[1] : a.s[0];
    const int j = blockIdx.x, h = blockIdx.y, k = threadIdx.x, C = S.C, d = blockDim.x;
    if (j >= C) return;
    if (j == 0 && k == 0) S.flag_cnt[h] = 0;           // the next assign step starts an empty list
    const size_t idx = ((size_t)h * C + j) * d + k;
    double c;
    if (mode != 0) {
        const int32_t *off = KM_SEL(S.offsets, set) + (size_t)h * (C + 1);
        const int cnt = off[j + 1] - off[j];
        const int32_t *fp = KM_SEL(S.first_piece, set) + (size_t)h * (C + 1);
        const int p0 = fp[j], p1 = fp[j + 1];
        const double *ps = KM_SEL(S.psum, set) + (size_t)h * S.max_pieces * d;
        double s = (mode == 2) ? S.csum[idx] : 0.0;
        // unrolled so that the loads of 8 pieces are in flight together: the largest cluster of a head has dozens
        // of pieces and its block decides how long the launch takes
#pragma unroll 8
        for (int q = p0; q < p1; ++q) s += ps[(size_t)q * d + k];
        if (mode == 2) {
            const int32_t *fo = KM_SEL(S.first_piece, 1 - set) + (size_t)h * (C + 1);
            const int o0 = fo[j], o1 = fo[j + 1];
            const double *po = KM_SEL(S.psum, 1 - set) + (size_t)h * S.max_pieces * d;
#pragma unroll 8
            for (int q = o0; q < o1; ++q) s -= po[(size_t)q * d + k];
        }
        if (cnt > 0) {
            c = s / (double)cnt;
        } else {
            s = 0.0;
            c = S.cd[idx];                              // an empty cluster keeps its centroid
        }
        S.csum[idx] = s;
        if (k == 0) S.counts[(size_t)h * C + j] = cnt;
    } else {
        c = (double)S.init[idx];
    }
    S.cd[idx] = c;
    S.centroids[idx] = (float)c;
    double cr = (double)(float)c;
    if (BF16) {
        const bf16_t b = f64_to_bf16(c);
        S.cb[idx] = b;
        S.cbT[(((size_t)h * (d / 8) + (k >> 3)) * C + j) * 8 + (k & 7)] = b;
        cr = (double)bf16_to_f32(b);
    }
    double sq = cr * cr;
    for (int o = 32; o > 0; o >>= 1) sq += __shfl_xor(sq, o);
    if ((k & 63) == 0) s_red[k >> 6] = sq;
    __syncthreads();
    if (k == 0) {
        const double n2 = (d > 64) ? s_red[0] + s_red[1] : s_red[0];
        S.cn64[(size_t)h * C + j] = n2;
        S.hcn[(size_t)h * C + j] = BF16 ? (float)(-0.5 * n2) : (float)n2;
    }
}

// ---------------------------------------------------------------- assign, bf16 MFMA
// grid (one workgroup per CU), block 64 * KM_NW.  The blocks of KM_WG_TOKENS tokens of all heads of a side form one
// sequence; workgroup w takes the w-th of gridDim.x equal parts of it, on both sides: even workgroups first on the
// second side (the K tokens of a layer: many centroids, bound by the matrix cores) and then on the first (the Q
// tokens: few centroids, waiting for memory), odd workgroups the other way round, so that the two kinds of work
// share the chip at any time.  A part is cut at head boundaries into spans; the head's centroids (up to KM_CMAX
// at a time) are staged in LDS once per span and stay there for all its blocks.  (One workgroup per 4096 tokens of
// one side, placed by the hardware, took 0.59 instead of 0.50 ms per launch on a layer of 40 heads of 75,600 tokens
// with 100 and 500 centroids: the sum of the times the two sides take alone.)  With more than KM_CMAX centroids the running best and runner-up of a token go through `best` / `second`
// between chunks.
//
// A wavefront takes 64 tokens at a time, as two blocks of 32.  Per 32-centroid row block it issues the 2 KS matrix
// instructions of both, then reduces their accumulators to (best, runner-up) with max3 / med3 trees while the other wavefront of
// the SIMD has the matrix cores.
//
// Near-ties (see KM_TIE_*) are listed for kmeans_settle_kernel.
struct KmTop2 {                 // temporaries of one top-2 reduction, alive across its chunks
    float key[16], t3, s3, T[4], U[4], T01, U01, m01, T23, Tb, Ub;
    bool upd;
};

template <int D, bool OBJ>
__global__ __launch_bounds__(64 * KM_NW, 1) void kmeans_assign_bf16_kernel(KmArgs a, KmIter it)
{
    constexpr int KS = D / 16;              // MFMA k-steps
    constexpr int ROW = D + 8;              // LDS row stride in elements (16 bytes of padding)
    constexpr int NCH = 8;                  // chunks of a top-2 reduction
    extern __shared__ __align__(16) unsigned char s_raw[];
    // -||c||^2 / 2 first: its reads then have offsets below 64 KB, which fit the instruction, and cost no address
    // arithmetic in the step loop
    float *s_hcn = reinterpret_cast<float *>(s_raw);                               // [KM_CMAX]: -||c||^2 / 2
    bf16_t *s_c = reinterpret_cast<bf16_t *>(s_raw + KM_CMAX * sizeof(float));     // [KM_CMAX][ROW]
    __shared__ int s_next;                  // next group of a span that no wavefront has taken yet

    const int N = a.N;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, col = lane & 31;
    const int nbh = (N + KM_WG_TOKENS - 1) / KM_WG_TOKENS;          // token blocks of a head
    const int nb_all = a.H * nbh;                                   // H N d < 2^40: below 2^25
    static_assert(64 * KM_NW == KM_CMAX, "one -||c||^2/2 per thread");

#define KM_FENCE __builtin_amdgcn_sched_barrier(0);
#define KM_PIN(X)
    // this workgroup's part of the block sequence, the same for both sides
    const int part_q = nb_all / (int)gridDim.x, part_r = nb_all % (int)gridDim.x;
    const int part_lo = (int)blockIdx.x * part_q + min((int)blockIdx.x, part_r);
    const int part_hi = part_lo + part_q + ((int)blockIdx.x < part_r ? 1 : 0);
#pragma unroll 1
    for (int sd = 0; sd < a.nsides; ++sd) {
    // odd workgroups start with the first side, even ones with the second: while one half of the CUs is on the Q
    // tokens of a layer (few centroids, waits for memory) the other is on the K tokens (many, matrix cores)
    const int side = (blockIdx.x & 1) ? sd : a.nsides - 1 - sd;
    const KmSide S = side ? a.s[1] : a.s[0];
    int32_t *labels = side ? it.lab[1] : it.lab[0];
    const int C = S.C;
    const int nchunk = (C + KM_CMAX - 1) / KM_CMAX;
#pragma unroll 1
    for (int sp = part_lo; sp < part_hi;) {
    // span: blocks blk0 .. blk0 + nblk of head h
    const int h = sp / nbh, blk0 = sp - h * nbh;
    const int nblk = min(nbh - blk0, part_hi - sp);
    sp += nblk;
    const bf16_t *Xh = reinterpret_cast<const bf16_t *>(S.X) + (size_t)h * N * D;
    const bf16_t *cbh = S.cb + (size_t)h * C * D;
    const float *hcnh = S.hcn + (size_t)h * C;
    float obj = 0.f;
    float cmax2 = 0.f;          // largest ||c||^2 of the head (over the chunks so far), for the near-tie bound
    for (int chunk = 0; chunk < nchunk; ++chunk) {
        const int c0 = chunk * KM_CMAX;
        const int cc = min(KM_CMAX, C - c0), ccp = (cc + 31) & ~31;
        const bool last_chunk = chunk + 1 == nchunk;
        __syncthreads();
        // The span is handed out in groups of KM_TB * 32 tokens: wavefront w starts with group w and then takes
        // the next one nobody has taken (the two wavefronts of a SIMD do not run at the same speed, see the
        // priorities below; with a fixed share the fast ones would wait for the slow ones at the end of the span).
        if (tid == 0) s_next = KM_NW;               // read after the barrier behind the staging
        // Two register buffers.  Tokens as the B operand: lane (col, half) holds elements 16 s + 8 half .. + 8 of
        // token `col`.  The KM_TB * KS loads of a group come in four parts; while a group is computed, the parts of
        // the wavefront's next one are requested one by one between its steps (all eight wavefronts of the
        // workgroup asking for a whole group at the same moment queue up in front of the texture unit, and each
        // of them waits for the queue).
        bf16x8 xb[2][KM_TB][KS];
        constexpr int NLD = KM_TB * KS, LPP = NLD / 4;
        auto load_part = [&](auto buf_tag, int g, auto part_tag) {
            constexpr int BUF = decltype(buf_tag)::value, PART = decltype(part_tag)::value;
            const int tok0 = blk0 * KM_WG_TOKENS + g * (KM_TB * 32);
#pragma unroll
            for (int i = PART * LPP; i < (PART + 1) * LPP; ++i) {
                const int tb = i / KS, s = i % KS;
                const int n = min(N - 1, tok0 + tb * 32 + col);
                const uint4 v = reinterpret_cast<const uint4 *>(Xh + (size_t)n * D + 8 * half)[2 * s];
                __builtin_memcpy(&xb[BUF][tb][s], &v, 16);
            }
        };
        auto load_x = [&](auto buf_tag, int g) {
            load_part(buf_tag, g, std::integral_constant<int, 0>{});
            load_part(buf_tag, g, std::integral_constant<int, 1>{});
            load_part(buf_tag, g, std::integral_constant<int, 2>{});
            load_part(buf_tag, g, std::integral_constant<int, 3>{});
        };
        // stage the chunk (rows past the last centroid are zero and can never win).  A thread requests all its
        // pieces before it stores the first, so the block waits for one round trip to memory, not sixteen;
        // no branches (a row past the end re-reads the last one and is zeroed in registers), and every workgroup
        // starts at another row, so that the workgroups of a head that run side by side do not ask the same L2
        // channel for the same line at the same moment.
        {
            constexpr int PER = KM_CMAX * (D / 8) / (64 * KM_NW), HALF = PER;
            static_assert((KM_CMAX & (KM_CMAX - 1)) == 0, "row rotation wraps with a mask");
            const int rot = (int)(blockIdx.x * 37u) & (KM_CMAX - 1);
            // the addresses are formed here, in every chunk: formed once in front of the chunk loop (where the
            // compiler would move them) they would sit in scratch memory while the token blocks are computed
            int tid_o = tid;
            asm volatile("" : "+v"(tid_o));
#pragma unroll
            for (int i0 = 0; i0 < PER; i0 += HALF) {
                uint4 v[HALF];
#pragma unroll
                for (int i = 0; i < HALF; ++i) {
                    const int e = tid_o + (i0 + i) * 64 * KM_NW, r = ((e / (D / 8)) + rot) & (KM_CMAX - 1);
                    v[i] = reinterpret_cast<const uint4 *>(cbh + (size_t)(c0 + min(r, cc - 1)) * D)[e % (D / 8)];
                }
                // in the same round trip: this thread's -||c||^2/2 and the wavefront's first block of tokens
                const float hv = hcnh[c0 + min(tid_o, cc - 1)];
                load_x(std::integral_constant<int, 0>{}, wave);
#pragma unroll
                for (int i = 0; i < HALF; ++i) {
                    const int e = tid_o + (i0 + i) * 64 * KM_NW, r = ((e / (D / 8)) + rot) & (KM_CMAX - 1);
                    if (r >= cc) v[i] = make_uint4(0, 0, 0, 0);
                    *reinterpret_cast<uint4 *>(&s_c[r * ROW + (e % (D / 8)) * 8]) = v[i];
                }
                s_hcn[tid] = tid < cc ? hv : KM_PAD_HCN;
            }
        }
        __syncthreads();
        {
            float m = cmax2;
#pragma unroll
            for (int k = 0; k < KM_CMAX / 64; ++k) {
                const int t = lane + 64 * k;
                m = fmaxf(m, t < cc ? -2.f * s_hcn[t] : 0.f);
            }
            for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
            cmax2 = m;
        }

        // What a block of tokens writes (label; running pair or the near-tie list) is held back until the tokens of
        // the next block have been waited for: that wait is for ALL outstanding memory operations, and behind the
        // stores it would last a round trip to memory although the tokens arrived long ago.
        int pend_n[KM_TB], pend_c[KM_TB];
        float pend_T[KM_TB], pend_U[KM_TB];
        bool pend_f[KM_TB], pend = false;
        auto flush = [&]() {
            if (!pend) return;
            pend = false;
#pragma unroll
            for (int tb = 0; tb < KM_TB; ++tb) {
                const int n = pend_n[tb];
                if (half == 0 && n < N) {
                    labels[(size_t)h * N + n] = pend_c[tb];
                    if (!last_chunk) {
                        S.best[(size_t)h * N + n] = pend_T[tb];
                        S.second[(size_t)h * N + n] = pend_U[tb];
                    } else if (pend_f[tb]) {
                        const int pos = atomicAdd(&S.flag_cnt[h], 1);
                        S.flag_list[(size_t)h * N + pos] = n;
                    }
                }
            }
        };
        // Accumulator i of a lane is centroid 8 (i/4) + 4 half + i%4 of the row block; its key is the accumulator
        // with i in its 4 lowest mantissa bits, compared as a float.  best = largest key seen, second = runner-up,
        // bbase = first centroid of the row block the best came from (the same number in every lane: the select
        // then takes it from a scalar register).
        auto compute = [&](auto buf_tag, int g) -> int {
            constexpr int BUF = decltype(buf_tag)::value;
            // the group after this one (taken here, so that the answer is there when the first step wants it)
            int g_next = 0;
            if (lane == 0) g_next = atomicAdd(&s_next, 1);
            g_next = __builtin_amdgcn_readfirstlane(g_next);
            const int tok0 = blk0 * KM_WG_TOKENS + g * (KM_TB * 32);
            float best[KM_TB], second[KM_TB];
            int bbase[KM_TB];
#pragma unroll
            for (int tb = 0; tb < KM_TB; ++tb) {
                best[tb] = -INFINITY;
                second[tb] = -INFINITY;
                bbase[tb] = 0;
            }
            // The two wavefronts of a SIMD (w and w + 4) get different priorities: with equal ones they fall into
            // step, both in their matrix instructions and then both in their reductions, and each unit idles
            // while the other works.
            if (wave & 4) __builtin_amdgcn_s_setprio(2); else __builtin_amdgcn_s_setprio(0);
            const int nrb = ccp / 32;
            // steps after which the four parts of the next block are requested: spread over the first half of a
            // long block (the loads then have the second half to land in), all at once when the block is short
            const int pstep = nrb >= 8 ? nrb / 8 : 0;
            // everything this wavefront has requested so far -- the tokens of this block -- has to be there; said
            // here, in front of the loop, the compiler places no wait inside it
            __builtin_amdgcn_s_waitcnt(0x0F70);
            flush();
            bf16x8 am[KS];
            f32x16 cinit;
            auto fetch_c = [&](int rb) {
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const float4 v = *reinterpret_cast<const float4 *>(&s_hcn[rb * 32 + 8 * g + 4 * half]);
                    cinit[4 * g] = v.x; cinit[4 * g + 1] = v.y; cinit[4 * g + 2] = v.z; cinit[4 * g + 3] = v.w;
                }
            };
            auto fetch_a = [&](int rb, int s) {
                const uint4 v = *reinterpret_cast<const uint4 *>(&s_c[(rb * 32 + col) * ROW + 8 * half + 16 * s]);
                __builtin_memcpy(&am[s], &v, 16);
            };
            // chunk c (0 .. NCH - 1) of the top-2 reduction of A into (bst, snd, bse)
            auto red_chunk = [&](int c, const f32x16 &A, KmTop2 &r, float &bst, float &snd, int &bse, int rbase) {
                auto pack = [&](int i) {
                    r.key[i] = __uint_as_float((__float_as_uint(A[i]) & 0xFFFFFFF0u) | (unsigned)i);
                    KM_PIN(r.key[i])
                };
                if (c == 0) {
                    pack(0); pack(1); pack(2); pack(3);
                    r.t3 = km_max3(r.key[0], r.key[1], r.key[2]);
                    r.s3 = km_med3(r.key[0], r.key[1], r.key[2]);
                    KM_PIN(r.t3) KM_PIN(r.s3)
                } else if (c == 1) {
                    r.T[0] = km_max(r.t3, r.key[3]);
                    r.U[0] = km_med3(r.t3, r.s3, r.key[3]);
                    pack(4); pack(5); pack(6); pack(7);
                    KM_PIN(r.T[0]) KM_PIN(r.U[0])
                } else if (c == 2) {
                    r.t3 = km_max3(r.key[4], r.key[5], r.key[6]);
                    r.s3 = km_med3(r.key[4], r.key[5], r.key[6]);
                    r.T[1] = km_max(r.t3, r.key[7]);
                    r.U[1] = km_med3(r.t3, r.s3, r.key[7]);
                    r.T01 = km_max(r.T[0], r.T[1]);
                    r.m01 = km_min(r.T[0], r.T[1]);
                    KM_PIN(r.U[1]) KM_PIN(r.T01) KM_PIN(r.m01)
                } else if (c == 3) {
                    r.U01 = km_max3(r.m01, r.U[0], r.U[1]);
                    pack(8); pack(9); pack(10); pack(11);
                    r.t3 = km_max3(r.key[8], r.key[9], r.key[10]);
                    KM_PIN(r.U01) KM_PIN(r.t3)
                } else if (c == 4) {
                    r.s3 = km_med3(r.key[8], r.key[9], r.key[10]);
                    r.T[2] = km_max(r.t3, r.key[11]);
                    r.U[2] = km_med3(r.t3, r.s3, r.key[11]);
                    pack(12); pack(13); pack(14);
                    KM_PIN(r.T[2]) KM_PIN(r.U[2])
                } else if (c == 5) {
                    pack(15);
                    r.t3 = km_max3(r.key[12], r.key[13], r.key[14]);
                    r.s3 = km_med3(r.key[12], r.key[13], r.key[14]);
                    r.T[3] = km_max(r.t3, r.key[15]);
                    r.U[3] = km_med3(r.t3, r.s3, r.key[15]);
                    r.T23 = km_max(r.T[2], r.T[3]);
                    KM_PIN(r.U[3]) KM_PIN(r.T23)
                } else if (c == 6) {
                    const float m23 = km_min(r.T[2], r.T[3]);
                    const float U23 = km_max3(m23, r.U[2], r.U[3]);
                    r.Tb = km_max(r.T01, r.T23);
                    const float mb = km_min(r.T01, r.T23);
                    r.Ub = km_max3(mb, r.U01, U23);
                    r.upd = r.Tb > bst;
                    KM_PIN(r.Tb) KM_PIN(r.Ub)
                } else {
                    bse = r.upd ? rbase : bse;
                    snd = km_max3(km_min(bst, r.Tb), snd, r.Ub);
                    bst = km_max(bst, r.Tb);
                    KM_PIN(bse) KM_PIN(snd) KM_PIN(bst)
                }
            };
            // One step = one 32-centroid row block against both token blocks: 2 KS matrix instructions back to back,
            // the LDS reads of the next row block's operands, then the two top-2 reductions on the vector ALU
            // while the other wavefront of the SIMD has the matrix cores.  (Interleaving the reduction of one token
            // block with the matrix instructions of the other, chunk by chunk, was measured slower: 0.49 against
            // 0.42 ms for the K side of the Wan-like layer.)
            fetch_c(0);
#pragma unroll
            for (int s = 0; s < KS; ++s) fetch_a(0, s);
#pragma unroll 1
            for (int rb = 0; rb < nrb; ++rb) {
                f32x16 acc[KM_TB];
#pragma unroll
                for (int s = 0; s < KS; ++s)
#pragma unroll
                    for (int q = 0; q < KM_TB; ++q)
                        acc[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(am[s], xb[BUF][q][s], s == 0 ? cinit : acc[q], 0, 0, 0);
                KM_FENCE
                if (rb + 1 < nrb) {
                    fetch_c(rb + 1);
#pragma unroll
                    for (int s = 0; s < KS; ++s) fetch_a(rb + 1, s);
                }
                {
                    using NB = std::integral_constant<int, BUF ^ 1>;
                    if (rb == 0) load_part(NB{}, g_next, std::integral_constant<int, 0>{});
                    if (rb == pstep) load_part(NB{}, g_next, std::integral_constant<int, 1>{});
                    if (rb == 2 * pstep) load_part(NB{}, g_next, std::integral_constant<int, 2>{});
                    if (rb == 3 * pstep) load_part(NB{}, g_next, std::integral_constant<int, 3>{});
                }
                KM_FENCE
                const int rbase = c0 + rb * 32;
#pragma unroll
                for (int q = 0; q < KM_TB; ++q) {
                    KmTop2 r;
#pragma unroll
                    for (int c = 0; c < NCH; ++c) red_chunk(c, acc[q], r, best[q], second[q], bbase[q], rbase);
                }
                KM_FENCE
            }
            KM_FENCE
#pragma unroll
            for (int tb = 0; tb < KM_TB; ++tb) {
                const unsigned kb = __float_as_uint(best[tb]);
                const int cown = bbase[tb] + 4 * half + (int)(((kb & 12u) << 1) | (kb & 3u));
                // the two lane halves of a token hold disjoint centroids
                const KmHalves hb = km_halves(kb), hs = km_halves(__float_as_uint(second[tb])),
                               hi = km_halves((unsigned)cown);
                const float b0 = __uint_as_float(hb.lo), b1 = __uint_as_float(hb.hi);
                float T = km_max(b0, b1), U = km_max3(km_min(b0, b1), __uint_as_float(hs.lo), __uint_as_float(hs.hi));
                int cidx = (b1 > b0) ? (int)hi.hi : (int)hi.lo;
                const int n = tok0 + tb * 32 + col;
                if (chunk > 0) {
                    // best and runner-up over the earlier chunks (read here, behind the loop: a load in front of
                    // it would make every step of the loop wait for all outstanding loads, the prefetch included)
                    const int nn = min(N - 1, n);
                    const float cb = S.best[(size_t)h * N + nn], cs = S.second[(size_t)h * N + nn];
                    const int cl = labels[(size_t)h * N + nn];
                    U = km_max3(km_min(T, cb), U, cs);
                    if (!(T > cb)) cidx = cl;
                    T = km_max(T, cb);
                }
                bool flagged = false;
                float x2 = 0.f;
                if (last_chunk) {
                    // ||x||^2, two elements per instruction (this lane's half of the token, then both halves)
#pragma unroll
                    for (int s = 0; s < KS; ++s)
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const bf16x2_t p2 = {xb[BUF][tb][s][2 * e], xb[BUF][tb][s][2 * e + 1]};
                            x2 = __builtin_amdgcn_fdot2_f32_bf16(p2, p2, x2, false);
                        }
                    {
                        const KmHalves hx = km_halves(__float_as_uint(x2));
                        x2 = __uint_as_float(hx.lo) + __uint_as_float(hx.hi);
                    }
                    // runner-up within the error of this contraction: the token is settled in double precision
                    // (a tie, including an exact one, always is)
                    const float tau = KM_TIE_KEY * fabsf(T) + KM_TIE_ACC * (0.5f * x2 + cmax2);
                    flagged = half == 0 && n < N && !(T - U > tau);
                    if (OBJ && S.objective && half == 0 && n < N) obj += x2 - 2.f * T;
                }
                pend_n[tb] = n; pend_c[tb] = cidx; pend_T[tb] = T; pend_U[tb] = U; pend_f[tb] = flagged;
            }
            pend = true;
            return g_next;
        };
        // The tokens of the group after the one being computed are ALWAYS requested (past the end of the span the
        // addresses are clamped and the values unused): with a conditional prefetch the compiler has to place waits
        // that are also right for the path without it.
        const int ng = nblk * KM_NW;
#pragma unroll 1
        for (int g = wave; g < ng;) {
            g = compute(std::integral_constant<int, 0>{}, g);
            if (g < ng) g = compute(std::integral_constant<int, 1>{}, g);
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);     // the last, unused request: the registers are reused from here on
        flush();
    }
    if (OBJ && S.objective) {
        for (int o = 32; o > 0; o >>= 1) obj += __shfl_xor(obj, o);
        if (lane == 0) atomicAdd(S.objective + (size_t)h * a.iters + it.t, obj);
    }
    }   // spans
    }   // sides
#undef KM_FENCE
#undef KM_PIN
}

// ---------------------------------------------------------------- settle near-ties, bf16 input
// grid (KM_SETTLE_BLOCKS, H * sides), block 256: one workgroup per listed token at a time.  The token's distance
// ||c_j||^2 - 2 x.c_j to EVERY centroid in double precision: wavefront w takes the centroid groups
// 64 (w + 4 i) .. + 64, lane l of it centroid l of the group (read from the chunk-major copy, so the 64 lanes of a
// load read 1 KB of consecutive memory); smallest distance wins, lowest index on an exact tie.  x and c are bf16
// numbers: every product is exact and the sums of 128 of them fit a double, so this is the argmin of the
// definition.  A token costs a wavefront a few thousand double-precision instructions, which is why the four
// wavefronts share it: what the launch takes is the time of ONE token (a head lists a few dozen).
template <int D>
__global__ __launch_bounds__(256) void kmeans_settle_kernel(KmArgs a, KmIter it)
{
    __shared__ __align__(16) double s_x[D];
    __shared__ double s_best[4];
    __shared__ int s_bj[4];
    const int side = blockIdx.y % a.nsides, h = blockIdx.y / a.nsides;
    const KmSide S = side ? a.s[1] : a.s[0];
    int32_t *labels = side ? it.lab[1] : it.lab[0];
    const int N = a.N, C = S.C;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int cnt = min(S.flag_cnt[h], N);
    const bf16_t *Xh = reinterpret_cast<const bf16_t *>(S.X) + (size_t)h * N * D;
    const uint4 *ct = reinterpret_cast<const uint4 *>(S.cbT) + (size_t)h * (D / 8) * C;
    const double *cn = S.cn64 + (size_t)h * C;
    for (int t = blockIdx.x; t < cnt; t += gridDim.x) {
        const int n = S.flag_list[(size_t)h * N + t];
        __syncthreads();                            // the previous token's s_x / s_best are no longer read
        if (tid < D) s_x[tid] = (double)bf16_to_f32(Xh[(size_t)n * D + tid]);
        __syncthreads();
        double best = INFINITY;
        int bj = 0x7FFFFFFF;
        for (int j0 = 64 * wave; j0 < C; j0 += 256) {
            // the token is read from LDS as it is used: kept in registers across this loop it takes 2 D of them, one
            // workgroup then fills a CU, and most workgroups of a launch find nothing to do -- how fast they come
            // and go decides how long the launch takes (55 us per launch on the Wan-like layer that way, 26 us so)
            asm volatile("" ::: "memory");
            const int j = min(j0 + lane, C - 1);
            uint4 w4[D / 8];
#pragma unroll
            for (int q = 0; q < D / 8; ++q) w4[q] = ct[(size_t)q * C + j];
            double dot = 0.0;
#pragma unroll
            for (int q = 0; q < D / 8; ++q) {
                const unsigned w[4] = {w4[q].x, w4[q].y, w4[q].z, w4[q].w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    dot = fma(s_x[8 * q + 2 * e], (double)__uint_as_float(w[e] << 16), dot);
                    dot = fma(s_x[8 * q + 2 * e + 1], (double)__uint_as_float(w[e] & 0xFFFF0000u), dot);
                }
            }
            const double dist = cn[j] - 2.0 * dot;
            // ascending j inside a lane: strict < keeps the lower index
            if (j0 + lane < C && dist < best) { best = dist; bj = j; }
        }
        for (int o = 32; o > 0; o >>= 1) {
            const double ob = __shfl_xor(best, o);
            const int oj = __shfl_xor(bj, o);
            if (ob < best || (ob == best && oj < bj)) { best = ob; bj = oj; }
        }
        if (lane == 0) { s_best[wave] = best; s_bj[wave] = bj; }
        __syncthreads();
        if (tid == 0) {
#pragma unroll
            for (int w = 1; w < 4; ++w)
                if (s_best[w] < best || (s_best[w] == best && s_bj[w] < bj)) { best = s_best[w]; bj = s_bj[w]; }
            labels[(size_t)h * N + n] = bj;
        }
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
// Segmented sum over the sorted order, one wavefront per piece (at most KM_SEG rows of one cluster).  A row is LPR
// lanes of 16 bytes; 64 / LPR rows are read per instruction and KM_UB instructions are in flight before their
// values are added, in double precision.
//   DELTA = false  grid (ceil(max_pieces / 4), H, sides): every row of the piece (set `it.set`).
//   DELTA = true   grid (.., H, 2 * sides), z = 2 * side + dir: only the rows of a piece whose label in `other`
//                  differs from the piece's cluster.  dir 0: the new order (set) against the previous labels --
//                  the tokens that JOINED the cluster; dir 1: the previous order (other set) against the new
//                  labels -- the tokens that LEFT it.  A wavefront first scans its piece one row per lane and
//                  packs the rows that qualify into a list, then reads only those rows of X.
template <typename T, int D, bool DELTA>
__global__ __launch_bounds__(256) void kmeans_segsum_kernel(KmArgs a, KmIter it)
{
    constexpr int EPL = 16 / sizeof(T);            // elements per lane
    constexpr int LPR = D / EPL;                   // lanes per row
    constexpr int RPI = 64 / LPR;                  // rows per instruction
    __shared__ int32_t s_list[DELTA ? 4 : 1][DELTA ? KM_SEG : 1];
    const int side = DELTA ? blockIdx.z >> 1 : blockIdx.z, dir = DELTA ? (blockIdx.z & 1) : 0;
    const KmSide S = side ? a.s[1] : a.s[0];
    const int set = dir ? 1 - it.set : it.set;
    const int h = blockIdx.y, lane = threadIdx.x & 63, wave = threadIdx.x >> 6, N = a.N;
    const int piece = blockIdx.x * 4 + wave;
    if (piece >= KM_SEL(S.n_pieces, set)[h]) return;
    const int4 desc = KM_SEL(S.pieces, set)[(size_t)h * S.max_pieces + piece];
    const int cl = desc.x, row0 = desc.y, nrows = desc.z;
    const int sub = lane / LPR, part = lane % LPR;
    const T *Xh = reinterpret_cast<const T *>(S.X) + (size_t)h * N * D;
    const int32_t *pm = KM_SEL(S.perm, set) + (size_t)h * N;
    int cnt = nrows;
    int32_t *list = s_list[DELTA ? wave : 0];
    if (DELTA) {
        const int32_t *other = (dir ? (side ? it.lab[1] : it.lab[0]) : (side ? it.lab_prev[1] : it.lab_prev[0])) + (size_t)h * N;
        const unsigned long long lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
        cnt = 0;
        // the rows of the piece and then their other labels are requested together: two memory round trips
        // for the piece instead of two per 64 rows
        constexpr int NG = KM_SEG / 64;
        int srcs[NG], oth[NG];
#pragma unroll
        for (int i = 0; i < NG; ++i) {
            const int rr = i * 64 + lane;
            srcs[i] = (rr < nrows) ? pm[row0 + rr] : 0;
        }
#pragma unroll
        for (int i = 0; i < NG; ++i) oth[i] = other[srcs[i]];
#pragma unroll
        for (int i = 0; i < NG; ++i) {
            if (i * 64 >= nrows) break;
            const bool take = i * 64 + lane < nrows && oth[i] != cl;
            const unsigned long long m = __ballot(take);
            if (take) list[cnt + __popcll(m & lt_mask)] = srcs[i];
            cnt += __popcll(m);
        }
    }
    double acc[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] = 0.0;
    for (int r = 0; r < cnt; r += RPI * KM_UB) {
        uint4 v[KM_UB];
        bool ok[KM_UB];
#pragma unroll
        for (int u = 0; u < KM_UB; ++u) {
            const int rr = r + u * RPI + sub;
            ok[u] = rr < cnt;
            const int src = DELTA ? list[min(rr, cnt - 1)] : pm[row0 + min(rr, cnt - 1)];
            v[u] = reinterpret_cast<const uint4 *>(Xh + (size_t)src * D)[part];
        }
#pragma unroll
        for (int u = 0; u < KM_UB; ++u) {
            if (!ok[u]) continue;
            const unsigned w[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
            if (sizeof(T) == 2) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    acc[2 * q] += (double)__uint_as_float(w[q] << 16);
                    acc[2 * q + 1] += (double)__uint_as_float(w[q] & 0xFFFF0000u);
                }
            } else {
#pragma unroll
                for (int q = 0; q < 4; ++q) acc[q] += (double)__uint_as_float(w[q]);
            }
        }
    }
    // lanes with the same `part` hold the same columns
#pragma unroll
    for (int o = LPR; o < 64; o <<= 1)
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[e] += __shfl_xor(acc[e], o);
    if (sub == 0) {
        double *out = KM_SEL(S.psum, set) + ((size_t)h * S.max_pieces + piece) * D + part * EPL;
#pragma unroll
        for (int e = 0; e < EPL; e += 2) *reinterpret_cast<double2 *>(out + e) = make_double2(acc[e], acc[e + 1]);
    }
}

__global__ void kmeans_zero_kernel(float *p, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0.f;
}

// ---------------------------------------------------------------- host side
static void kmeans_carve_side(Carver &c, KmSide &k, int H, int N, int d, int C)
{
    k.C = C;
    k.max_pieces = cdiv(N, KM_SEG) + C;
    k.cb = c.take<bf16_t>((size_t)H * C * d);
    k.cbT = c.take<bf16_t>((size_t)H * C * d);
    k.hcn = c.take<float>((size_t)H * C);
    k.cn64 = c.take<double>((size_t)H * C);
    k.cd = c.take<double>((size_t)H * C * d);
    k.csum = c.take<double>((size_t)H * C * d);
    for (int s = 0; s < 2; ++s) {
        k.offsets[s] = c.take<int32_t>((size_t)H * (C + 1));
        k.perm[s] = c.take<int32_t>((size_t)H * N);
        k.first_piece[s] = c.take<int32_t>((size_t)H * (C + 1));
        k.n_pieces[s] = c.take<int32_t>((size_t)H);
        k.pieces[s] = c.take<int4>((size_t)H * k.max_pieces);
        k.psum[s] = c.take<double>((size_t)H * k.max_pieces * d);
    }
    k.labels_alt = c.take<int32_t>((size_t)H * N);
    k.flag_cnt = c.take<int32_t>((size_t)H);
    k.flag_list = c.take<int32_t>((size_t)H * N);
    k.best = c.take<float>(C > KM_CMAX ? (size_t)H * N : 0);
    k.second = c.take<float>(C > KM_CMAX ? (size_t)H * N : 0);
    k.hist = reinterpret_cast<int32_t *>(c.take<char>(permute_ws_bytes(H, N, C)));
}

size_t kmeans_ws_bytes(int dtype, int H, int N, int d, int C)
{
    (void)dtype;
    Carver c(nullptr);
    KmSide k;
    kmeans_carve_side(c, k, H, N, d, C);
    return c.used;
}

size_t kmeans_pair_ws_bytes(int dtype, int H, int N, int d, int Cq, int Ck)
{
    return kmeans_ws_bytes(dtype, H, N, d, Cq) + kmeans_ws_bytes(dtype, H, N, d, Ck);
}

// dynamic LDS of the bf16 assign kernel
template <int D> static constexpr size_t kmeans_assign_lds()
{
    return (size_t)KM_CMAX * (D + 8) * sizeof(bf16_t) + KM_CMAX * sizeof(float);
}

int kmeans_prepare(int dtype, int d)
{
    if (dtype != SVG2_BF16) return SVG2_OK;
    if (d == 128) {
        SVG2_TRY(set_dynamic_lds(reinterpret_cast<const void *>(kmeans_assign_bf16_kernel<128, true>), kmeans_assign_lds<128>()));
        SVG2_TRY(set_dynamic_lds(reinterpret_cast<const void *>(kmeans_assign_bf16_kernel<128, false>), kmeans_assign_lds<128>()));
    } else {
        SVG2_TRY(set_dynamic_lds(reinterpret_cast<const void *>(kmeans_assign_bf16_kernel<64, true>), kmeans_assign_lds<64>()));
        SVG2_TRY(set_dynamic_lds(reinterpret_cast<const void *>(kmeans_assign_bf16_kernel<64, false>), kmeans_assign_lds<64>()));
    }
    return SVG2_OK;
}

// number of compute units of the current device (the bf16 assign kernel runs one workgroup on each)
static int device_cu_count(int *ncu)
{
    static std::atomic<int> known[64];
    int dev = -1;
    SVG2_HIP_CHECK(hipGetDevice(&dev));
    int n = (dev >= 0 && dev < 64) ? known[dev].load() : 0;
    if (n <= 0) {
        SVG2_HIP_CHECK(hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev));
        SVG2_REQUIRE(n > 0, SVG2_HIP_ERROR, "device %d reports %d compute units", dev, n);
        if (dev >= 0 && dev < 64) known[dev].store(n);
    }
    *ncu = n;
    return SVG2_OK;
}

template <typename T, int D, bool BF16>
static int kmeans_run(KmArgs a, hipStream_t st)
{
    const int H = a.H, N = a.N, iters = a.iters, ns = a.nsides;
    int ncu = 0;
    if (BF16) SVG2_TRY(device_cu_count(&ncu));
    int cmax = 0, pmax = 0;
    bool any_obj = false;
    for (int s = 0; s < ns; ++s) {
        cmax = std::max(cmax, a.s[s].C);
        pmax = std::max(pmax, a.s[s].max_pieces);
        if (a.s[s].objective) {
            any_obj = true;
            hipLaunchKernelGGL(kmeans_zero_kernel, dim3(cdiv(H * iters, 256)), dim3(256), 0, st, a.s[s].objective, H * iters);
        }
    }
    {
        ProfileSpan sp(SVG2_K_KMEANS_FINALIZE, st);
        hipLaunchKernelGGL((kmeans_finalize_kernel<BF16>), dim3(cmax, H, ns), dim3(D), 0, st, a, 0, 0);
    }
    for (int t = 0; t < iters; ++t) {
        // Update step: the first iteration, and every KM_FULL_EVERY-th after that, sums every cluster afresh; the
        // others only move the tokens whose label changed (a quarter in the second iteration, a few per cent from
        // the third on) between the cluster sums, which reads a fraction of X.
        const bool full = t % KM_FULL_EVERY == 0;
        KmIter it;
        it.t = t;
        it.set = t & 1;
        for (int s = 0; s < 2; ++s) {
            // the labels of iteration t go to the caller's buffer when iters - 1 - t is even, else to the scratch
            // buffer: the last iteration lands in the caller's buffer, the previous labels are always the other one
            const bool alt = (iters - 1 - t) & 1;
            it.lab[s] = alt ? a.s[s].labels_alt : a.s[s].labels;
            it.lab_prev[s] = alt ? a.s[s].labels : a.s[s].labels_alt;
        }
        if (BF16) {
            const long long nb_all = (long long)H * cdiv(N, KM_WG_TOKENS);
            const dim3 grid((unsigned)std::min<long long>(ncu, nb_all));
            auto kern = any_obj ? kmeans_assign_bf16_kernel<D, true> : kmeans_assign_bf16_kernel<D, false>;
            {
                ProfileSpan sp(SVG2_K_KMEANS_ASSIGN, st);
                hipLaunchKernelGGL(kern, grid, dim3(64 * KM_NW), kmeans_assign_lds<D>(), st, a, it);
            }
            {
                ProfileSpan sp(SVG2_K_KMEANS_SETTLE, st);
                hipLaunchKernelGGL((kmeans_settle_kernel<D>), dim3(KM_SETTLE_BLOCKS, H * ns), dim3(256), 0, st, a, it);
            }
        } else {
            const dim3 grid(cdiv(N, 128), H);
            ProfileSpan sp(SVG2_K_KMEANS_ASSIGN, st);
            for (int s = 0; s < ns; ++s) {
                const float *Xf = reinterpret_cast<const float *>(a.s[s].X);
                float *obj = a.s[s].objective ? a.s[s].objective + t : nullptr;
                if (obj)
                    hipLaunchKernelGGL((kmeans_assign_f32_kernel<D, true>), grid, dim3(128), 0, st, Xf, a.s[s].centroids,
                                       a.s[s].hcn, N, a.s[s].C, it.lab[s], obj, iters);
                else
                    hipLaunchKernelGGL((kmeans_assign_f32_kernel<D, false>), grid, dim3(128), 0, st, Xf, a.s[s].centroids,
                                       a.s[s].hcn, N, a.s[s].C, it.lab[s], obj, iters);
            }
        }
        // label-sorted order of the tokens and its pieces, then the segmented sum over it
        SortArgs sa = {};
        for (int s = 0; s < ns; ++s) {
            const KmSide &k = a.s[s];
            sa.s[s].labels = it.lab[s];
            sa.s[s].C = k.C;
            sa.s[s].hist = k.hist;
            sa.s[s].offsets = k.offsets[it.set];
            sa.s[s].perm = k.perm[it.set];
            sa.s[s].inv_perm = nullptr;
            sa.s[s].pieces = k.pieces[it.set];
            sa.s[s].first_piece = k.first_piece[it.set];
            sa.s[s].n_pieces = k.n_pieces[it.set];
            sa.s[s].max_pieces = k.max_pieces;
            sa.s[s].seg = KM_SEG;
        }
        {
            ProfileSpan sp(SVG2_K_KMEANS_SORT, st);
            SVG2_TRY(sort_launch(sa, ns, H, N, st));
        }
        if (full) {
            ProfileSpan sp(SVG2_K_KMEANS_SEGSUM_FULL, st);
            hipLaunchKernelGGL((kmeans_segsum_kernel<T, D, false>), dim3(cdiv(pmax, 4), H, ns), dim3(256), 0, st, a, it);
        } else {
            ProfileSpan sp(SVG2_K_KMEANS_SEGSUM_DELTA, st);
            hipLaunchKernelGGL((kmeans_segsum_kernel<T, D, true>), dim3(cdiv(pmax, 4), H, 2 * ns), dim3(256), 0, st, a, it);
        }
        {
            ProfileSpan sp(SVG2_K_KMEANS_FINALIZE, st);
            hipLaunchKernelGGL((kmeans_finalize_kernel<BF16>), dim3(cmax, H, ns), dim3(D), 0, st, a, full ? 1 : 2, it.set);
        }
    }
    return SVG2_OK;
}

static int kmeans_dispatch(const KmArgs &a, int dtype, int d, hipStream_t st)
{
    int rc;
    if (dtype == SVG2_BF16) rc = d == 128 ? kmeans_run<bf16_t, 128, true>(a, st) : kmeans_run<bf16_t, 64, true>(a, st);
    else rc = d == 128 ? kmeans_run<float, 128, false>(a, st) : kmeans_run<float, 64, false>(a, st);
    if (rc != SVG2_OK) return rc;
    SVG2_HIP_CHECK(hipGetLastError());
    return SVG2_OK;
}

static void kmeans_fill_side(KmSide &k, const void *X, const float *init, float *centroids, int32_t *labels,
                             int32_t *counts, float *objective)
{
    k.X = X;
    k.init = init;
    k.centroids = centroids;
    k.labels = labels;
    k.counts = counts;
    k.objective = objective;
}

int kmeans_launch(const void *X, int dtype, int H, int N, int d, int C, int iters, const float *init,
                  float *centroids, int32_t *labels, int32_t *counts, float *objective, void *ws, hipStream_t st)
{
    KmArgs a = {};
    a.nsides = 1; a.H = H; a.N = N; a.iters = iters;
    Carver c(ws);
    kmeans_carve_side(c, a.s[0], H, N, d, C);
    kmeans_fill_side(a.s[0], X, init, centroids, labels, counts, objective);
    a.s[1] = a.s[0];
    return kmeans_dispatch(a, dtype, d, st);
}

int kmeans_pair_launch(const void *Q, const void *K, int dtype, int H, int N, int d, int Cq, int Ck, int iters,
                       float *cq_inout, float *ck_inout, int32_t *labels_q, int32_t *labels_k, int32_t *counts_q,
                       int32_t *counts_k, void *ws, hipStream_t st)
{
    KmArgs a = {};
    a.nsides = 2; a.H = H; a.N = N; a.iters = iters;
    Carver c(ws);
    kmeans_carve_side(c, a.s[0], H, N, d, Cq);
    kmeans_carve_side(c, a.s[1], H, N, d, Ck);
    kmeans_fill_side(a.s[0], Q, cq_inout, cq_inout, labels_q, counts_q, nullptr);
    kmeans_fill_side(a.s[1], K, ck_inout, ck_inout, labels_k, counts_k, nullptr);
    return kmeans_dispatch(a, dtype, d, st);
}

}  // namespace svg2
