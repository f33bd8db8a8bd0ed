// Pieces shared by the attention kernels (bf16 / fp32 / fp8 storage): vector types, tile constants,
// LDS readers, the key-run lookup, cross-half reductions and the carving of the plan workspace.
#pragma once

#include "svg2_common.h"

namespace svg2 {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

static constexpr int ATT_BN = 64;          // keys per tile
static constexpr int ATT_GROUP = 8;        // consecutive tiles handed to one XCD
static constexpr int ATT_NW = 4;           // wavefronts per workgroup of the matrix-core kernels, 32 queries each

// LDS transposing read: the 16 lanes of a block each pass the address of 4
// consecutive 16-bit values (row r = lane % 16); lane L gets element L % 4 of
// rows L / 4, L / 4 + 4, L / 4 + 8, L / 4 + 12.

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

// v_max_f32 / v_max3_f32 as they are: fmaxf() makes the compiler first canonicalise each operand it cannot prove
// quiet (one extra v_max_f32 x, x per operand); the scores here come out of the matrix cores and are never
// signalling NaNs.  Not volatile: the scheduler may still place them.
__device__ __forceinline__ float max2_raw(float a, float b)
{
    float r;
    asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}
__device__ __forceinline__ float max3_raw(float a, float b, float c)
{
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

// max / sum of a value with the one held by lane ^ 32 (v_permlane32_swap: no LDS round trip)
__device__ __forceinline__ float max_xor32(float x)
{
    const unsigned u = __float_as_uint(x);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return max2_raw(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float sum_xor32(float x)
{
    const unsigned u = __float_as_uint(x);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// ---- plan workspace (host)
inline int attn_bm(int dtype) { return dtype == SVG2_BF16 ? 32 * ATT_NW : 64; }   // rows per tile

struct AttnWs {
    int4 *tiles;
    int32_t *n_tiles, *tile_base;
    int2 *runs;
    int32_t *row_keys;
    int32_t *cl_first;                  // [H][Cq] first tile (inside its head) of every query cluster
    int32_t *order;                     // [all tiles] work items, longest first
    int32_t *tile_run;                  // [H][Cq][key_tiles] CSR entry (relative to the row's first) of the run that
                                        // holds key 64 t of the row's virtual key sequence
    int max_tiles, key_tiles;
    size_t bytes;
};

inline AttnWs attn_carve(void *ws, int dtype, int H, int N, int Cq, int Ck)
{
    AttnWs a;
    a.max_tiles = cdiv(N, attn_bm(dtype)) + Cq;
    a.key_tiles = cdiv(N, ATT_BN) + 1;
    Carver c(ws);
    a.tiles = c.take<int4>((size_t)H * a.max_tiles);
    a.n_tiles = c.take<int32_t>((size_t)H);
    a.tile_base = c.take<int32_t>((size_t)H + 1);
    a.runs = c.take<int2>((size_t)H * Cq * Ck);
    a.row_keys = c.take<int32_t>((size_t)H * Cq);
    a.cl_first = c.take<int32_t>((size_t)H * Cq);
    a.order = c.take<int32_t>((size_t)H * a.max_tiles);
    a.tile_run = c.take<int32_t>((size_t)H * Cq * a.key_tiles);
    a.bytes = c.used;
    return a;
}

}  // namespace svg2
