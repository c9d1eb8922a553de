// fp32 values as three bf16 pieces, and the piece layout ("planes") in which wrapper-sized operands are
// handed to the d_block 128 chains.  gfx950 only.
#pragma once
#include "armor_internal.h"

namespace armor {

// ---- fp32 products on the bf16 matrix instruction ------------------------------------------------
// Every fp32 value is cut EXACTLY into three bf16 pieces (x = x1 + x2 + x3: the top 8 significant bits,
// the next 8, the last 8, by truncation) and a product x y is formed as the six partial products
// x3 y1 + x1 y3 + x2 y2 + x2 y1 + x1 y2 + x1 y1 on v_mfma_f32_32x32x16_bf16 (fp32 accumulation); the
// three dropped ones are below 2^-23 |x y|, the size of one fp32 rounding.  Sixteen inner indices then
// cost six 8-pass instructions instead of eight 16-pass ones of v_mfma_f32_32x32x2_f32.
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t uintx4 __attribute__((ext_vector_type(4)));

// Eight floats (the inner indices one lane supplies to a 16-deep matrix instruction) as three vectors
// of eight bf16: pieces 1, 2, 3 of the exact three-way cut.
struct Pieces {
    uint32_t p1[4], p2[4], p3[4];
};
__device__ __forceinline__ uintx4 vec4(const uint32_t (&a)[4]) {
    uintx4 v = {a[0], a[1], a[2], a[3]};
    return v;
}
__device__ __forceinline__ void cut3(const float (&x)[8], Pieces &o) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const uint32_t ua = __float_as_uint(x[2 * e]), ub = __float_as_uint(x[2 * e + 1]);
        o.p1[e] = __builtin_amdgcn_perm(ub, ua, 0x07060302u); // the two upper halves
        const float ra = x[2 * e] - __uint_as_float(ua & 0xffff0000u), rb = x[2 * e + 1] - __uint_as_float(ub & 0xffff0000u);
        const uint32_t va = __float_as_uint(ra), vb = __float_as_uint(rb);
        o.p2[e] = __builtin_amdgcn_perm(vb, va, 0x07060302u);
        const float sa = ra - __uint_as_float(va & 0xffff0000u), sb = rb - __uint_as_float(vb & 0xffff0000u);
        o.p3[e] = __builtin_amdgcn_perm(__float_as_uint(sb), __float_as_uint(sa), 0x07060302u); // at most 8 bits left: exact
    }
}

// One entry of a plane set: the 16 values op(x, 16 run .. 16 run + 15) of block-sized operand `blk_base`
// (3 * 128 * 128 16-bit elements: P[piece][run of 16 inner indices][lane half h][x][8]) become what lane
// (x, h = 0) and lane (x, h = 1) supply to a 16-deep matrix instruction for that run: half h holds the inner
// indices 16 run + 4 h + i and 16 run + 8 + 4 h + i (i = 0..3).  Six 16-byte stores.
constexpr int PLANE_B = 128;
__device__ __forceinline__ void plane_emit(uint16_t *__restrict__ blk_base, int run, int x, const float (&v)[16]) {
    float h0[8], h1[8];
#pragma unroll
    for (int e = 0; e < 4; ++e) { h0[e] = v[e]; h0[4 + e] = v[8 + e]; h1[e] = v[4 + e]; h1[4 + e] = v[12 + e]; }
    Pieces a, b;
    cut3(h0, a);
    cut3(h1, b);
    constexpr int SB = PLANE_B;
    uint16_t *o = blk_base + ((run * 2) * SB + x) * 8;
    *reinterpret_cast<uintx4 *>(o) = vec4(a.p1);
    *reinterpret_cast<uintx4 *>(o + SB * 8) = vec4(b.p1);
    *reinterpret_cast<uintx4 *>(o + SB * SB) = vec4(a.p2);
    *reinterpret_cast<uintx4 *>(o + SB * SB + SB * 8) = vec4(b.p2);
    *reinterpret_cast<uintx4 *>(o + 2 * SB * SB) = vec4(a.p3);
    *reinterpret_cast<uintx4 *>(o + 2 * SB * SB + SB * 8) = vec4(b.p3);
}

} // namespace armor
