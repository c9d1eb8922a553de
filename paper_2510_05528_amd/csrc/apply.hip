// The factorized layer applied to a batch of activations (Sec. 3.1: y = A (S (B x)), the wrappers as
// batched block products around the 2:4 core; Sec. 4.4 times this on a batch of tokens).
// bf16 operands, fp32 accumulation, the two intermediates rounded to bf16.  gfx950:
//   apply_pre_kernel   U = X B^T (block-diagonal), dense v_mfma_f32_32x32x16_bf16, operands straight
//                      from global memory (the kernel is bound by reading X and writing U once);
//   apply_main_kernel  Y = (U S^T) A^T: the core product on the 2:4 structured-sparse matrix
//                      instruction v_smfmac_f32_32x32x32_bf16 (the compressed values and the 2-bit
//                      in-group columns of armor_pack_nm are exactly its sparse operand and index),
//                      then the A wrapper as an epilogue on the accumulator tile.
#include "armor_internal.h"

namespace armor {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ uint32_t pack_bf16x2_rne(float lo, float hi) {
    uint32_t a = __float_as_uint(lo), b = __float_as_uint(hi);
    a = (a & 0x7fffffffu) > 0x7f800000u ? (a | 0x400000u) : a + 0x7fffu + ((a >> 16) & 1u);
    b = (b & 0x7fffffffu) > 0x7f800000u ? (b | 0x400000u) : b + 0x7fffu + ((b >> 16) & 1u);
    return (a >> 16) | (b & 0xffff0000u);
}

__global__ __launch_bounds__(256) void to_bf16_kernel(const float *__restrict__ in, int64_t n, uint16_t *__restrict__ out) {
    int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e < n) out[e] = (uint16_t)(pack_bf16x2_rne(in[e], 0.f) & 0xffffu);
}

void launch_to_bf16(const float *in, int64_t n, void *out, hipStream_t s) {
    hipLaunchKernelGGL(to_bf16_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, in, n,
                       reinterpret_cast<uint16_t *>(out));
}

// ------------------------------------------------------------------------------------------------
// U[t][j*b + p] = sum_q B^j[p][q] X[t][j*b + q].   One wave: 32 tokens x the b columns of block j.
// MFMA rows = tokens (operand from X: 8 consecutive q per lane), columns = p (operand from B^j:
// 8 consecutive q of row p per lane); a lane of the result holds one column p, so a store
// instruction writes 32 consecutive bf16 of one token row.
// ------------------------------------------------------------------------------------------------
template <int B>
__global__ __launch_bounds__(256) void apply_pre_kernel(const uint16_t *__restrict__ X, int64_t n, int64_t d_in,
                                                        const uint16_t *__restrict__ Bw, uint16_t *__restrict__ U) {
    constexpr int PT = B / 32; // column tiles
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, l32 = lane & 31, half = lane >> 5;
    const int j = blockIdx.y;
    const int64_t t0 = ((int64_t)blockIdx.x * 4 + w) * 32;
    if (t0 >= n) return;
    const int64_t trow = min(t0 + l32, n - 1); // clamped: rows past the end are computed and dropped
    const uint16_t *xrow = X + trow * d_in + (int64_t)j * B + 8 * half;
    const uint16_t *brow = Bw + (int64_t)j * B * B + (int64_t)l32 * B + 8 * half;
    floatx16 acc[PT];
#pragma unroll
    for (int pt = 0; pt < PT; ++pt)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[pt][r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < B / 16; ++ks) {
        const bf16x8 a = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(xrow + 16 * ks));
#pragma unroll
        for (int pt = 0; pt < PT; ++pt) {
            const bf16x8 bb = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(brow + (int64_t)pt * 32 * B + 16 * ks));
            acc[pt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bb, acc[pt], 0, 0, 0);
        }
    }
#pragma unroll
    for (int pt = 0; pt < PT; ++pt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int64_t t = t0 + 8 * (r >> 2) + 4 * half + (r & 3);
            if (t < n) U[t * d_in + (int64_t)j * B + pt * 32 + l32] = (uint16_t)(pack_bf16x2_rne(acc[pt][r], 0.f) & 0xffffu);
        }
}

void launch_apply_pre(const void *X, int64_t n, int64_t d_in, int b, const void *Bw, void *U, hipStream_t s) {
    dim3 grid((unsigned)((n + 127) / 128), (unsigned)(d_in / b));
    const uint16_t *x = reinterpret_cast<const uint16_t *>(X), *bw = reinterpret_cast<const uint16_t *>(Bw);
    uint16_t *u = reinterpret_cast<uint16_t *>(U);
    switch (b) {
    case 32: hipLaunchKernelGGL(apply_pre_kernel<32>, grid, dim3(256), 0, s, x, n, d_in, bw, u); break;
    case 64: hipLaunchKernelGGL(apply_pre_kernel<64>, grid, dim3(256), 0, s, x, n, d_in, bw, u); break;
    case 128: hipLaunchKernelGGL(apply_pre_kernel<128>, grid, dim3(256), 0, s, x, n, d_in, bw, u); break;
    default: break;
    }
}

// ------------------------------------------------------------------------------------------------
// Y[t][o] = sum_q A^i[p][q] V[t][i*b + q],  V[t][o] = sum_k S[o][k] U[t][k]  (V rounded to bf16).
// Workgroup: 256 rows of S x 256 tokens, 8 waves as 2 (rows) x 4 (tokens), a wave owns 128 x 64
// (4 x 2 accumulator tiles).  Per stage of 64 dense k: the compressed values (256 x 64 B), their
// index bits (256 x 8 B) and the activations (256 x 128 B) go through LDS (two stages, register
// prefetch of the next one).  Sparse operand of the instruction: lane (row, h) = the 8 kept values
// of dense k in [16h, 16h+16) of the 32-k step and their 16 index bits; dense operand: lane
// (token, h) = k in [8h, 8h+8) and [16+8h, 16+8h+8).
// Epilogue: each wave's 128 rows are whole blocks of A (b <= 128), so it needs only its own V patch:
// written to LDS as [token][q] bf16, multiplied by A^i with the dense bf16 instruction (rows =
// tokens, columns = p), stored like the kernel above.
// ------------------------------------------------------------------------------------------------
constexpr int AP_TM = 256, AP_TN = 256, AP_KT = 64;
constexpr int AP_SUP_R = 8, AP_SUP_T = 4; // super-tile of one XCD: 8 row tiles x 4 token tiles = 32 workgroups
constexpr int AP_SV_PITCH = 80;   // bytes per row of compressed values (64 + 16 pad)
constexpr int AP_U_PITCH = 144;   // bytes per token row (128 + 16 pad)
constexpr int AP_SV_BYTES = AP_TM * AP_SV_PITCH, AP_SM_BYTES = AP_TM * 8, AP_U_BYTES = AP_TN * AP_U_PITCH;
constexpr int AP_STAGE_BYTES = AP_SV_BYTES + AP_SM_BYTES + AP_U_BYTES;
constexpr int AP_V_PITCH = 272;   // epilogue: bytes per token row of a wave's V patch (128 bf16 + 16 pad)
constexpr int AP_V_BYTES = 8 * 64 * AP_V_PITCH;
constexpr int AP_LDS_BYTES = 2 * AP_STAGE_BYTES > AP_V_BYTES ? 2 * AP_STAGE_BYTES : AP_V_BYTES;

template <int B>
__global__ __launch_bounds__(512) void apply_main_kernel(const uint16_t *__restrict__ U, int64_t n, int64_t d_in,
                                                         int64_t d_out, const uint16_t *__restrict__ Sv,
                                                         const uint8_t *__restrict__ Sm,
                                                         const uint16_t *__restrict__ Aw, uint16_t *__restrict__ Y,
                                                         int n_row_tiles, int n_tok_tiles) {
    __shared__ __attribute__((aligned(16))) uint8_t lds[AP_LDS_BYTES];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, l32 = lane & 31, half = lane >> 5;
    const int wm = w & 1, wn = w >> 1;
    // Workgroups go to the 8 XCDs round-robin, each XCD with its own L2.  The 32 workgroups that are
    // resident on one XCD together work on a super-tile of 8 row tiles x 4 token tiles, so that per
    // stage the XCD fetches 8 + 4 operand tiles instead of 32 + 32.
    int row_tile, tok_tile;
    {
        const int xcd = blockIdx.x & 7, seq = blockIdx.x >> 3, sup = (seq >> 5) * 8 + xcd, within = seq & 31;
        const int sup_rows = (n_row_tiles + AP_SUP_R - 1) / AP_SUP_R;
        row_tile = (sup % sup_rows) * AP_SUP_R + (within % AP_SUP_R);
        tok_tile = (sup / sup_rows) * AP_SUP_T + (within / AP_SUP_R);
    }
    if (row_tile >= n_row_tiles || tok_tile >= n_tok_tiles) return; // uniform for the workgroup
    const int64_t row0 = (int64_t)row_tile * AP_TM, tok0 = (int64_t)tok_tile * AP_TN;
    const int64_t val_pitch = d_in / 2 /* bf16 per row */, meta_pitch = d_in / 8 /* bytes per row */;

    // ---- loader assignment (global -> registers -> LDS): 16-byte chunks, consecutive threads on
    // consecutive chunks of a row ----
    const uint16_t *sv_src0 = Sv + min(row0 + (tid >> 2), d_out - 1) * val_pitch + (tid & 3) * 8;
    const uint16_t *sv_src1 = Sv + min(row0 + (tid >> 2) + 128, d_out - 1) * val_pitch + (tid & 3) * 8;
    const int sv_dst = (tid >> 2) * AP_SV_PITCH + (tid & 3) * 16; // second chunk: + 128 rows
    const uint16_t *u_src0 = U + min(tok0 + (tid >> 3), n - 1) * d_in + (tid & 7) * 8;
    const uint16_t *u_src1 = U + min(tok0 + (tid >> 3) + 64, n - 1) * d_in + (tid & 7) * 8;
    const uint16_t *u_src2 = U + min(tok0 + (tid >> 3) + 128, n - 1) * d_in + (tid & 7) * 8;
    const uint16_t *u_src3 = U + min(tok0 + (tid >> 3) + 192, n - 1) * d_in + (tid & 7) * 8;
    const int u_dst = AP_SV_BYTES + AP_SM_BYTES + (tid >> 3) * AP_U_PITCH + (tid & 7) * 16; // + 64 token rows each
    const uint8_t *sm_src = Sm + min(row0 + (tid & 255), d_out - 1) * meta_pitch;
    const int sm_dst = AP_SV_BYTES + (tid & 255) * 8;

    uint4 pv0, pv1, pu0, pu1, pu2, pu3;
    uint2 pm = make_uint2(0u, 0u);
#define AP_GLOAD(k0)                                                                            \
    {                                                                                           \
        pv0 = *reinterpret_cast<const uint4 *>(sv_src0 + (k0) / 2);                             \
        pv1 = *reinterpret_cast<const uint4 *>(sv_src1 + (k0) / 2);                             \
        pu0 = *reinterpret_cast<const uint4 *>(u_src0 + (k0));                                  \
        pu1 = *reinterpret_cast<const uint4 *>(u_src1 + (k0));                                  \
        pu2 = *reinterpret_cast<const uint4 *>(u_src2 + (k0));                                  \
        pu3 = *reinterpret_cast<const uint4 *>(u_src3 + (k0));                                  \
        if (tid < 256) pm = *reinterpret_cast<const uint2 *>(sm_src + (k0) / 8);                \
    }
#define AP_LSTORE(stage)                                                                        \
    {                                                                                           \
        uint8_t *sb = lds + (stage) * AP_STAGE_BYTES;                                           \
        *reinterpret_cast<uint4 *>(sb + sv_dst) = pv0;                                          \
        *reinterpret_cast<uint4 *>(sb + sv_dst + 128 * AP_SV_PITCH) = pv1;                      \
        *reinterpret_cast<uint4 *>(sb + u_dst) = pu0;                                           \
        *reinterpret_cast<uint4 *>(sb + u_dst + 64 * AP_U_PITCH) = pu1;                         \
        *reinterpret_cast<uint4 *>(sb + u_dst + 128 * AP_U_PITCH) = pu2;                        \
        *reinterpret_cast<uint4 *>(sb + u_dst + 192 * AP_U_PITCH) = pu3;                        \
        if (tid < 256) *reinterpret_cast<uint2 *>(sb + sm_dst) = pm;                            \
    }

    floatx16 acc[4][2];
#pragma unroll
    for (int tm = 0; tm < 4; ++tm)
#pragma unroll
        for (int tn = 0; tn < 2; ++tn)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[tm][tn][r] = 0.f;

    const int a_off = (128 * wm + l32) * AP_SV_PITCH + half * 16;
    const int m_off = AP_SV_BYTES + (128 * wm + l32) * 8;
    const int b_off = AP_SV_BYTES + AP_SM_BYTES + (64 * wn + l32) * AP_U_PITCH + half * 16;

    AP_GLOAD((int64_t)0);
    AP_LSTORE(0);
    __syncthreads();
    const int nstages = (int)(d_in / AP_KT);
    for (int st = 0; st < nstages; ++st) {
        const uint8_t *base = lds + (st & 1) * AP_STAGE_BYTES;
        if (st + 1 < nstages) AP_GLOAD((int64_t)(st + 1) * AP_KT);
        uint2 meta[4];
#pragma unroll
        for (int tm = 0; tm < 4; ++tm) meta[tm] = *reinterpret_cast<const uint2 *>(base + m_off + tm * 32 * 8);
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            bf16x8 a[4];
            bf16x16 b[2];
            int idx[4];
#pragma unroll
            for (int tm = 0; tm < 4; ++tm) {
                a[tm] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(base + a_off + tm * 32 * AP_SV_PITCH + s * 32));
                const uint32_t word = s == 0 ? meta[tm].x : meta[tm].y; // 32 index bits of this 32-k step
                const uint32_t f = (word >> (16 * half)) & 0xffffu;
                idx[tm] = (int)(f | (f << 16));
            }
#pragma unroll
            for (int tn = 0; tn < 2; ++tn) {
                const bf16x8 lo = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(base + b_off + tn * 32 * AP_U_PITCH + s * 64));
                const bf16x8 hi = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(base + b_off + tn * 32 * AP_U_PITCH + s * 64 + 32));
                b[tn] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15);
            }
#pragma unroll
            for (int tm = 0; tm < 4; ++tm)
#pragma unroll
                for (int tn = 0; tn < 2; ++tn)
                    acc[tm][tn] = __builtin_amdgcn_smfmac_f32_32x32x32_bf16(a[tm], b[tn], acc[tm][tn], idx[tm], 0, 0);
        }
        if (st + 1 < nstages) AP_LSTORE((st + 1) & 1);
        __syncthreads();
    }
#undef AP_GLOAD
#undef AP_LSTORE

    // ---- epilogue: V patch -> LDS [token][q] bf16, then Y = V A^T per block of A ----
    uint8_t *vbuf = lds + w * (64 * AP_V_PITCH);
#pragma unroll
    for (int tm = 0; tm < 4; ++tm)
#pragma unroll
        for (int tn = 0; tn < 2; ++tn)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                uint2 pk;
                pk.x = pack_bf16x2_rne(acc[tm][tn][4 * g], acc[tm][tn][4 * g + 1]);
                pk.y = pack_bf16x2_rne(acc[tm][tn][4 * g + 2], acc[tm][tn][4 * g + 3]);
                *reinterpret_cast<uint2 *>(vbuf + (32 * tn + l32) * AP_V_PITCH + (32 * tm + 8 * g + 4 * half) * 2) = pk;
            }
    __syncthreads();
    const int64_t prow0 = row0 + 128 * wm; // first output column (row of S) of this wave
#pragma unroll
    for (int pt = 0; pt < 4; ++pt) {
        const int q0 = (pt * 32 / B) * B; // first q of the block of A that holds these 32 columns
        const int64_t prow = prow0 + pt * 32 + l32;
        const int64_t pclamped = min(prow, d_out - 1);
        const uint16_t *arow = Aw + pclamped * B + 8 * half; // A^i[p][q]: (i*b + p)*b + q = prow*b + (q - q0)
        floatx16 o[2];
#pragma unroll
        for (int tn = 0; tn < 2; ++tn)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[tn][r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < B / 16; ++ks) {
            const bf16x8 bb = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(arow + 16 * ks));
#pragma unroll
            for (int tn = 0; tn < 2; ++tn) {
                const bf16x8 a = __builtin_bit_cast(
                    bf16x8, *reinterpret_cast<const uint4 *>(vbuf + (32 * tn + l32) * AP_V_PITCH + (q0 + 16 * ks + 8 * half) * 2));
                o[tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bb, o[tn], 0, 0, 0);
            }
        }
        if (prow < d_out) {
#pragma unroll
            for (int tn = 0; tn < 2; ++tn)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int64_t t = tok0 + 64 * wn + 32 * tn + 8 * (r >> 2) + 4 * half + (r & 3);
                    if (t < n) Y[t * d_out + prow] = (uint16_t)(pack_bf16x2_rne(o[tn][r], 0.f) & 0xffffu);
                }
        }
    }
}

hipError_t launch_apply_main(const void *U, int64_t n, int64_t d_in, int64_t d_out, int b, const void *Sv,
                             const uint8_t *Sm, const void *Aw, void *Y, hipStream_t s) {
    const int n_row_tiles = (int)((d_out + AP_TM - 1) / AP_TM), n_tok_tiles = (int)((n + AP_TN - 1) / AP_TN);
    const int sups = ((n_row_tiles + AP_SUP_R - 1) / AP_SUP_R) * ((n_tok_tiles + AP_SUP_T - 1) / AP_SUP_T);
    dim3 grid((unsigned)(((sups + 7) / 8) * 8 * 32)), block(512);
    const uint16_t *u = reinterpret_cast<const uint16_t *>(U), *sv = reinterpret_cast<const uint16_t *>(Sv),
                   *aw = reinterpret_cast<const uint16_t *>(Aw);
    uint16_t *y = reinterpret_cast<uint16_t *>(Y);
    switch (b) {
    case 32: hipLaunchKernelGGL(apply_main_kernel<32>, grid, block, 0, s, u, n, d_in, d_out, sv, Sm, aw, y, n_row_tiles, n_tok_tiles); break;
    case 64: hipLaunchKernelGGL(apply_main_kernel<64>, grid, block, 0, s, u, n, d_in, d_out, sv, Sm, aw, y, n_row_tiles, n_tok_tiles); break;
    case 128: hipLaunchKernelGGL(apply_main_kernel<128>, grid, block, 0, s, u, n, d_in, d_out, sv, Sm, aw, y, n_row_tiles, n_tok_tiles); break;
    default: return hipErrorInvalidValue;
    }
    return hipSuccess;
}

} // namespace armor
