// The factorized layer applied to a batch of activations (Sec. 3.1: y = A (S (B x)), the wrappers as
// batched block products around the 2:4 core; Sec. 4.4 times this on a batch of tokens).
// bf16 operands, fp32 accumulation, the two intermediates rounded to bf16.  gfx950:
//   apply_prepare_kernel  one-off re-tiling of the compressed core (values + 2-bit in-group columns
//                      of armor_pack_nm) into the order the product streams it in;
//   apply_pre_kernel   U = X B^T (block-diagonal), dense v_mfma_f32_32x32x16_bf16, operands straight
//                      from global memory (the kernel is bound by reading X and writing U once);
//   apply_main_kernel  Y = (U S^T) A^T: the core product on the 2:4 structured-sparse matrix
//                      instruction v_smfmac_f32_32x32x32_bf16 (the compressed values and the 2-bit
//                      in-group columns are exactly its sparse operand and index), then the A
//                      wrapper as an epilogue on the accumulator tile.
//
// Streaming layout ("stage-major"): the product consumes 64 dense k per stage.  For stage s the
// 64 B of compressed values of every row are contiguous ([s][row][64 B]), likewise the 8 B of index
// bits ([s][row][8 B]) and the 128 B of activations of every token ([s][token][128 B]); rows and
// tokens are padded to a multiple of 256.  A tile-stage is then one contiguous run of whole cache
// lines (16 KB + 2 KB + 32 KB) instead of 768 separately requested lines.  Inside a row the 16-byte
// parts are stored permuted (part p of row r sits in slot p ^ key(r)) so that the 16-byte operand
// reads from LDS, where the rows land unpadded, are free of bank conflicts.
#include "armor_internal.h"

namespace armor {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x16 __attribute__((ext_vector_type(16)));

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx2 __attribute__((ext_vector_type(2)));

// two floats -> two bf16 (round to nearest even) in one register: v_cvt_pk_bf16_f32
__device__ __forceinline__ uint32_t pack_bf16x2_rne(float lo, float hi) {
    const floatx2 f = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));
}

__global__ __launch_bounds__(256) void to_bf16_kernel(const float *__restrict__ in, int64_t n, uint16_t *__restrict__ out) {
    int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e < n) out[e] = (uint16_t)(pack_bf16x2_rne(in[e], 0.f) & 0xffffu);
}

void launch_to_bf16(const float *in, int64_t n, void *out, hipStream_t s) {
    hipLaunchKernelGGL(to_bf16_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, in, n,
                       reinterpret_cast<uint16_t *>(out));
}

// slot permutation keys: 16 consecutive rows (8 for the narrower LDS of older parts) read 16 bytes each
// from distinct bank groups
__device__ __forceinline__ int key_values(int r) { return ((r >> 2) ^ (r >> 1)) & 3; }        // 4 parts of 16 B per row
__device__ __forceinline__ int key_acts(int t) { return ((t >> 1) ^ ((t & 1) << 2)) & 7; }   // 8 parts of 16 B per row

__host__ __device__ inline int64_t pad256(int64_t x) { return (x + 255) / 256 * 256; }

// prepared = [stages][rows_pad][64 B] values, then [stages][rows_pad][8 B] index bits
__global__ __launch_bounds__(256) void apply_prepare_kernel(const uint16_t *__restrict__ values,
                                                            const uint8_t *__restrict__ meta, int64_t d_out,
                                                            int64_t d_in, uint8_t *__restrict__ prepared) {
    const int64_t rows_pad = pad256(d_out), stages = d_in / 64;
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; // one 16-byte slot of the values per thread
    if (e >= stages * rows_pad * 4) return;
    const int slot = (int)(e & 3);
    const int64_t r = (e >> 2) % rows_pad, s = (e >> 2) / rows_pad;
    uint4 v = make_uint4(0u, 0u, 0u, 0u);
    if (r < d_out) v = *reinterpret_cast<const uint4 *>(values + r * (d_in / 2) + s * 32 + (slot ^ key_values((int)r)) * 8);
    reinterpret_cast<uint4 *>(prepared)[e] = v;
    if (slot == 0) {
        uint2 m = make_uint2(0u, 0u);
        if (r < d_out) m = *reinterpret_cast<const uint2 *>(meta + r * (d_in / 8) + s * 8);
        reinterpret_cast<uint2 *>(prepared + stages * rows_pad * 64)[s * rows_pad + r] = m;
    }
}

int64_t apply_prepared_bytes(int64_t d_out, int64_t d_in) { return (d_in / 64) * pad256(d_out) * 72; }
int64_t apply_acts_bytes(int64_t n, int64_t d_in) { return (d_in / 64) * pad256(n) * 128; }

void launch_apply_prepare(const void *values, const uint8_t *meta, int64_t d_out, int64_t d_in, void *prepared,
                          hipStream_t s) {
    const int64_t total = (d_in / 64) * pad256(d_out) * 4;
    hipLaunchKernelGGL(apply_prepare_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s,
                       reinterpret_cast<const uint16_t *>(values), meta, d_out, d_in, reinterpret_cast<uint8_t *>(prepared));
}

// 4 x 4 transpose inside every quad of lanes (x[i] of lane j <-> x[j] of lane i), two rounds of
// neighbour swaps with DPP quad permutations
__device__ __forceinline__ void quad_transpose(float (&x)[4], int lane) {
    const bool b0 = lane & 1, b1 = lane & 2;
#pragma unroll
    for (int a = 0; a < 4; a += 2) { // pairs (0,1), (2,3) with the lane whose bit 0 differs
        const float send = b0 ? x[a] : x[a + 1];
        const float recv = __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, send), 0xB1, 0xF, 0xF, true));
        if (b0) x[a] = recv; else x[a + 1] = recv;
    }
#pragma unroll
    for (int a = 0; a < 2; ++a) { // pairs (0,2), (1,3) with the lane whose bit 1 differs
        const float send = b1 ? x[a] : x[a + 2];
        const float recv = __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, send), 0x4E, 0xF, 0xF, true));
        if (b1) x[a] = recv; else x[a + 2] = recv;
    }
}

// ------------------------------------------------------------------------------------------------
// U[t][j*b + p] = sum_q B^j[p][q] X[t][j*b + q].   Workgroup: block j x 256 tokens (4 waves x 64).
// MFMA rows = tokens (operand from X: 8 consecutive q per lane, straight from global memory),
// columns = p (operand from B^j, staged once per workgroup in LDS).  A lane of the result holds
// one column p of 16 token rows; a transpose inside each quad of lanes turns that into 4
// consecutive columns of one row, stored as 8 bytes.  U is written in the stage-major layout
// described at the top: [column / 64][token][128 B], 16-byte parts permuted.
// ------------------------------------------------------------------------------------------------
template <int B>
__global__ __launch_bounds__(256) void apply_pre_kernel(const uint16_t *__restrict__ X, int64_t n, int64_t d_in,
                                                        const uint16_t *__restrict__ Bw, uint8_t *__restrict__ U,
                                                        int64_t n_pad) {
    constexpr int PT = B / 32, KS = B / 16; // column tiles, k steps
    constexpr int PITCH = B * 2 + 16;       // LDS bytes per row of B^j
    __shared__ __attribute__((aligned(16))) uint8_t lb[B * PITCH];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, l32 = lane & 31, half = lane >> 5;
    const int j = blockIdx.y;
    const int64_t t0 = (int64_t)blockIdx.x * 256 + w * 64;
    // The wave's two 32-token row tiles are processed together while operands and accumulators fit in
    // the register file (b <= 128), one after the other at b = 256.
    constexpr int RT = B <= 128 ? 2 : 1;
    // X operands of this wave first (the long latency), then B^j -> LDS underneath
    uint4 xa[RT][KS];
    auto load_x = [&](int rt0) {
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            const int64_t trow = min(t0 + 32 * (rt0 + rt) + l32, n - 1); // clamped: rows past the end are computed and dropped
            const uint16_t *xrow = X + trow * d_in + (int64_t)j * B + 8 * half;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) xa[rt][ks] = *reinterpret_cast<const uint4 *>(xrow + 16 * ks);
        }
    };
    load_x(0);
    {
        const uint16_t *bj = Bw + (int64_t)j * B * B;
        constexpr int CH = B * B / 8; // 16-byte chunks
#pragma unroll
        for (int c = tid; c < CH; c += 256) {
            const int row = c / (B / 8), part = c % (B / 8);
            *reinterpret_cast<uint4 *>(lb + row * PITCH + part * 16) = *reinterpret_cast<const uint4 *>(bj + row * B + part * 8);
        }
    }
    __syncthreads();
    const int q4 = lane & 3; // after the transpose this lane holds row (4g + q4) of each group of 4 rows
#pragma unroll 1
    for (int rt0 = 0; rt0 < 2; rt0 += RT) {
        if (rt0 > 0) load_x(rt0);
        floatx16 acc[RT][PT];
#pragma unroll
        for (int rt = 0; rt < RT; ++rt)
#pragma unroll
            for (int pt = 0; pt < PT; ++pt)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[rt][pt][r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
            for (int pt = 0; pt < PT; ++pt) {
                const bf16x8 bb = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(lb + (pt * 32 + l32) * PITCH + (16 * ks + 8 * half) * 2));
#pragma unroll
                for (int rt = 0; rt < RT; ++rt)
                    acc[rt][pt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, xa[rt][ks]), bb, acc[rt][pt], 0, 0, 0);
            }
            // b = 256: keep the scheduler from hoisting all 128 operand reads above the matrix work
            if (B > 128 && (ks & 1)) __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int rt = 0; rt < RT; ++rt)
#pragma unroll
            for (int pt = 0; pt < PT; ++pt)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    float x[4] = {acc[rt][pt][4 * g], acc[rt][pt][4 * g + 1], acc[rt][pt][4 * g + 2], acc[rt][pt][4 * g + 3]};
                    quad_transpose(x, lane);
                    const int64_t t = t0 + 32 * (rt0 + rt) + 8 * g + 4 * half + q4;
                    const int64_t col = (int64_t)j * B + pt * 32 + (l32 & ~3); // first of the 4 columns
                    const int within = (int)(col & 63), slot = (within >> 3) ^ key_acts((int)(t & 255));
                    uint2 pk;
                    pk.x = pack_bf16x2_rne(x[0], x[1]);
                    pk.y = pack_bf16x2_rne(x[2], x[3]);
                    if (t < n) *reinterpret_cast<uint2 *>(U + ((col >> 6) * n_pad + t) * 128 + slot * 16 + (within & 7) * 2) = pk;
                }
    }
}

void launch_apply_pre(const void *X, int64_t n, int64_t d_in, int b, const void *Bw, void *U, hipStream_t s) {
    dim3 grid((unsigned)((n + 255) / 256), (unsigned)(d_in / b));
    const uint16_t *x = reinterpret_cast<const uint16_t *>(X), *bw = reinterpret_cast<const uint16_t *>(Bw);
    uint8_t *u = reinterpret_cast<uint8_t *>(U);
    const int64_t n_pad = pad256(n);
    switch (b) {
    case 32: hipLaunchKernelGGL(apply_pre_kernel<32>, grid, dim3(256), 0, s, x, n, d_in, bw, u, n_pad); break;
    case 64: hipLaunchKernelGGL(apply_pre_kernel<64>, grid, dim3(256), 0, s, x, n, d_in, bw, u, n_pad); break;
    case 128: hipLaunchKernelGGL(apply_pre_kernel<128>, grid, dim3(256), 0, s, x, n, d_in, bw, u, n_pad); break;
    case 256: hipLaunchKernelGGL(apply_pre_kernel<256>, grid, dim3(256), 0, s, x, n, d_in, bw, u, n_pad); break;
    default: break;
    }
}

// ------------------------------------------------------------------------------------------------
// Y[t][o] = sum_q A^i[p][q] V[t][i*b + q],  V[t][o] = sum_k S[o][k] U[t][k]  (V rounded to bf16).
// Workgroup: 256 rows of S x 256 tokens, 8 waves as 2 (rows) x 4 (tokens), a wave owns 128 x 64
// (4 x 2 accumulator tiles).  Per stage of 64 dense k the compressed values (256 x 64 B), their
// index bits (256 x 8 B) and the activations (256 x 128 B) are loaded from global memory straight
// into LDS (global_load_lds, 16 B per lane; no register staging), three LDS slots, two stages in
// flight while one is consumed; one barrier per stage.  Both operands arrive in the stage-major
// layout, so every load instruction copies 1 KB of consecutive bytes; the slot permutation inside a
// row is already in the data and the reader applies the same XOR.
// Sparse operand of the instruction: lane (row, h) = the 8 kept values of dense k in [16h, 16h+16)
// of the 32-k step and their 16 index bits; dense operand: lane (token, h) = k in [8h, 8h+8) and
// [16+8h, 16+8h+8).
// Epilogue: each wave's V patch is written to LDS as [token][q] bf16 and multiplied by A^i with the
// dense bf16 instruction (rows = tokens, columns = p), stored like the kernel above.  Up to b = 128
// a wave's 128 rows are whole blocks of A and it needs only its own patch; at b = 256 the tile is
// one block of A and a wave also reads the patch of the wave that holds the other 128 rows of the
// same tokens.
// ------------------------------------------------------------------------------------------------
constexpr int AP_TM = 256, AP_TN = 256, AP_KT = 64;
constexpr int AP_SUP_R = 8, AP_SUP_T = 4; // super-tile of one XCD: 8 row tiles x 4 token tiles = 32 workgroups
constexpr int AP_SV_BYTES = AP_TM * 64, AP_SM_BYTES = AP_TM * 8, AP_U_BYTES = AP_TN * 128;
constexpr int AP_SM_OFF = AP_SV_BYTES, AP_U_OFF = AP_SV_BYTES + AP_SM_BYTES;
constexpr int AP_SLOT_BYTES = AP_SV_BYTES + AP_SM_BYTES + AP_U_BYTES; // 51200
constexpr int AP_SLOTS = 3;
constexpr int AP_V_PITCH = 272;   // epilogue: bytes per token row of a wave's V patch (128 bf16 + 16 pad)
constexpr int AP_V_BYTES = 8 * 64 * AP_V_PITCH;
constexpr int AP_LDS_BYTES = AP_SLOTS * AP_SLOT_BYTES > AP_V_BYTES ? AP_SLOTS * AP_SLOT_BYTES : AP_V_BYTES;
constexpr int AP_DMA_PER_STAGE = 7; // load instructions per wave per stage: 2 (values) + 4 (activations) + 1 (index bits)

typedef __attribute__((address_space(3))) void *lds_ptr_t;

// One global -> LDS load instruction: every lane fetches 16 (or 4) bytes from its own global address,
// the wave's 64 pieces land contiguously at the wave-uniform LDS byte address held in M0.  Issued as
// inline assembly on purpose: the compiler then keeps no book on these loads, so it does not make the
// operand reads of the stage being consumed wait for the stages still in flight; completion is waited
// for explicitly (s_waitcnt vmcnt) before the barrier that publishes a stage.
__device__ __forceinline__ void dma_load16(const void *g, uint32_t lds_byte_addr) {
    asm volatile("s_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "{m0}"(lds_byte_addr) : "memory");
}
__device__ __forceinline__ void dma_load4(const void *g, uint32_t lds_byte_addr) {
    asm volatile("s_nop 0\n\tglobal_load_lds_dword %0, off" ::"v"(g), "{m0}"(lds_byte_addr) : "memory");
}

// s_waitcnt vmcnt(n) alone (expcnt and lgkmcnt fields left at "no wait")
#define AP_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(0x0f70 | ((n) & 15) | (((n) >> 4) << 14))
// workgroup barrier that the compiler may not move memory accesses across, without the fence of
// __syncthreads (a fence would wait for every outstanding load, including the stages in flight)
#define AP_BARRIER()                        \
    {                                       \
        asm volatile("" ::: "memory");      \
        __builtin_amdgcn_s_barrier();       \
        asm volatile("" ::: "memory");      \
    }

template <int B>
__global__ __launch_bounds__(512) void apply_main_kernel(const uint8_t *__restrict__ U, int64_t n, int64_t d_in,
                                                         int64_t d_out, const uint8_t *__restrict__ prepared,
                                                         const uint16_t *__restrict__ Aw, uint16_t *__restrict__ Y,
                                                         int n_row_tiles, int n_tok_tiles) {
    __shared__ __attribute__((aligned(16))) uint8_t lds[AP_LDS_BYTES];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, l32 = lane & 31, half = lane >> 5;
    const int wm = w & 1, wn = w >> 1;
    // Workgroups go to the 8 XCDs round-robin, each XCD with its own L2.  The grid is persistent (one
    // workgroup per CU); in round k the 32 workgroups of XCD x work on super-tile 8k + x, 8 row tiles x
    // 4 token tiles, so that per stage the XCD fetches 8 + 4 operand tiles instead of 32 + 32.
    const int xcd = blockIdx.x & 7, within = (blockIdx.x >> 3) & 31, wg_round0 = blockIdx.x >> 8;
    const int sup_rows = (n_row_tiles + AP_SUP_R - 1) / AP_SUP_R, sup_cols = (n_tok_tiles + AP_SUP_T - 1) / AP_SUP_T;
    const int rounds_stride = (int)(gridDim.x >> 8);
    for (int round = wg_round0; round * 8 + xcd < sup_rows * sup_cols; round += rounds_stride) {
    const int sup = round * 8 + xcd;
    const int row_tile = (sup % sup_rows) * AP_SUP_R + (within % AP_SUP_R);
    const int tok_tile = (sup / sup_rows) * AP_SUP_T + (within / AP_SUP_R);
    if (row_tile >= n_row_tiles || tok_tile >= n_tok_tiles) continue; // uniform for the workgroup
    const int64_t row0 = (int64_t)row_tile * AP_TM, tok0 = (int64_t)tok_tile * AP_TN;
    const int64_t rows_pad = (int64_t)n_row_tiles * AP_TM, n_pad = (int64_t)n_tok_tiles * AP_TN;
    const int64_t nst = d_in / AP_KT;

    // ---- this lane's share of a stage: 1 KB runs of the stage-major operands (padded: no edge cases) ----
    const uint8_t *sv_src = prepared + (row0 + 32 * w) * 64 + lane * 16;                       // + stage * rows_pad * 64, + 1024
    const uint8_t *sm_src = prepared + nst * rows_pad * 64 + (row0 + 32 * w) * 8 + lane * 4;   // + stage * rows_pad * 8
    const uint8_t *u_src = U + (tok0 + 32 * w) * 128 + lane * 16;                              // + stage * n_pad * 128, + c * 1024

    const uint32_t lds0 = (uint32_t)(size_t)(lds_ptr_t)lds; // LDS byte address of the buffer
#define AP_ISSUE(stage)                                                                    \
    {                                                                                      \
        const uint32_t sb = lds0 + ((stage) % AP_SLOTS) * AP_SLOT_BYTES;                   \
        const uint8_t *sv = sv_src + (int64_t)(stage) * rows_pad * 64;                     \
        const uint8_t *uu = u_src + (int64_t)(stage) * n_pad * 128;                        \
        dma_load16(sv, sb + (2 * w) * 1024);                                               \
        dma_load16(sv + 1024, sb + (2 * w + 1) * 1024);                                    \
        dma_load16(uu, sb + AP_U_OFF + (4 * w) * 1024);                                    \
        dma_load16(uu + 1024, sb + AP_U_OFF + (4 * w + 1) * 1024);                         \
        dma_load16(uu + 2048, sb + AP_U_OFF + (4 * w + 2) * 1024);                         \
        dma_load16(uu + 3072, sb + AP_U_OFF + (4 * w + 3) * 1024);                         \
        dma_load4(sm_src + (int64_t)(stage) * rows_pad * 8, sb + AP_SM_OFF + w * 256);     \
    }

    floatx16 acc[4][2];
#pragma unroll
    for (int tm = 0; tm < 4; ++tm)
#pragma unroll
        for (int tn = 0; tn < 2; ++tn)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[tm][tn][r] = 0.f;

    // reader offsets inside a slot (the keys use row bits 0..3 only and tile offsets are multiples of 32 rows)
    int a_off[2], b_off[2][2];
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        a_off[s] = (128 * wm + l32) * 64 + (((2 * s + half) ^ key_values(l32)) * 16);
        b_off[s][0] = AP_U_OFF + (64 * wn + l32) * 128 + (((4 * s + half) ^ key_acts(l32)) * 16);
        b_off[s][1] = AP_U_OFF + (64 * wn + l32) * 128 + (((4 * s + 2 + half) ^ key_acts(l32)) * 16);
    }
    const int m_off = AP_SM_OFF + (128 * wm + l32) * 8;

    // one stage of matrix work; meta words: 32 index bits per 32-k step (x: first step, y: second)
#define AP_COMPUTE(st)                                                                   \
    {                                                                                    \
        const uint8_t *base = lds + ((st) % AP_SLOTS) * AP_SLOT_BYTES;                               \
        uint2 meta[4];                                                                               \
_Pragma("unroll")                                                                                    \
        for (int tm = 0; tm < 4; ++tm) meta[tm] = *reinterpret_cast<const uint2 *>(base + m_off + tm * 32 * 8); \
_Pragma("unroll")                                                                                    \
        for (int s = 0; s < 2; ++s) {                                                                \
            bf16x8 a[4];                                                                             \
            bf16x16 b[2];                                                                            \
            int idx[4];                                                                              \
_Pragma("unroll")                                                                                    \
            for (int tm = 0; tm < 4; ++tm) {                                                         \
                a[tm] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(base + a_off[s] + tm * 32 * 64)); \
                const uint32_t word = s == 0 ? meta[tm].x : meta[tm].y;                              \
                const uint32_t f = (word >> (16 * half)) & 0xffffu;                                  \
                idx[tm] = (int)(f | (f << 16));                                                      \
            }                                                                                        \
_Pragma("unroll")                                                                                    \
            for (int tn = 0; tn < 2; ++tn) {                                                         \
                const bf16x8 lo = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(base + b_off[s][0] + tn * 32 * 128)); \
                const bf16x8 hi = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(base + b_off[s][1] + tn * 32 * 128)); \
                b[tn] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15); \
            }                                                                                        \
_Pragma("unroll")                                                                                    \
            for (int tm = 0; tm < 4; ++tm)                                                           \
_Pragma("unroll")                                                                                    \
                for (int tn = 0; tn < 2; ++tn)                                                       \
                    acc[tm][tn] = __builtin_amdgcn_smfmac_f32_32x32x32_bf16(a[tm], b[tn], acc[tm][tn], idx[tm], 0, 0); \
        }                                                                                            \
    }

    const int nstages = (int)(d_in / AP_KT);
    AP_ISSUE(0);
    if (nstages > 1) AP_ISSUE(1);
    int st = 0;
    // steady state: stage st has landed once at most the loads of stage st+1 are outstanding; after the
    // barrier everyone is done reading stage st-1, whose slot takes stage st+2.  No branches in the trip.
    for (; st + 2 < nstages; ++st) {
        AP_WAIT_VMCNT(AP_DMA_PER_STAGE);
        AP_BARRIER();
        AP_ISSUE(st + 2);
        AP_COMPUTE(st);
    }
    for (; st < nstages; ++st) { // the last two stages: nothing left to issue
        if (st + 1 < nstages) { AP_WAIT_VMCNT(AP_DMA_PER_STAGE); } else { AP_WAIT_VMCNT(0); }
        AP_BARRIER();
        AP_COMPUTE(st);
    }
#undef AP_COMPUTE
#undef AP_ISSUE
    __syncthreads(); // every wave is done with the stage slots: the epilogue reuses them

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
    const int64_t prow0 = row0 + 128 * wm; // first output column (row of S) of this wave
    // wrapper operands: all of the wave's in one round of loads up to b = 128 (the accumulators are dead
    // by now), one 32-column tile at a time at b = 256 (64 registers each)
    constexpr int APT = B <= 128 ? 4 : 1, AKS = B / 16;
    uint4 afrag[APT][AKS];
    auto load_afrag = [&](int pt0) {
#pragma unroll
        for (int pt = 0; pt < APT; ++pt) {
            const int64_t pclamped = min(prow0 + (pt0 + pt) * 32 + l32, d_out - 1);
            // A^i[p][q] sits at (i*b + p)*b + q = prow*b + q, q counted from the block's first column
            const uint16_t *arow = Aw + pclamped * B + 8 * half;
#pragma unroll
            for (int ks = 0; ks < AKS; ++ks) afrag[pt][ks] = *reinterpret_cast<const uint4 *>(arow + 16 * ks);
        }
    };
    load_afrag(0);
    __syncthreads();
    // V patches by 128-row half of the tile: this wave's own and, at b = 256, its partner's (same tokens)
    const uint8_t *vhalf[2] = {lds + (0 + 2 * wn) * (64 * AP_V_PITCH), lds + (1 + 2 * wn) * (64 * AP_V_PITCH)};
#pragma unroll
    for (int pt = 0; pt < 4; ++pt) {
        if (APT == 1 && pt > 0) load_afrag(pt);
        const int q0 = B <= 128 ? (pt * 32 / B) * B : 0; // first q (in this wave's patch) of the block of A that holds these 32 columns
        const int64_t prow = prow0 + pt * 32 + l32;
        floatx16 o[2];
#pragma unroll
        for (int tn = 0; tn < 2; ++tn)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[tn][r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < AKS; ++ks) {
            const bf16x8 bb = __builtin_bit_cast(bf16x8, afrag[APT == 1 ? 0 : pt][ks]);
            // b <= 128: q0 + 16 ks lies in this wave's patch; b = 256: k steps 0..7 in the patch of rows 0..127, 8..15 in the other
            const uint8_t *vsrc = B <= 128 ? vbuf : vhalf[ks / 8];
            const int qoff = B <= 128 ? q0 + 16 * ks : 16 * (ks % 8);
#pragma unroll
            for (int tn = 0; tn < 2; ++tn) {
                const bf16x8 a = __builtin_bit_cast(
                    bf16x8, *reinterpret_cast<const uint4 *>(vsrc + (32 * tn + l32) * AP_V_PITCH + (qoff + 8 * half) * 2));
                o[tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bb, o[tn], 0, 0, 0);
            }
        }
        // A lane holds column p of 16 token rows.  Neighbouring lanes swap one value per pair of rows, so
        // that an even lane stores (p, p+1) of the first row and the odd lane (p-1, p) of the second:
        // 4-byte stores, 64 consecutive bytes of a token row per half-wave.
        const bool odd = lane & 1;
        if (prow < d_out) { // d_out is a multiple of 32: a pair of columns is inside or outside together
#pragma unroll
            for (int tn = 0; tn < 2; ++tn) {
                // first token row of this lane in the tile, and how many rows of the batch are left from there
                const int64_t tl = tok0 + 64 * wn + 32 * tn + 4 * half + (odd ? 1 : 0);
                const int left = (int)min((int64_t)64, n - tl);
                uint16_t *ybase = Y + tl * d_out + (prow & ~(int64_t)1);
#pragma unroll
                for (int r = 0; r < 16; r += 2) {
                    const float mine = odd ? o[tn][r + 1] : o[tn][r], send = odd ? o[tn][r] : o[tn][r + 1];
                    const float recv = __builtin_bit_cast(
                        float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, send), 0xB1 /* quad_perm [1,0,3,2] */, 0xF, 0xF, true));
                    const int roff = 8 * (r >> 2) + (r & 3); // row offset from tl (same for both lanes of a pair)
                    const uint32_t pk = odd ? pack_bf16x2_rne(recv, mine) : pack_bf16x2_rne(mine, recv);
                    if (roff < left) *reinterpret_cast<uint32_t *>(ybase + (int64_t)roff * d_out) = pk;
                }
            }
        }
    }
    __syncthreads(); // the next tile's loads overwrite the patch buffers
    } // tiles of this workgroup
}

hipError_t launch_apply_main(const void *U, int64_t n, int64_t d_in, int64_t d_out, int b, const void *prepared,
                             const void *Aw, void *Y, hipStream_t s) {
    const int n_row_tiles = (int)((d_out + AP_TM - 1) / AP_TM), n_tok_tiles = (int)((n + AP_TN - 1) / AP_TN);
    const int sups = ((n_row_tiles + AP_SUP_R - 1) / AP_SUP_R) * ((n_tok_tiles + AP_SUP_T - 1) / AP_SUP_T);
    // persistent grid: 256 workgroups (one per CU, 32 per XCD) walk the super-tiles
    (void)sups;
    dim3 grid(256), block(512);
    const uint8_t *u = reinterpret_cast<const uint8_t *>(U), *pr = reinterpret_cast<const uint8_t *>(prepared);
    const uint16_t *aw = reinterpret_cast<const uint16_t *>(Aw);
    uint16_t *y = reinterpret_cast<uint16_t *>(Y);
    switch (b) {
    case 32: hipLaunchKernelGGL(apply_main_kernel<32>, grid, block, 0, s, u, n, d_in, d_out, pr, aw, y, n_row_tiles, n_tok_tiles); break;
    case 64: hipLaunchKernelGGL(apply_main_kernel<64>, grid, block, 0, s, u, n, d_in, d_out, pr, aw, y, n_row_tiles, n_tok_tiles); break;
    case 128: hipLaunchKernelGGL(apply_main_kernel<128>, grid, block, 0, s, u, n, d_in, d_out, pr, aw, y, n_row_tiles, n_tok_tiles); break;
    case 256: hipLaunchKernelGGL(apply_main_kernel<256>, grid, block, 0, s, u, n, d_in, d_out, pr, aw, y, n_row_tiles, n_tok_tiles); break;
    default: return hipErrorInvalidValue;
    }
    return hipSuccess;
}

} // namespace armor
