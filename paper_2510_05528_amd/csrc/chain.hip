// Fused per-block contraction chains of the continuous step (Alg. 2, App. D) and of the core
// gradient that feeds the sparse-core step (Alg. 3), for gfx950.
//
// The proxy loss splits over the b x b blocks of the weight matrix (Eq. 5), and so does every
// product of the iteration: block (i,j) only touches C^(i,j), Wbar^(i,j), A^(i), B^(j), D^(j).
// One workgroup owns one block at a time and runs the whole chain of b x b x b products on it with
// the operand tiles resident in LDS (two tiles of b x (b+1) fp32; the odd pitch makes row-wise and
// column-wise MFMA operand reads both bank-conflict free, so a tile can serve as either operand,
// transposed or not).  Products run on v_mfma_f32_32x32x2_f32; each wave owns a (TM*32) x (TN*32)
// patch of the b x b result in accumulator registers.  Only C, Wbar (HBM) and A^i, B^j (L2) are
// read per block; intermediates never leave the CU.
// At b = 128 the A, B and W' phases and the two joint-Adam chains run in a second form
// (chain_stream.hip: one operand tile in LDS, the other streamed, two workgroups per CU); the kernels
// here serve b = 32 and 64, and at b = 128 the loss-only pass and the wrapper Grams.  The b = 128
// geometry of chain_common.h (8 waves) is also what the sub-tiled b = 256 chains are built on.
#include "chain_common.h"

#include <algorithm>
#include <cmath>

namespace armor {

// ------------------------------------------------------------------------------------------------
// Scheduling common to the three chains below: every global read of an operand tile is issued
// into registers one matrix product before the tile is needed and only written to LDS after that
// product (gload_tile ... mma ... lstore_tile), Wbar is read straight into the accumulator layout
// underneath the product whose result it is subtracted from, and the first tiles of the next block
// are requested underneath the last product of the current one.  With one workgroup per CU (two
// 66 KB tiles fill LDS) this is what keeps HBM/L2 latency off the critical path.
// ------------------------------------------------------------------------------------------------

// ------------------------------------------------------------------------------------------------
// A-phase (Alg. 2, first gradient step; App. D.1).  Workgroup (i, c) walks the column blocks j of
// its chunk c and accumulates  sum_j (R D)^(i,j) S^(i,j)T  in registers.
//   gpart[(i*nsplit + c)][b][b] = -2 * that sum          (partial grad_A^(i))
//   beta_part[i*nbj + j] = || S^(i,j) D^(j) S^(i,j)T ||_F (Eq. 9 summand / 2)
//   loss_part[i*nbj + j] = sum (R^(i,j))^2 D^(j)          (Eq. 5 summand)
// LOSS_ONLY stops after the block loss; a non-null gpart then receives the residual R sqrt(D) itself,
// laid out like Wbar (the full-matrix loss evaluation passes D = 1 and reads R from it).
// ------------------------------------------------------------------------------------------------
template <int B, bool LOSS_ONLY>
__global__ __launch_bounds__(Chain<B>::NT) void phase_A_kernel(
    const float *__restrict__ Wbar, const float *__restrict__ C, const float *__restrict__ A,
    const float *__restrict__ Bw, const float *__restrict__ D, int64_t d_in, int nbj, int nsplit,
    float *__restrict__ gpart, float *__restrict__ beta_part, float *__restrict__ loss_part) {
    using CH = Chain<B>;
    __shared__ Smem<B> sm;
    const int tid = threadIdx.x;
    const typename CH::Pos p(tid);
    const int ldw = (int)d_in;
    const uint32_t wboff = p.lane_boff(ldw);
    const int i = blockIdx.x / nsplit, c = blockIdx.x % nsplit;
    const int chunk = (nbj + nsplit - 1) / nsplit;
    const int j0 = c * chunk, j1 = min(nbj, j0 + chunk);
    typename CH::Acc gacc, acc;
    typename CH::TileRegs t0, t1;
    gacc.zero();
    if (j0 < j1) {
        CH::gload_tile(t0, C + (int64_t)i * B * d_in + (int64_t)j0 * B, ldw, tid);
        CH::gload_tile(t1, Bw + (int64_t)j0 * B * B, B, tid);
    }
    for (int j = j0; j < j1; ++j) {
        const float *Wij = Wbar + (int64_t)i * B * d_in + (int64_t)j * B;
        CH::lstore_tile(sm.X, t0, tid);
        CH::lstore_tile(sm.Y, t1, tid);
        if (tid < B) sm.Dl[tid] = D[(int64_t)j * B + tid];
        __syncthreads();
        CH::gload_tile(t0, A + (int64_t)i * B * B, B, tid);
        CH::template mma<false, false, false, true, true>(acc, sm.X, sm.Y, nullptr, p); // S = C B
        // Everything downstream needs S only as S sqrt(D) (columns scaled): (R D) S^T = (R sqrt D)(S sqrt D)^T,
        // S D S^T = (S sqrt D)(S sqrt D)^T, and A S = (A S sqrt D) / sqrt D column by column.  Scaling here
        // once keeps the per-k multiply out of the product loops.  A zero weight gives a zero column.
        float sq[CH::TN], isq[CH::TN];
#pragma unroll
        for (int tn = 0; tn < CH::TN; ++tn) {
            const float dj = sm.Dl[p.col(tn)];
            sq[tn] = sqrtf(dj);
            isq[tn] = dj > 0.f ? 1.f / sq[tn] : 0.f;
#pragma unroll
            for (int tm = 0; tm < CH::TM; ++tm)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc.v[tm][tn][r] *= sq[tn];
        }
        __syncthreads();
        CH::store_acc(sm.X, acc, p);
        CH::lstore_tile(sm.Y, t0, tid);
        float wb[CH::TM][CH::TN][16];
        const uint32_t lb = opaque_u(wboff);
#pragma unroll
        for (int tm = 0; tm < CH::TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < CH::TN; ++tn)
#pragma unroll
                for (int r = 0; r < 16; ++r) wb[tm][tn][r] = gld(Wij, lb + CH::Pos::unif_boff(tm, tn, r, ldw));
        __syncthreads();
        CH::template mma<false, false, false, true, true>(acc, sm.Y, sm.X, nullptr, p); // A (S sqrt D)
        float lsum = 0.f;
#pragma unroll
        for (int tm = 0; tm < CH::TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < CH::TN; ++tn) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    float res = (wb[tm][tn][r] - acc.v[tm][tn][r] * isq[tn]) * sq[tn]; // R sqrt(D)
                    lsum += res * res;
                    acc.v[tm][tn][r] = res;
                }
            }
        if (LOSS_ONLY && gpart != nullptr) { // the loss-only pass can leave R sqrt(D) (d_out x d_in, like Wbar) in gpart
            float *Rij = gpart + (int64_t)i * B * d_in + (int64_t)j * B;
#pragma unroll
            for (int tm = 0; tm < CH::TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < CH::TN; ++tn)
#pragma unroll
                    for (int r = 0; r < 16; ++r) gst(Rij, lb + CH::Pos::unif_boff(tm, tn, r, ldw), acc.v[tm][tn][r]);
        }
        float ltot = CH::block_sum(lsum, sm.red, tid); // (has barriers: every wave is done reading Y)
        if (tid == 0) loss_part[i * nbj + j] = ltot;
        if (!LOSS_ONLY) {
            CH::store_acc(sm.Y, acc, p); // R sqrt(D)
            __syncthreads();
        }
        if (j + 1 < j1) { // next block's first operands, underneath the remaining products
            CH::gload_tile(t0, C + (int64_t)i * B * d_in + (int64_t)(j + 1) * B, ldw, tid);
            CH::gload_tile(t1, Bw + (int64_t)(j + 1) * B * B, B, tid);
        }
        if (!LOSS_ONLY) {
            CH::template mma<false, true, false>(gacc, sm.Y, sm.X, nullptr, p); // += (R D) S^T
            const float f2 = CH::template sym_frob2<false>(sm.X, p, tid); // ||S D S^T||_F^2 (symmetric: upper tiles)
            float ftot = CH::block_sum(f2, sm.red, tid);
            if (tid == 0) beta_part[i * nbj + j] = sqrtf(ftot);
        }
        __syncthreads();
    }
    if (!LOSS_ONLY) {
        float *gp = gpart + (int64_t)blockIdx.x * B * B;
        const uint32_t lb = opaque_u(p.lane_boff(B));
#pragma unroll
        for (int tm = 0; tm < CH::TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < CH::TN; ++tn)
#pragma unroll
                for (int r = 0; r < 16; ++r) gst(gp, lb + CH::Pos::unif_boff(tm, tn, r, B), -2.f * gacc.v[tm][tn][r]);
    }
}

// ------------------------------------------------------------------------------------------------
// B-phase (Alg. 2, second gradient step, at the updated A; App. D.2).  Workgroup (j, c) walks the
// row blocks i of its chunk.
//   gpart[(j*nsplit + c)][b][b] = -2 * sum_i S'^(i,j)T (R D)^(i,j)
//   beta_part[i*nbj + j] = || S'^(i,j)T S'^(i,j) ||_F * ||D^(j)||_F     (Eq. 10 summand / 2)
// ------------------------------------------------------------------------------------------------
template <int B>
__global__ __launch_bounds__(Chain<B>::NT) void phase_B_kernel(
    const float *__restrict__ Wbar, const float *__restrict__ C, const float *__restrict__ A,
    const float *__restrict__ Bw, const float *__restrict__ D, int64_t d_in, int nbi, int nbj, int nsplit,
    float *__restrict__ gpart, float *__restrict__ beta_part, float *__restrict__ Sp) {
    using CH = Chain<B>;
    __shared__ Smem<B> sm;
    const int tid = threadIdx.x;
    const typename CH::Pos p(tid);
    const int ldw = (int)d_in;
    const uint32_t wboff = p.lane_boff(ldw);
    const int j = blockIdx.x / nsplit, c = blockIdx.x % nsplit;
    const int chunk = (nbi + nsplit - 1) / nsplit;
    const int i0 = c * chunk, i1 = min(nbi, i0 + chunk);
    typename CH::Acc gacc, acc;
    typename CH::TileRegs t0, t1;
    gacc.zero();
    if (i0 < i1) {
        CH::gload_tile(t0, C + (int64_t)i0 * B * d_in + (int64_t)j * B, ldw, tid);
        CH::gload_tile(t1, A + (int64_t)i0 * B * B, B, tid);
    }
    if (tid < B) sm.Dl[tid] = D[(int64_t)j * B + tid];
    __syncthreads();
    float dn2 = 0.f;
    if (tid == 0)
        for (int q = 0; q < B; ++q) dn2 += sm.Dl[q] * sm.Dl[q];
    for (int i = i0; i < i1; ++i) {
        const float *Wij = Wbar + (int64_t)i * B * d_in + (int64_t)j * B;
        CH::lstore_tile(sm.X, t0, tid);
        CH::lstore_tile(sm.Y, t1, tid);
        __syncthreads();
        CH::gload_tile(t0, Bw + (int64_t)j * B * B, B, tid);
        CH::template mma<false, false, false, true, true>(acc, sm.Y, sm.X, nullptr, p); // S' = A C
        __syncthreads();
        CH::store_acc(sm.X, acc, p);
        if (Sp != nullptr) { // A and C do not change until the W' step: that step takes S' from here
            float *Sij = Sp + (int64_t)i * B * d_in + (int64_t)j * B;
            const uint32_t lb = opaque_u(wboff);
#pragma unroll
            for (int tm = 0; tm < CH::TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < CH::TN; ++tn)
#pragma unroll
                    for (int r = 0; r < 16; ++r) gst(Sij, lb + CH::Pos::unif_boff(tm, tn, r, ldw), acc.v[tm][tn][r]);
        }
        CH::lstore_tile(sm.Y, t0, tid);
        float wb[CH::TM][CH::TN][16];
        const uint32_t lb = opaque_u(wboff);
#pragma unroll
        for (int tm = 0; tm < CH::TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < CH::TN; ++tn)
#pragma unroll
                for (int r = 0; r < 16; ++r) wb[tm][tn][r] = gld(Wij, lb + CH::Pos::unif_boff(tm, tn, r, ldw));
        __syncthreads();
        CH::template mma<false, false, false, true, true>(acc, sm.X, sm.Y, nullptr, p); // What = S' B
#pragma unroll
        for (int tm = 0; tm < CH::TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < CH::TN; ++tn) {
                float dj = sm.Dl[p.col(tn)];
#pragma unroll
                for (int r = 0; r < 16; ++r) acc.v[tm][tn][r] = (wb[tm][tn][r] - acc.v[tm][tn][r]) * dj;
            }
        __syncthreads();
        CH::store_acc(sm.Y, acc, p); // R D
        __syncthreads();
        if (i + 1 < i1) {
            CH::gload_tile(t0, C + (int64_t)(i + 1) * B * d_in + (int64_t)j * B, ldw, tid);
            CH::gload_tile(t1, A + (int64_t)(i + 1) * B * B, B, tid);
        }
        CH::template mma<true, false, false>(gacc, sm.X, sm.Y, nullptr, p); // += S'^T (R D)
        const float f2 = CH::template sym_frob2<true>(sm.X, p, tid); // ||S'^T S'||_F^2 (symmetric: upper tiles)
        float ftot = CH::block_sum(f2, sm.red, tid);
        if (tid == 0) beta_part[i * nbj + j] = sqrtf(ftot) * sqrtf(dn2);
        __syncthreads();
    }
    float *gp = gpart + (int64_t)blockIdx.x * B * B;
    const uint32_t lb = opaque_u(p.lane_boff(B));
#pragma unroll
    for (int tm = 0; tm < CH::TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < CH::TN; ++tn)
#pragma unroll
            for (int r = 0; r < 16; ++r) gst(gp, lb + CH::Pos::unif_boff(tm, tn, r, B), -2.f * gacc.v[tm][tn][r]);
}

// ------------------------------------------------------------------------------------------------
// W' step of Alg. 2 on its own (unstructured mode, Sec. 4.5, where no sparse-core step follows):
//   G^(i,j) = A^(i)T ((Wbar - A C B) D)^(i,j) B^(j)T   (App. D.3),   C <- C + (2 / beta_W') G (.) M   (Eq. 11).
// Blocks are independent; workgroup w handles blocks w, w + gridDim.x, ...
// ------------------------------------------------------------------------------------------------
template <int B>
__global__ __launch_bounds__(Chain<B>::NT) void phase_W_kernel(
    const float *__restrict__ Wbar, float *__restrict__ C, const float *__restrict__ A,
    const float *__restrict__ Bw, const float *__restrict__ D, const uint8_t *__restrict__ mask, int mask_group,
    const float *__restrict__ fro2A, int nA, const float *__restrict__ fro2K, int nK, int64_t d_in, int nbj,
    int nblocks) {
    using CH = Chain<B>;
    __shared__ Smem<B> sm;
    const int tid = threadIdx.x;
    const typename CH::Pos p(tid);
    const int ldw = (int)d_in;
    const uint32_t wboff = p.lane_boff(ldw);
    typename CH::Acc acc;
    typename CH::TileRegs t0, tc;
    const int64_t mrow = d_in / mask_group;
    int blk = blockIdx.x;
    if (blk < nblocks) CH::gload_tile(t0, C + (int64_t)(blk / nbj) * B * d_in + (int64_t)(blk % nbj) * B, ldw, tid);
    publish_eta_W(sm, tid, fro2A, nA, fro2K, nK); // its loads travel with the first tile's
    for (; blk < nblocks; blk += gridDim.x) {
        const int i = blk / nbj, j = blk % nbj;
        float *Cij = C + (int64_t)i * B * d_in + (int64_t)j * B;
        const float *Wij = Wbar + (int64_t)i * B * d_in + (int64_t)j * B;
        CH::lstore_tile(sm.X, t0, tid);
        CH::gload_tile(t0, A + (int64_t)i * B * B, B, tid);
        if (tid < B) sm.Dl[tid] = D[(int64_t)j * B + tid];
        CH::lstore_tile(sm.Y, t0, tid);
        __syncthreads();
        CH::gload_tile(t0, Bw + (int64_t)j * B * B, B, tid);
        acc.zero();
        CH::template mma<false, false, false, false>(acc, sm.Y, sm.X, nullptr, p); // S' = A C
        __syncthreads();
        CH::store_acc(sm.X, acc, p);
        CH::lstore_tile(sm.Y, t0, tid);
        {
            float wb[CH::TM][CH::TN][16];
            const uint32_t lb = opaque_u(wboff);
#pragma unroll
            for (int tm = 0; tm < CH::TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < CH::TN; ++tn)
#pragma unroll
                    for (int r = 0; r < 16; ++r) wb[tm][tn][r] = gld(Wij, lb + CH::Pos::unif_boff(tm, tn, r, ldw));
            __syncthreads();
            acc.zero();
            CH::template mma<false, false, false, false>(acc, sm.X, sm.Y, nullptr, p); // What = S' B
#pragma unroll
            for (int tm = 0; tm < CH::TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < CH::TN; ++tn) {
                    float dj = sm.Dl[p.col(tn)];
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc.v[tm][tn][r] = (wb[tm][tn][r] - acc.v[tm][tn][r]) * dj;
                }
        }
        __syncthreads();
        CH::store_acc(sm.X, acc, p); // R D   (Y still holds B^j)
        __syncthreads();
        CH::gload_tile(t0, A + (int64_t)i * B * B, B, tid);
        acc.zero();
        CH::template mma<false, true, false, false>(acc, sm.X, sm.Y, nullptr, p); // U = (R D) B^T
        __syncthreads();
        CH::store_acc(sm.X, acc, p);
        CH::lstore_tile(sm.Y, t0, tid);
        // operands of the epilogue and the next block's core tile, underneath the last product
        uint32_t mraw[CH::PER][2];
        CH::gload_tile(tc, Cij, ldw, tid); // this block's core again (L2), in the coalesced loader layout
#pragma unroll
        for (int it = 0; it < CH::PER; ++it) {
            const int row = it * CH::ROWS_PER_IT + CH::loader_row(tid);
            const int64_t gcol = (int64_t)j * B + CH::loader_c4(tid) * 4;
            const uint8_t *mp = mask + ((int64_t)i * B + row) * mrow + gcol / mask_group;
            mraw[it][0] = mp[0];
            mraw[it][1] = mask_group == 2 ? mp[1] : 0u;
        }
        const int nblk = blk + gridDim.x;
        {   // unconditional (the last block asks for its own tile again): a request under a condition makes
            // the wait for the epilogue's operands cover it too
            const int nb = nblk < nblocks ? nblk : blk;
            CH::gload_tile(t0, C + (int64_t)(nb / nbj) * B * d_in + (int64_t)(nb % nbj) * B, ldw, tid);
        }
        __syncthreads();
        acc.zero();
        CH::template mma<true, false, false, false>(acc, sm.Y, sm.X, nullptr, p); // G = A^T U
        {
            // C <- C + (2/beta) G on kept entries, as one coalesced float4 pass: G goes through LDS
            const float eta2 = read_eta_W(sm);
            __syncthreads();
            CH::store_acc(sm.X, acc, p);
            __syncthreads();
            const int off0 = opaque(CH::loader_row(tid) * ldw + CH::loader_c4(tid) * 4);
            const int lrow = opaque(CH::loader_row(tid)), c4 = opaque(CH::loader_c4(tid));
#pragma unroll
            for (int it = 0; it < CH::PER; ++it) {
                const int row = it * CH::ROWS_PER_IT + lrow;
                const int shift = (int)(((int64_t)j * B + c4 * 4) % mask_group);
                const uint32_t nib = mask_group == 2 ? ((mraw[it][0] & 3u) | ((mraw[it][1] & 3u) << 2))
                                                     : ((mraw[it][0] >> shift) & 0xFu);
                const float *g = sm.X + row * CH::P + c4 * 4;
                float4 v = tc.v[it];
                if (nib & 1u) v.x += eta2 * g[0];
                if (nib & 2u) v.y += eta2 * g[1];
                if (nib & 4u) v.z += eta2 * g[2];
                if (nib & 8u) v.w += eta2 * g[3];
                *reinterpret_cast<float4 *>(Cij + (off0 + it * CH::ROWS_PER_IT * ldw)) = v;
            }
        }
        __syncthreads();
    }
}

// ------------------------------------------------------------------------------------------------
// W' step of Alg. 2 fused with the core gradient that Alg. 3 needs afterwards (N:M mode).
// With G = A^T ((Wbar - A C B) D) B^T, Delta = G (.) M and eta = 2 / beta_W' (Eq. 11):
//     C_new = C + eta * Delta                                        (the W' step, App. D.3)
//     G_new = A^T ((Wbar - A C_new B) D) B^T = G - eta * (A^T A) Delta (B D B^T)
//     L(C_new) = L(C) - 2 eta ||Delta||_F^2 + eta^2 <Delta, (A^T A) Delta (B D B^T)>
// so the gradient at the updated core costs two more b-deep products on tiles that are already
// on the CU (Delta, and the precomputed wrapper Grams A^T A and K = B D B^T) instead of a second
// pass of four.  Gout = -2 G_new (unmasked; selection scores and q-vectors of Alg. 3 read it),
// loss_part[block] = block loss after the continuous step.
// ------------------------------------------------------------------------------------------------
template <int B>
__global__ __launch_bounds__(Chain<B>::NT) void phase_WS_kernel(
    const float *__restrict__ Wbar, float *__restrict__ C, const float *__restrict__ A,
    const float *__restrict__ Bw, const float *__restrict__ D, const float *__restrict__ AtA,
    const float *__restrict__ K, const uint8_t *__restrict__ mask, int mask_group,
    const float *__restrict__ fro2A, int nA, const float *__restrict__ fro2K, int nK, int64_t d_in, int nbj,
    int nblocks, float *__restrict__ Gout, float *__restrict__ loss_part, const float *__restrict__ Sp) {
    using CH = Chain<B>;
    __shared__ Smem<B> sm;
    const int tid = threadIdx.x;
    const typename CH::Pos p(tid);
    const int ldw = (int)d_in;
    const uint32_t wboff = p.lane_boff(ldw);
    typename CH::Acc acc, acc2;
    typename CH::TileRegs t0, t1;
    const int64_t mrow = d_in / mask_group;
    // S' = A C either comes from the B step, which formed it at the same A and C (Sp), or is formed here
    const float *first = Sp != nullptr ? Sp : C;
    int blk = blockIdx.x;
    if (blk < nblocks) {
        CH::gload_tile(t0, first + (int64_t)(blk / nbj) * B * d_in + (int64_t)(blk % nbj) * B, ldw, tid);
        if (Sp != nullptr) CH::gload_tile(t1, Bw + (int64_t)(blk % nbj) * B * B, B, tid);
    }
    publish_eta_W(sm, tid, fro2A, nA, fro2K, nK); // eta of the comment above; its loads travel with the first tiles'
    for (; blk < nblocks; blk += gridDim.x) {
        const int i = blk / nbj, j = blk % nbj;
        float *Cij = C + (int64_t)i * B * d_in + (int64_t)j * B;
        const float *Wij = Wbar + (int64_t)i * B * d_in + (int64_t)j * B;
        CH::lstore_tile(sm.X, t0, tid);
        if (tid < B) sm.Dl[tid] = D[(int64_t)j * B + tid];
        if (Sp != nullptr) {
            CH::lstore_tile(sm.Y, t1, tid); // X = S', Y = B^j
        } else {
            CH::gload_tile(t0, A + (int64_t)i * B * B, B, tid);
            CH::lstore_tile(sm.Y, t0, tid);
            __syncthreads();
            CH::gload_tile(t0, Bw + (int64_t)j * B * B, B, tid);
            acc.zero();
            CH::template mma<false, false, false, false>(acc, sm.Y, sm.X, nullptr, p); // S' = A C
            __syncthreads();
            CH::store_acc(sm.X, acc, p);
            CH::lstore_tile(sm.Y, t0, tid);
        }
        float lsum = 0.f;
        {
            float wb[CH::TM][CH::TN][16];
            const uint32_t lb = opaque_u(wboff);
#pragma unroll
            for (int tm = 0; tm < CH::TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < CH::TN; ++tn)
#pragma unroll
                    for (int r = 0; r < 16; ++r) wb[tm][tn][r] = gld(Wij, lb + CH::Pos::unif_boff(tm, tn, r, ldw));
            __syncthreads();
            acc.zero();
            CH::template mma<false, false, false, false>(acc, sm.X, sm.Y, nullptr, p); // What = S' B
#pragma unroll
            for (int tm = 0; tm < CH::TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < CH::TN; ++tn) {
                    float dj = sm.Dl[p.col(tn)];
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        float res = wb[tm][tn][r] - acc.v[tm][tn][r];
                        lsum += res * res * dj;
                        acc.v[tm][tn][r] = res * dj;
                    }
                }
        }
        __syncthreads();
        CH::store_acc(sm.X, acc, p); // R D   (Y still holds B^j)
        __syncthreads();
        CH::gload_tile(t0, A + (int64_t)i * B * B, B, tid);
        acc.zero();
        CH::template mma<false, true, false>(acc, sm.X, sm.Y, nullptr, p); // U = (R D) B^T
        __syncthreads();
        CH::store_acc(sm.X, acc, p);
        CH::lstore_tile(sm.Y, t0, tid);
        // current core values and mask bytes in the accumulator layout, underneath the next product
        float cv[CH::TM][CH::TN][16];
        uint32_t mraw[CH::TM][CH::TN][16];
        {
            const uint32_t lb = opaque_u(wboff);
            // mask bytes: uniform block base + 32-bit lane offset (b is a multiple of the group size)
            const uint8_t *mb = mask + (int64_t)i * B * mrow + (int64_t)j * B / mask_group;
#pragma unroll
            for (int tm = 0; tm < CH::TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < CH::TN; ++tn) {
                    const uint32_t ml = opaque_u((uint32_t)((p.wm0 + p.kh * 4) * (int)mrow + p.col(tn) / mask_group));
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        cv[tm][tn][r] = gld(Cij, lb + CH::Pos::unif_boff(tm, tn, r, ldw));
                        mraw[tm][tn][r] = gld(mb, ml + (uint32_t)((tm * 32 + (r >> 2) * 8 + (r & 3)) * (int)mrow));
                    }
                }
        }
        CH::gload_tile(t0, K + (int64_t)j * B * B, B, tid);
        __syncthreads();
        acc.zero();
        CH::template mma<true, false, false, false>(acc, sm.Y, sm.X, nullptr, p); // G = A^T U   (stays in acc)
        const float eta2 = read_eta_W(sm);
        // W' step on kept entries; Delta = G (.) M goes to LDS for the two extra products
        uint32_t keep[CH::TM][CH::TN];
        float dd = 0.f;
        __syncthreads();
        {
            float *d0 = sm.X + opaque(p.lane_off(CH::P));
            const uint32_t lb = opaque_u(wboff);
#pragma unroll
            for (int tm = 0; tm < CH::TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < CH::TN; ++tn) {
                    const int sh = p.col(tn) % mask_group;
                    keep[tm][tn] = 0u;
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const bool kp = (mraw[tm][tn][r] >> sh) & 1u;
                        keep[tm][tn] |= (kp ? 1u : 0u) << r;
                        const float dl = kp ? acc.v[tm][tn][r] : 0.f;
                        dd += dl * dl;
                        d0[CH::Pos::unif_off(tm, tn, r, CH::P)] = dl;
                        if (kp) gst(Cij, lb + CH::Pos::unif_boff(tm, tn, r, ldw), cv[tm][tn][r] + eta2 * dl);
                    }
                }
        }
        CH::lstore_tile(sm.Y, t0, tid); // K^j
        __syncthreads();
        CH::gload_tile(t0, AtA + (int64_t)i * B * B, B, tid);
        acc2.zero();
        CH::template mma<false, false, false, false>(acc2, sm.X, sm.Y, nullptr, p); // V = Delta K
        __syncthreads();
        CH::store_acc(sm.X, acc2, p);
        CH::lstore_tile(sm.Y, t0, tid); // A^T A (symmetric)
        __syncthreads();
        const int nblk = blk + gridDim.x;
        if (nblk < nblocks) {
            CH::gload_tile(t0, first + (int64_t)(nblk / nbj) * B * d_in + (int64_t)(nblk % nbj) * B, ldw, tid);
            if (Sp != nullptr) CH::gload_tile(t1, Bw + (int64_t)(nblk % nbj) * B * B, B, tid);
        }
        acc2.zero();
        CH::template mma<false, false, false, false>(acc2, sm.Y, sm.X, nullptr, p); // Z = (A^T A) V
        float dz = 0.f;
        {
            float *Gij = Gout + (int64_t)i * B * d_in + (int64_t)j * B;
            const uint32_t lb = opaque_u(wboff);
#pragma unroll
            for (int tm = 0; tm < CH::TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < CH::TN; ++tn)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const float g = acc.v[tm][tn][r], z = acc2.v[tm][tn][r];
                        if ((keep[tm][tn] >> r) & 1u) dz += g * z;
                        gst(Gij, lb + CH::Pos::unif_boff(tm, tn, r, ldw), -2.f * (g - eta2 * z));
                    }
        }
        float ltot = CH::block_sum(lsum - 2.f * eta2 * dd + eta2 * eta2 * dz, sm.red, tid);
        if (tid == 0) loss_part[blk] = ltot;
        __syncthreads();
    }
}

// ------------------------------------------------------------------------------------------------
// Joint-Adam variant of the continuous step (Sec. 3.3.1): one forward/backward pass per block gives
// the gradients of A, B and W' at the same point.  With S = C B, R = Wbar - A S, T = A^T (R D):
//   grad_A^(i) = -2 sum_j (R D) S^T      (accumulated in registers over the chunk of j; gApart)
//   grad_B^(j) = -2 sum_i C^T T          (one partial per block: gBpart[(j*nbi + i)])
//   grad_W'    = -2 (T B^T) (.) M        (complete per block: the Adam update of the core and of its
//                                         moments happens here, moments also decay on pruned entries)
// Workgroup (i, c) walks the column blocks j of its chunk.  loss_part = block loss at the old point.
// ------------------------------------------------------------------------------------------------
template <int B>
__global__ __launch_bounds__(Chain<B>::NT) void phase_FB_kernel(
    const float *__restrict__ Wbar, float *__restrict__ C, const float *__restrict__ A,
    const float *__restrict__ Bw, const float *__restrict__ D, const uint8_t *__restrict__ mask, int mask_group,
    float *__restrict__ mC, float *__restrict__ vC, AdamCoef k, int64_t d_in, int nbi, int nbj, int nsplit,
    float *__restrict__ gApart, float *__restrict__ gBpart, float *__restrict__ loss_part) {
    using CH = Chain<B>;
    __shared__ Smem<B> sm;
    const int tid = threadIdx.x;
    const typename CH::Pos p(tid);
    const int ldw = (int)d_in;
    const uint32_t wboff = p.lane_boff(ldw);
    const int i = blockIdx.x / nsplit, c = blockIdx.x % nsplit;
    const int chunk = (nbj + nsplit - 1) / nsplit;
    const int j0 = c * chunk, j1 = min(nbj, j0 + chunk);
    const int64_t mrow = d_in / mask_group;
    typename CH::Acc gacc, acc;
    typename CH::TileRegs t0, t1;
    gacc.zero();
    if (j0 < j1) {
        CH::gload_tile(t0, C + (int64_t)i * B * d_in + (int64_t)j0 * B, ldw, tid);
        CH::gload_tile(t1, Bw + (int64_t)j0 * B * B, B, tid);
    }
    for (int j = j0; j < j1; ++j) {
        float *Cij = C + (int64_t)i * B * d_in + (int64_t)j * B;
        const float *Wij = Wbar + (int64_t)i * B * d_in + (int64_t)j * B;
        CH::lstore_tile(sm.X, t0, tid);
        CH::lstore_tile(sm.Y, t1, tid);
        if (tid < B) sm.Dl[tid] = D[(int64_t)j * B + tid];
        __syncthreads();
        CH::gload_tile(t0, A + (int64_t)i * B * B, B, tid);
        acc.zero();
        CH::template mma<false, false, false>(acc, sm.X, sm.Y, nullptr, p); // S = C B
        __syncthreads();
        CH::store_acc(sm.X, acc, p);
        CH::lstore_tile(sm.Y, t0, tid);
        float lsum = 0.f;
        {
            float wb[CH::TM][CH::TN][16];
            const uint32_t lb = opaque_u(wboff);
#pragma unroll
            for (int tm = 0; tm < CH::TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < CH::TN; ++tn)
#pragma unroll
                    for (int r = 0; r < 16; ++r) wb[tm][tn][r] = gld(Wij, lb + CH::Pos::unif_boff(tm, tn, r, ldw));
            __syncthreads();
            acc.zero();
            CH::template mma<false, false, false>(acc, sm.Y, sm.X, nullptr, p); // What = A S
#pragma unroll
            for (int tm = 0; tm < CH::TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < CH::TN; ++tn) {
                    float dj = sm.Dl[p.col(tn)];
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        float res = wb[tm][tn][r] - acc.v[tm][tn][r];
                        lsum += res * res * dj;
                        acc.v[tm][tn][r] = res * dj;
                    }
                }
        }
        float ltot = CH::block_sum(lsum, sm.red, tid);
        if (tid == 0) loss_part[i * nbj + j] = ltot;
        CH::store_acc(sm.Y, acc, p); // R D          [X = S, Y = R D]
        __syncthreads();
        CH::gload_tile(t0, A + (int64_t)i * B * B, B, tid);
        CH::template mma<false, true, false>(gacc, sm.Y, sm.X, nullptr, p); // grad_A += (R D) S^T
        __syncthreads();
        CH::lstore_tile(sm.X, t0, tid); //            [X = A, Y = R D]
        __syncthreads();
        CH::gload_tile(t0, Bw + (int64_t)j * B * B, B, tid);
        acc.zero();
        CH::template mma<true, false, false>(acc, sm.X, sm.Y, nullptr, p); // T = A^T (R D)
        __syncthreads();
        CH::store_acc(sm.Y, acc, p);
        CH::lstore_tile(sm.X, t0, tid); //            [X = B, Y = T]
        __syncthreads();
        CH::gload_tile(t0, Cij, ldw, tid);
        uint32_t keep[CH::TM][CH::TN];
        {   // mask bytes of this block, fetched underneath the product and folded into one bit per element
            uint32_t mraw[CH::TM][CH::TN][16];
#pragma unroll
            for (int tm = 0; tm < CH::TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < CH::TN; ++tn) {
                    // uniform block base + 32-bit lane offset (B is a multiple of the group size)
                    const uint8_t *mb = mask + (int64_t)i * B * mrow + (int64_t)j * B / mask_group;
                    const uint32_t mlane = opaque_u((uint32_t)((p.wm0 + p.kh * 4) * (int)mrow + p.col(tn) / mask_group));
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        mraw[tm][tn][r] = gld(mb, mlane + (uint32_t)((tm * 32 + (r >> 2) * 8 + (r & 3)) * (int)mrow));
                }
            acc.zero();
            CH::template mma<false, true, false>(acc, sm.Y, sm.X, nullptr, p); // T B^T  (stays in acc for the core update)
#pragma unroll
            for (int tm = 0; tm < CH::TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < CH::TN; ++tn) {
                    const int sh = p.col(tn) % mask_group;
                    keep[tm][tn] = 0u;
#pragma unroll
                    for (int r = 0; r < 16; ++r) keep[tm][tn] |= ((mraw[tm][tn][r] >> sh) & 1u) << r;
                }
        }
        __syncthreads();
        CH::lstore_tile(sm.X, t0, tid); //            [X = C, Y = T]
        float *mij = mC + (int64_t)i * B * d_in + (int64_t)j * B, *vij = vC + (int64_t)i * B * d_in + (int64_t)j * B;
        __syncthreads();
        typename CH::Acc acc2;
        acc2.zero();
        CH::template mma<true, false, false>(acc2, sm.X, sm.Y, nullptr, p); // C^T T
        {
            float *gb = gBpart + ((int64_t)j * nbi + i) * B * B;
            const uint32_t lb = opaque_u(p.lane_boff(B));
#pragma unroll
            for (int tm = 0; tm < CH::TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < CH::TN; ++tn)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        gst(gb, lb + CH::Pos::unif_boff(tm, tn, r, B), -2.f * acc2.v[tm][tn][r]);
        }
        __builtin_amdgcn_sched_barrier(0); // keep the moment loads below the product: they would not fit beside it
        float mo[CH::TM][CH::TN][16], vo[CH::TM][CH::TN][16];
        const uint32_t lb = opaque_u(wboff);
#pragma unroll
        for (int tm = 0; tm < CH::TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < CH::TN; ++tn)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const uint32_t off = lb + CH::Pos::unif_boff(tm, tn, r, ldw);
                    mo[tm][tn][r] = gld(mij, off);
                    vo[tm][tn][r] = gld(vij, off);
                }
        // next block's core tile, underneath the core update below.  Unconditional (the last block asks
        // for its own tile again): under a condition, the paths that meet in front of the update differ
        // in their outstanding loads and the wait for the moments would cover this request as well.
        const int jn = min(j + 1, j1 - 1);
        CH::gload_tile(t0, C + (int64_t)i * B * d_in + (int64_t)jn * B, ldw, tid);
        {   // Adam on the core: g = -2 (T B^T) (.) M; the current values are still in LDS (X = C)
            const float *c0 = sm.X + opaque(p.lane_off(CH::P));
            const uint32_t lb = opaque_u(wboff);
#pragma unroll
            for (int tm = 0; tm < CH::TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < CH::TN; ++tn) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const uint32_t off = lb + CH::Pos::unif_boff(tm, tn, r, ldw);
                        const bool kp = (keep[tm][tn] >> r) & 1u;
                        const float g = kp ? -2.f * acc.v[tm][tn][r] : 0.f;
                        const float mn = k.b1 * mo[tm][tn][r] + k.one_minus_b1 * g;
                        const float vn = k.b2 * vo[tm][tn][r] + k.one_minus_b2 * g * g;
                        gst(mij, off, mn);
                        gst(vij, off, vn);
                        if (kp)
                            gst(Cij, off, c0[CH::Pos::unif_off(tm, tn, r, CH::P)] -
                                              k.lr * (mn * k.inv_c1) / (sqrtf(vn * k.inv_c2) + k.eps));
                    }
                }
        }
        __builtin_amdgcn_sched_barrier(0); // the wrapper tile only once the moments have left their registers
        CH::gload_tile(t1, Bw + (int64_t)jn * B * B, B, tid);
        __syncthreads();
    }
    float *gp = gApart + (int64_t)blockIdx.x * B * B;
    const uint32_t lb = opaque_u(p.lane_boff(B));
#pragma unroll
    for (int tm = 0; tm < CH::TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < CH::TN; ++tn)
#pragma unroll
            for (int r = 0; r < 16; ++r) gst(gp, lb + CH::Pos::unif_boff(tm, tn, r, B), -2.f * gacc.v[tm][tn][r]);
}

// ------------------------------------------------------------------------------------------------
// Core gradient at the current point for Alg. 3 (used after the Adam step, where A and B moved too and
// the gradient cannot be updated incrementally):  Gout = -2 A^T ((Wbar - A C B) D) B^T (unmasked),
// loss_part[block] = block loss (the loss after the continuous step).
// ------------------------------------------------------------------------------------------------
template <int B>
__global__ __launch_bounds__(Chain<B>::NT) void phase_GS_kernel(
    const float *__restrict__ Wbar, const float *__restrict__ C, const float *__restrict__ A,
    const float *__restrict__ Bw, const float *__restrict__ D, int64_t d_in, int nbj, int nblocks,
    float *__restrict__ Gout, float *__restrict__ loss_part) {
    using CH = Chain<B>;
    __shared__ Smem<B> sm;
    const int tid = threadIdx.x;
    const typename CH::Pos p(tid);
    const int ldw = (int)d_in;
    const uint32_t wboff = p.lane_boff(ldw);
    typename CH::Acc acc;
    typename CH::TileRegs t0, t1;
    int blk = blockIdx.x;
    if (blk < nblocks) {
        CH::gload_tile(t0, C + (int64_t)(blk / nbj) * B * d_in + (int64_t)(blk % nbj) * B, ldw, tid);
        CH::gload_tile(t1, A + (int64_t)(blk / nbj) * B * B, B, tid);
    }
    for (; blk < nblocks; blk += gridDim.x) {
        const int i = blk / nbj, j = blk % nbj;
        const float *Wij = Wbar + (int64_t)i * B * d_in + (int64_t)j * B;
        CH::lstore_tile(sm.X, t0, tid);
        CH::lstore_tile(sm.Y, t1, tid);
        if (tid < B) sm.Dl[tid] = D[(int64_t)j * B + tid];
        __syncthreads();
        CH::gload_tile(t0, Bw + (int64_t)j * B * B, B, tid);
        CH::template mma<false, false, false, true, true>(acc, sm.Y, sm.X, nullptr, p); // S' = A C
        __syncthreads();
        CH::store_acc(sm.X, acc, p);
        CH::lstore_tile(sm.Y, t0, tid);
        float lsum = 0.f;
        {
            float wb[CH::TM][CH::TN][16];
            const uint32_t lb = opaque_u(wboff);
#pragma unroll
            for (int tm = 0; tm < CH::TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < CH::TN; ++tn)
#pragma unroll
                    for (int r = 0; r < 16; ++r) wb[tm][tn][r] = gld(Wij, lb + CH::Pos::unif_boff(tm, tn, r, ldw));
            __syncthreads();
            CH::template mma<false, false, false, true, true>(acc, sm.X, sm.Y, nullptr, p); // What = S' B
#pragma unroll
            for (int tm = 0; tm < CH::TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < CH::TN; ++tn) {
                    float dj = sm.Dl[p.col(tn)];
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        float res = wb[tm][tn][r] - acc.v[tm][tn][r];
                        lsum += res * res * dj;
                        acc.v[tm][tn][r] = res * dj;
                    }
                }
        }
        float ltot = CH::block_sum(lsum, sm.red, tid);
        if (tid == 0) loss_part[blk] = ltot;
        CH::store_acc(sm.X, acc, p); // R D   (Y still holds B^j)
        __syncthreads();
        CH::gload_tile(t0, A + (int64_t)i * B * B, B, tid);
        CH::template mma<false, true, false, true, true>(acc, sm.X, sm.Y, nullptr, p); // U = (R D) B^T
        __syncthreads();
        CH::store_acc(sm.X, acc, p);
        CH::lstore_tile(sm.Y, t0, tid);
        __syncthreads();
        const int nblk = blk + gridDim.x;
        if (nblk < nblocks) {
            CH::gload_tile(t0, C + (int64_t)(nblk / nbj) * B * d_in + (int64_t)(nblk % nbj) * B, ldw, tid);
            CH::gload_tile(t1, A + (int64_t)(nblk / nbj) * B * B, B, tid);
        }
        CH::template mma<true, false, false, true, true>(acc, sm.Y, sm.X, nullptr, p); // G = A^T U
        float *Gij = Gout + (int64_t)i * B * d_in + (int64_t)j * B;
        const uint32_t lb = opaque_u(wboff);
#pragma unroll
        for (int tm = 0; tm < CH::TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < CH::TN; ++tn)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    gst(Gij, lb + CH::Pos::unif_boff(tm, tn, r, ldw), -2.f * acc.v[tm][tn][r]);
        __syncthreads();
    }
}

// ------------------------------------------------------------------------------------------------
// Small Gram-type products of the wrappers themselves (Eq. 11 and the shortcuts of Alg. 3):
//   block <  nbi : AtA^(i) = A^(i)T A^(i), colnorm2[i*b+p] = its diagonal = ||A^(i)[:,p]||^2 (the ||a||^2 of
//                  Eq. 7), fro2A[i*b/32 + slab] = squared Frobenius norm of one 32-column slab of it
//   block >= nbi : K^(j) = B^(j) D^(j) B^(j)T (holds every B' D B'^T of Eq. 7), fro2K likewise
// ------------------------------------------------------------------------------------------------
template <int B>
__global__ __launch_bounds__((B / 32) * 64) void wrapper_grams_kernel(
    const float *__restrict__ A, const float *__restrict__ Bw, const float *__restrict__ D, int nbi,
    float *__restrict__ colnorm2, float *__restrict__ fro2A, float *__restrict__ AtA, float *__restrict__ K,
    float *__restrict__ fro2K, uint16_t *__restrict__ PAtA, uint16_t *__restrict__ PK) {
    // One workgroup per (block, 32-column slab of the result), one wave per 32 x 32 tile of the slab:
    // the b x b products are few (d_out/b + d_in/b), so each is spread over b/32 compute units.
    using CH = Chain<B>;
    constexpr int NS = B / 32, NTH = NS * 64, P = CH::P;
    __shared__ float X[CH::TILE_FLOATS];
    __shared__ float Dl[B];
    __shared__ float red[NS];
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, l32 = lane & 31, kh = lane >> 5;
    const int blk = blockIdx.x / NS, ct = blockIdx.x % NS, rt = w;
    const bool isA = blk < nbi;
    const int idx = isA ? blk : blk - nbi;
    const float *src = (isA ? A : Bw) + (int64_t)idx * B * B;
    {   // whole block -> LDS (loader lane mapping of Chain, for this workgroup size)
        constexpr int ROWS_PER_IT = NTH / (B / 4), PER = B * B / 4 / NTH;
        const int lrow = ((tid >> 5) / (B / 32)) * 4 + ((tid & 31) >> 3), c4 = ((tid >> 5) % (B / 32)) * 8 + (tid & 7);
        float4 v[PER];
#pragma unroll
        for (int it = 0; it < PER; ++it)
            v[it] = *reinterpret_cast<const float4 *>(src + (lrow + it * ROWS_PER_IT) * B + c4 * 4);
#pragma unroll
        for (int it = 0; it < PER; ++it) {
            float *d = X + (lrow + it * ROWS_PER_IT) * P + c4 * 4;
            d[0] = v[it].x; d[1] = v[it].y; d[2] = v[it].z; d[3] = v[it].w;
        }
        if (!isA && tid < B) Dl[tid] = D[(int64_t)idx * B + tid];
    }
    __syncthreads();
    floatx16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    if (isA) { // (A^T A)[m][n] = sum_k A[k][m] A[k][n]
        const float *xa = X + kh * P + 32 * rt + l32, *xb = X + kh * P + 32 * ct + l32;
#pragma unroll 8
        for (int k = 0; k < B; k += 2) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(xa[k * P], xb[k * P], acc, 0, 0, 0);
    } else {   // K[m][n] = sum_k B[m][k] D[k] B[n][k]
        const float *xa = X + (32 * rt + l32) * P + kh, *xb = X + (32 * ct + l32) * P + kh;
#pragma unroll 8
        for (int k = 0; k < B; k += 2)
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(xa[k] * Dl[k + kh], xb[k], acc, 0, 0, 0);
    }
    float f2 = 0.f;
    float *dst = (isA ? AtA : K) + (int64_t)idx * B * B;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const float v = acc[r];
        const int row = 32 * rt + (r >> 2) * 8 + kh * 4 + (r & 3), col = 32 * ct + l32;
        f2 += v * v;
        if (isA && row == col) colnorm2[(int64_t)idx * B + row] = v;
        dst[row * B + col] = v;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) f2 += __shfl_xor(f2, off, 64);
    uint16_t *planes = isA ? PAtA : PK;
    const bool emit = B == PLANE_B && planes != nullptr; // uniform over the workgroup
    if (emit) {
        // The result also as bf16 pieces for the d_block 128 chains.  Both results are symmetric, so the slab
        // (all rows, columns 32 ct .. + 32) holds op(x, k) = M[x][k] for the two runs of 16 inner indices
        // inside it; it goes through LDS (the operand tile is dead) to turn "one column per lane" into
        // "sixteen columns of one row per thread".
        __syncthreads();
#pragma unroll
        for (int r = 0; r < 16; ++r) X[(32 * rt + (r >> 2) * 8 + kh * 4 + (r & 3)) * 33 + l32] = acc[r];
    }
    if (lane == 0) red[w] = f2;
    __syncthreads();
    if (tid == 0) {
        float s = 0.f;
        for (int q = 0; q < NS; ++q) s += red[q];
        (isA ? fro2A : fro2K)[idx * NS + ct] = s;
    }
    if constexpr (B == PLANE_B) {
        if (emit) {
            const int x = tid & (B - 1), rl = tid / B; // 256 threads: 128 rows x 2 runs
            float v[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) v[i] = X[x * 33 + 16 * rl + i];
            plane_emit(planes + (int64_t)idx * 3 * B * B, 2 * ct + rl, x, v);
        }
    }
}

// ------------------------------------------------------------------------------------------------
// host launchers
// ------------------------------------------------------------------------------------------------
int chain_max_nsplit() { return 64; }

// partial squared norms the wrapper-Gram kernels leave per block (one per 32-column slab up to b = 128)
int gram_parts(int b) { return b <= 128 ? b / 32 : 1; }

// Diagnostic: the step size 1 / beta_W' (Eq. 11) exactly as the W' kernels derive it (they apply
// 2 / beta_W' to the half gradient A^T (R D) B^T).
__global__ __launch_bounds__(64) void eta_W_trace_kernel(const float *__restrict__ fro2A, int nA,
                                                         const float *__restrict__ fro2K, int nK,
                                                         double *__restrict__ eta_out) {
    const float e = wave_eta_W(fro2A, nA, fro2K, nK);
    if (threadIdx.x == 0) *eta_out = 0.5 * (double)e;
}

void launch_eta_W_trace(const Dims &d, const float *fro2A, const float *fro2K, double *eta_out, hipStream_t s) {
    hipLaunchKernelGGL(eta_W_trace_kernel, dim3(1), dim3(64), 0, s, fro2A, d.nbi * gram_parts(d.b), fro2K,
                       d.nbj * gram_parts(d.b), eta_out);
}

#define ARMOR_DISPATCH_B(bval, ...)                      \
    switch (bval) {                                      \
    case 32:  { constexpr int BB = 32;  __VA_ARGS__; } break; \
    case 64:  { constexpr int BB = 64;  __VA_ARGS__; } break; \
    case 128: { constexpr int BB = 128; __VA_ARGS__; } break; \
    default: break;                                      \
    }

// b = 32 and 64 only: at b = 128 the phase runs in the streamed-operand form (chain_stream.hip)
#define ARMOR_DISPATCH_B_SMALL(bval, ...)                \
    switch (bval) {                                      \
    case 32:  { constexpr int BB = 32;  __VA_ARGS__; } break; \
    case 64:  { constexpr int BB = 64;  __VA_ARGS__; } break; \
    default: break;                                      \
    }

// Loss-only forward pass (d_block <= 128): block losses to loss_part and, if Rout is given, the residual
// R sqrt(D) as a d_out x d_in matrix (leading dimension d_in).
void launch_residual(const Dims &d, const float *Wbar, const float *C, const float *A, const float *B, const float *D,
                     int nsplit, float *Rout, float *loss_part, hipStream_t s) {
    ARMOR_DISPATCH_B(d.b, {
        dim3 grid(d.nbi * nsplit), block(Chain<BB>::NT);
        hipLaunchKernelGGL((phase_A_kernel<BB, true>), grid, block, 0, s, Wbar, C, A, B, D, d.d_in, d.nbj, nsplit, Rout,
                           (float *)nullptr, loss_part);
    });
}

void launch_phase_A(const Dims &d, const float *Wbar, const float *C, const float *A, const float *B,
                    const float *D, int nsplit, float *gpart, float *beta_part, float *loss_part,
                    bool loss_only, float *stream_scratch, const WrapperPlanes *planes, hipStream_t s) {
    if (loss_only) { // (the kernel's gradient argument doubles as the residual output in this mode: never the partials)
        launch_residual(d, Wbar, C, A, B, D, nsplit, nullptr, loss_part, s);
        return;
    }
    if (d.b == 128) { // two workgroups per CU
        launch_phase_A_stream(d, Wbar, C, A, B, D, nsplit, gpart, beta_part, loss_part, stream_scratch, planes, s);
        return;
    }
    ARMOR_DISPATCH_B_SMALL(d.b, {
        dim3 grid(d.nbi * nsplit), block(Chain<BB>::NT);
        hipLaunchKernelGGL((phase_A_kernel<BB, false>), grid, block, 0, s, Wbar, C, A, B, D, d.d_in, d.nbj, nsplit,
                           gpart, beta_part, loss_part);
    });
}

void launch_phase_B(const Dims &d, const float *Wbar, const float *C, const float *A, const float *B,
                    const float *D, int nsplit, float *gpart, float *beta_part, float *Sp, float *stream_scratch,
                    const WrapperPlanes *planes, hipStream_t s) {
    if (d.b == 128) {
        launch_phase_B_stream(d, Wbar, C, A, B, D, nsplit, gpart, beta_part, Sp, stream_scratch, planes, s);
        return;
    }
    ARMOR_DISPATCH_B_SMALL(d.b, {
        dim3 grid(d.nbj * nsplit), block(Chain<BB>::NT);
        hipLaunchKernelGGL((phase_B_kernel<BB>), grid, block, 0, s, Wbar, C, A, B, D, d.d_in, d.nbi, d.nbj, nsplit,
                           gpart, beta_part, Sp);
    });
}

void launch_phase_W(const Dims &d, const float *Wbar, float *C, const float *A, const float *B, const float *D,
                    const uint8_t *mask, int mask_group, const float *fro2A, const float *fro2K, const float *Sp,
                    int grid_cap, const WrapperPlanes *planes, hipStream_t s) {
    if (d.b == 128) { // the streamed W' kernel, stopping after the W' step; S' comes from the B step
        launch_phase_WS_stream(d, Wbar, C, A, B, D, nullptr, nullptr, mask, mask_group, fro2A, fro2K, nullptr, nullptr, Sp,
                               stream_wgs_per_cu() * grid_cap, planes, s);
        return;
    }
    ARMOR_DISPATCH_B_SMALL(d.b, {
        dim3 grid(std::min(d.nblocks, grid_cap)), block(Chain<BB>::NT);
        hipLaunchKernelGGL((phase_W_kernel<BB>), grid, block, 0, s, Wbar, C, A, B, D, mask, mask_group, fro2A,
                           d.nbi * gram_parts(d.b), fro2K, d.nbj * gram_parts(d.b), d.d_in, d.nbj, d.nblocks);
    });
}

void launch_wrapper_grams(const Dims &d, const float *A, const float *B, const float *D, float *colnorm2,
                          float *fro2A, float *AtA, float *K, float *fro2K, uint16_t *PAtA, uint16_t *PK,
                          hipStream_t s) {
    ARMOR_DISPATCH_B(d.b, {
        dim3 grid((d.nbi + d.nbj) * (BB / 32)), block((BB / 32) * 64);
        hipLaunchKernelGGL((wrapper_grams_kernel<BB>), grid, block, 0, s, A, B, D, d.nbi, colnorm2, fro2A, AtA, K,
                           fro2K, PAtA, PK);
    });
}

void launch_phase_FB(const Dims &d, const float *Wbar, float *C, const float *A, const float *B, const float *D,
                     const uint8_t *mask, int mask_group, float *mC, float *vC, double lr, double b1, double b2,
                     double eps, int64_t t, int nsplit, float *gApart, float *gBpart, float *loss_part,
                     float *stream_scratch, hipStream_t s) {
    if (d.b == 128) {
        launch_phase_FB_stream(d, Wbar, C, A, B, D, mask, mask_group, mC, vC, lr, b1, b2, eps, t, nsplit, gApart,
                               gBpart, loss_part, stream_scratch, s);
        return;
    }
    const AdamCoef k = make_adam_coef(lr, b1, b2, eps, t);
    ARMOR_DISPATCH_B_SMALL(d.b, {
        dim3 grid(d.nbi * nsplit), block(Chain<BB>::NT);
        hipLaunchKernelGGL((phase_FB_kernel<BB>), grid, block, 0, s, Wbar, C, A, B, D, mask, mask_group, mC, vC, k,
                           d.d_in, d.nbi, d.nbj, nsplit, gApart, gBpart, loss_part);
    });
}

void launch_phase_GS(const Dims &d, const float *Wbar, const float *C, const float *A, const float *B, const float *D,
                     float *Gout, float *loss_part, int grid_cap, hipStream_t s) {
    if (d.b == 128) {
        launch_phase_GS_stream(d, Wbar, C, A, B, D, Gout, loss_part, 2 * grid_cap, s);
        return;
    }
    ARMOR_DISPATCH_B_SMALL(d.b, {
        dim3 grid(std::min(d.nblocks, grid_cap)), block(Chain<BB>::NT);
        hipLaunchKernelGGL((phase_GS_kernel<BB>), grid, block, 0, s, Wbar, C, A, B, D, d.d_in, d.nbj, d.nblocks, Gout,
                           loss_part);
    });
}

void launch_phase_WS(const Dims &d, const float *Wbar, float *C, const float *A, const float *B, const float *D,
                     const float *AtA, const float *K, const uint8_t *mask, int mask_group, const float *fro2A,
                     const float *fro2K, float *Gout, float *loss_part, const float *Sp, int grid_cap,
                     const WrapperPlanes *planes, hipStream_t s) {
    if (d.b == 128) {
        launch_phase_WS_stream(d, Wbar, C, A, B, D, AtA, K, mask, mask_group, fro2A, fro2K, Gout, loss_part, Sp,
                               stream_wgs_per_cu() * grid_cap, planes, s);
        return;
    }
    ARMOR_DISPATCH_B_SMALL(d.b, {
        dim3 grid(std::min(d.nblocks, grid_cap)), block(Chain<BB>::NT);
        hipLaunchKernelGGL((phase_WS_kernel<BB>), grid, block, 0, s, Wbar, C, A, B, D, AtA, K, mask, mask_group,
                           fro2A, d.nbi * gram_parts(d.b), fro2K, d.nbj * gram_parts(d.b), d.d_in, d.nbj, d.nblocks, Gout,
                           loss_part, Sp);
    });
}

} // namespace armor
