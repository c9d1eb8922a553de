// Chains for wrapper blocks larger than one LDS tile (d_block = 256): the same products as
// chain.hip, computed on 128 x 128 sub-tiles.  A b x b operand no longer fits in LDS (256 KB), so
// the intermediates of a block (S or S', R D, U, Delta, V) live in a per-workgroup scratch area in
// global memory that is written and re-read by the same workgroup only and therefore stays in
// L2; every sub-product streams its two operand sub-tiles through the two LDS tile slots.
// At b = 256 each product has 64 flop/B of arithmetic intensity even unfused, so the extra L2
// round trips cost little against the matrix time.
#include "chain_common.h"

#include <algorithm>

namespace armor {

namespace {

constexpr int TB = 128; // sub-tile edge
// Four waves, each a 64 x 64 patch of a sub-tile, products on the bf16 matrix instruction (1), or the
// eight waves of 64 x 32 and the fp32 instruction (0).  The cut of an fp32 operand into its bf16 pieces
// costs 11 vector instructions per pair of values, so the larger patch (each operand value cut by two
// waves instead of four and two) is what keeps the cuts below the matrix time; it needs the 512
// registers of a one-wave-per-SIMD workgroup.  28672 x 8192, one iteration: 14.2 ms against 15.3 ms.
#ifndef ARMOR_BIG_BF16X3
#define ARMOR_BIG_BF16X3 1
#endif
#if ARMOR_BIG_BF16X3
struct CfgBig { static constexpr int WM = 2, WN = 2, TM = 2, TN = 2; static constexpr bool SPLIT = true; };
#else
struct CfgBig { static constexpr int WM = 2, WN = 4, TM = 2, TN = 1; static constexpr bool SPLIT = false; };
#endif
using CH = Chain<TB, CfgBig>;

// acc over the NS inner sub-tiles of  op(L) (pt, :) * op(R) (:, qt)  for every output sub-tile,
// then epi(pt, qt, acc).  L, R: b x b row-major with leading dimensions ldl, ldr (global memory;
// may be this workgroup's scratch: the leading barrier orders its earlier stores before the loads;
// no product writes one of its own operands).  The two operand sub-tiles of the next step are
// requested into registers before the matrix work of the current one and go to LDS after it, so
// the L2 round trip is hidden.  SYM: the product is symmetric and only its Frobenius norm is
// wanted, so output sub-tiles below the diagonal are skipped (the caller counts the others twice).
// pre(pt, qt) runs before the last matrix step of an output sub-tile: the place to request what
// the epilogue reads from global memory, so that its latency is covered by that step.
template <int NS, bool LT, bool RT, bool SCALE, bool SYM, class Pre, class Epi>
__device__ __forceinline__ void big_mma(Smem<TB> &sm, int tid, const CH::Pos &p, const float *__restrict__ L, int ldl,
                                        const float *__restrict__ R, int ldr, const float *__restrict__ Dk,
                                        Pre &&pre, Epi &&epi) {
    auto lsub = [&](int pt, int rt) { return LT ? L + (rt * TB) * ldl + pt * TB : L + (pt * TB) * ldl + rt * TB; };
    auto rsub = [&](int qt, int rt) { return RT ? R + (qt * TB) * ldr + rt * TB : R + (rt * TB) * ldr + qt * TB; };
    CH::TileRegs tx, ty;
    float dnext = 0.f;
    __syncthreads();
    CH::gload_tile(tx, lsub(0, 0), ldl, tid);
    CH::gload_tile(ty, rsub(0, 0), ldr, tid);
    if (SCALE && tid < TB) dnext = Dk[tid];
    CH::lstore_tile(sm.X, tx, tid);
    CH::lstore_tile(sm.Y, ty, tid);
    if (SCALE && tid < TB) sm.Dl[tid] = dnext;
    __syncthreads();
    for (int pt = 0; pt < NS; ++pt)
        for (int qt = SYM ? pt : 0; qt < NS; ++qt) {
            CH::Acc acc;
            acc.zero();
            for (int rt = 0; rt < NS; ++rt) {
                // the step after this one
                int nr = rt + 1, nq = qt, np = pt;
                if (nr == NS) { nr = 0; ++nq; }
                if (nq == NS) { ++np; nq = SYM ? np : 0; }
                const bool more = np < NS;
                if (more) {
                    CH::gload_tile(tx, lsub(np, nr), ldl, tid);
                    CH::gload_tile(ty, rsub(nq, nr), ldr, tid);
                    if (SCALE && tid < TB) dnext = Dk[nr * TB + tid];
                }
                CH::template mma<LT, RT, SCALE, true, false>(acc, sm.X, sm.Y, sm.Dl, p, [&]() { if (rt == NS - 1) pre(pt, qt); });
                __syncthreads();
                if (more) {
                    CH::lstore_tile(sm.X, tx, tid);
                    CH::lstore_tile(sm.Y, ty, tid);
                    if (SCALE && tid < TB) sm.Dl[tid] = dnext;
                }
                __syncthreads();
            }
            epi(pt, qt, acc);
        }
}

// visit every accumulator element of output sub-tile (pt, qt): f(off, value, ...) with off the byte
// offset (for gld / gst) in a row-major fp32 matrix of leading dimension ld
struct NoPre {
    __device__ void operator()(int, int) const {}
};

// this lane's 32 elements of output sub-tile (pt, qt) of a row-major matrix: load / visit
struct Patch {
    float v[CH::TM][CH::TN][16];
};
__device__ __forceinline__ void load_patch(Patch &w, const float *__restrict__ g, const CH::Pos &p, int pt, int qt,
                                           int ld) {
    const uint32_t base = opaque_u(4u * (uint32_t)((pt * TB + p.wm0 + p.kh * 4) * ld + qt * TB + p.wn0 + p.l32));
#pragma unroll
    for (int tm = 0; tm < CH::TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < CH::TN; ++tn)
#pragma unroll
            for (int r = 0; r < 16; ++r) w.v[tm][tn][r] = gld(g, base + CH::Pos::unif_boff(tm, tn, r, ld));
}

template <class F>
__device__ __forceinline__ void for_acc(CH::Acc &acc, const CH::Pos &p, int pt, int qt, int ld, F &&f) {
    const uint32_t base = opaque_u(4u * (uint32_t)((pt * TB + p.wm0 + p.kh * 4) * ld + qt * TB + p.wn0 + p.l32));
#pragma unroll
    for (int tm = 0; tm < CH::TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < CH::TN; ++tn)
#pragma unroll
            for (int r = 0; r < 16; ++r) f(base + CH::Pos::unif_boff(tm, tn, r, ld), acc.v[tm][tn][r], tm, tn, r);
}

// ---- A-phase (see chain.hip) -------------------------------------------------------------------
template <int NS, bool LOSS_ONLY>
__global__ __launch_bounds__(CH::NT) void big_phase_A_kernel(
    const float *__restrict__ Wbar, const float *__restrict__ C, const float *__restrict__ A,
    const float *__restrict__ Bw, const float *__restrict__ D, int64_t d_in, int nbj, int nsplit, int nitems,
    float *__restrict__ gpart, float *__restrict__ beta_part, float *__restrict__ loss_part,
    float *__restrict__ scratch) {
    constexpr int b = NS * TB;
    __shared__ Smem<TB> sm;
    const int tid = threadIdx.x;
    const CH::Pos p(tid);
    const int ldw = (int)d_in;
    float *s0 = scratch + (int64_t)blockIdx.x * 2 * b * b, *s1 = s0 + b * b;
    const int chunk = (nbj + nsplit - 1) / nsplit;
    for (int item = blockIdx.x; item < nitems; item += gridDim.x) { // item = (row block i, chunk c)
    const int i = item / nsplit, c = item % nsplit;
    const int j0 = c * chunk, j1 = min(nbj, j0 + chunk);
    float *gp = gpart + (int64_t)item * b * b;
    const float *Ai = A + (int64_t)i * b * b;
    for (int j = j0; j < j1; ++j) {
        const float *Cij = C + (int64_t)i * b * d_in + (int64_t)j * b;
        const float *Wij = Wbar + (int64_t)i * b * d_in + (int64_t)j * b;
        const float *Bj = Bw + (int64_t)j * b * b, *Dj = D + (int64_t)j * b;
        big_mma<NS, false, false, false, false>(sm, tid, p, Cij, ldw, Bj, b, nullptr, NoPre(), [&](int pt, int qt, CH::Acc &acc) {
            for_acc(acc, p, pt, qt, b, [&](uint32_t off, float v, int, int, int) { gst(s0, off, v); }); // S = C B
        });
        float lsum = 0.f;
        Patch wp;
        big_mma<NS, false, false, false, false>(sm, tid, p, Ai, b, s0, b, nullptr,
                                                [&](int pt, int qt) { load_patch(wp, Wij, p, pt, qt, ldw); },
                                                [&](int pt, int qt, CH::Acc &acc) {
#pragma unroll
            for (int tm = 0; tm < CH::TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < CH::TN; ++tn) {
                    const float dj = Dj[qt * TB + p.col(tn)];
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        float res = wp.v[tm][tn][r] - acc.v[tm][tn][r];
                        lsum += res * res * dj;
                        acc.v[tm][tn][r] = res * dj;
                    }
                }
            if (!LOSS_ONLY) for_acc(acc, p, pt, qt, b, [&](uint32_t off, float v, int, int, int) { gst(s1, off, v); });
            else if (gpart != nullptr) // loss-only pass: R D of the block, laid out like Wbar (see phase_A_kernel)
                for_acc(acc, p, pt, qt, ldw, [&](uint32_t off, float v, int, int, int) {
                    gst(gpart + (int64_t)i * b * d_in + (int64_t)j * b, off, v);
                });
        });
        float ltot = CH::block_sum(lsum, sm.red, tid);
        if (tid == 0) loss_part[i * nbj + j] = ltot;
        if (!LOSS_ONLY) {
            const bool first = j == j0;
            big_mma<NS, false, true, false, false>(sm, tid, p, s1, b, s0, b, nullptr,
                                                   [&](int pt, int qt) { if (!first) load_patch(wp, gp, p, pt, qt, b); },
                                                   [&](int pt, int qt, CH::Acc &acc) {
                for_acc(acc, p, pt, qt, b, [&](uint32_t off, float v, int tm, int tn, int r) {
                    gst(gp, off, (first ? 0.f : wp.v[tm][tn][r]) - 2.f * v); // += -2 (R D) S^T, same workgroup, fixed order
                });
            });
            float f2 = 0.f;
            big_mma<NS, false, true, true, true>(sm, tid, p, s0, b, s0, b, Dj, NoPre(), [&](int pt, int qt, CH::Acc &acc) {
                float t2 = 0.f; // S D S^T is symmetric: upper sub-tiles only, off-diagonal ones twice
#pragma unroll
                for (int tm = 0; tm < CH::TM; ++tm)
#pragma unroll
                    for (int tn = 0; tn < CH::TN; ++tn)
#pragma unroll
                        for (int r = 0; r < 16; ++r) t2 += acc.v[tm][tn][r] * acc.v[tm][tn][r];
                f2 += pt == qt ? t2 : 2.f * t2;
            });
            float ftot = CH::block_sum(f2, sm.red, tid);
            if (tid == 0) beta_part[i * nbj + j] = sqrtf(ftot);
        }
    }
    }
}

// ---- B-phase -----------------------------------------------------------------------------------
template <int NS>
__global__ __launch_bounds__(CH::NT) void big_phase_B_kernel(
    const float *__restrict__ Wbar, const float *__restrict__ C, const float *__restrict__ A,
    const float *__restrict__ Bw, const float *__restrict__ D, int64_t d_in, int nbi, int nbj, int nsplit,
    int nitems, float *__restrict__ gpart, float *__restrict__ beta_part, float *__restrict__ Sp,
    float *__restrict__ scratch) {
    constexpr int b = NS * TB;
    __shared__ Smem<TB> sm;
    const int tid = threadIdx.x;
    const CH::Pos p(tid);
    const int ldw = (int)d_in;
    float *s0 = scratch + (int64_t)blockIdx.x * 2 * b * b, *s1 = s0 + b * b;
    const int chunk = (nbi + nsplit - 1) / nsplit;
    for (int item = blockIdx.x; item < nitems; item += gridDim.x) { // item = (column block j, chunk c)
    const int j = item / nsplit, c = item % nsplit;
    const int i0 = c * chunk, i1 = min(nbi, i0 + chunk);
    float *gp = gpart + (int64_t)item * b * b;
    const float *Bj = Bw + (int64_t)j * b * b, *Dj = D + (int64_t)j * b;
    float dn2 = 0.f;
    if (tid == 0)
        for (int q = 0; q < b; ++q) dn2 += Dj[q] * Dj[q];
    for (int i = i0; i < i1; ++i) {
        const float *Cij = C + (int64_t)i * b * d_in + (int64_t)j * b;
        const float *Wij = Wbar + (int64_t)i * b * d_in + (int64_t)j * b;
        const float *Ai = A + (int64_t)i * b * b;
        float *Spij = Sp ? Sp + (int64_t)i * b * d_in + (int64_t)j * b : nullptr;
        big_mma<NS, false, false, false, false>(sm, tid, p, Ai, b, Cij, ldw, nullptr, NoPre(), [&](int pt, int qt, CH::Acc &acc) {
            for_acc(acc, p, pt, qt, b, [&](uint32_t off, float v, int, int, int) { gst(s0, off, v); }); // S' = A C
            // the W' step sees the same A and C: hand S' over instead of forming it again there
            if (Spij) for_acc(acc, p, pt, qt, ldw, [&](uint32_t off, float v, int, int, int) { gst(Spij, off, v); });
        });
        Patch wp;
        big_mma<NS, false, false, false, false>(sm, tid, p, s0, b, Bj, b, nullptr,
                                                [&](int pt, int qt) { load_patch(wp, Wij, p, pt, qt, ldw); },
                                                [&](int pt, int qt, CH::Acc &acc) {
#pragma unroll
            for (int tm = 0; tm < CH::TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < CH::TN; ++tn) {
                    const float dj = Dj[qt * TB + p.col(tn)];
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc.v[tm][tn][r] = (wp.v[tm][tn][r] - acc.v[tm][tn][r]) * dj;
                }
            for_acc(acc, p, pt, qt, b, [&](uint32_t off, float v, int, int, int) { gst(s1, off, v); }); // R D
        });
        const bool first = i == i0;
        big_mma<NS, true, false, false, false>(sm, tid, p, s0, b, s1, b, nullptr,
                                               [&](int pt, int qt) { if (!first) load_patch(wp, gp, p, pt, qt, b); },
                                               [&](int pt, int qt, CH::Acc &acc) {
            for_acc(acc, p, pt, qt, b, [&](uint32_t off, float v, int tm, int tn, int r) {
                gst(gp, off, (first ? 0.f : wp.v[tm][tn][r]) - 2.f * v); // += -2 S'^T (R D)
            });
        });
        float f2 = 0.f;
        big_mma<NS, true, false, false, true>(sm, tid, p, s0, b, s0, b, nullptr, NoPre(), [&](int pt, int qt, CH::Acc &acc) {
            float t2 = 0.f; // S'^T S' is symmetric: upper sub-tiles only, off-diagonal ones twice
#pragma unroll
            for (int tm = 0; tm < CH::TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < CH::TN; ++tn)
#pragma unroll
                    for (int r = 0; r < 16; ++r) t2 += acc.v[tm][tn][r] * acc.v[tm][tn][r];
            f2 += pt == qt ? t2 : 2.f * t2;
        });
        float ftot = CH::block_sum(f2, sm.red, tid);
        if (tid == 0) beta_part[i * nbj + j] = sqrtf(ftot) * sqrtf(dn2);
    }
    }
}

// ---- W' step (FUSED = false) or W' step + core gradient at the updated core (FUSED = true) --------
template <int NS, bool FUSED>
__global__ __launch_bounds__(CH::NT) void big_phase_WS_kernel(
    const float *__restrict__ Wbar, float *__restrict__ C, const float *__restrict__ A,
    const float *__restrict__ Bw, const float *__restrict__ D, const float *__restrict__ AtA,
    const float *__restrict__ K, const uint8_t *__restrict__ mask, int mask_group,
    const float *__restrict__ fro2A, int nA, const float *__restrict__ fro2K, int nK, int64_t d_in, int nbj,
    int nblocks, float *__restrict__ Gout, float *__restrict__ loss_part, const float *__restrict__ Sp,
    float *__restrict__ scratch) {
    constexpr int b = NS * TB;
    __shared__ Smem<TB> sm;
    const int tid = threadIdx.x;
    const CH::Pos p(tid);
    const int ldw = (int)d_in;
    publish_eta_W(sm, tid, fro2A, nA, fro2K, nK);
    __syncthreads();
    const float eta2 = read_eta_W(sm);
    const int64_t mrow = d_in / mask_group;
    float *s0 = scratch + (int64_t)blockIdx.x * 2 * b * b, *s1 = s0 + b * b;
    for (int blk = blockIdx.x; blk < nblocks; blk += gridDim.x) {
        const int i = blk / nbj, j = blk % nbj;
        float *Cij = C + (int64_t)i * b * d_in + (int64_t)j * b;
        const float *Wij = Wbar + (int64_t)i * b * d_in + (int64_t)j * b;
        const float *Ai = A + (int64_t)i * b * b, *Bj = Bw + (int64_t)j * b * b, *Dj = D + (int64_t)j * b;
        float *Gij = FUSED ? Gout + (int64_t)i * b * d_in + (int64_t)j * b : nullptr;
        const float *Sl = s0; // S' = A C: from the B step when it left it, else formed here
        int lds = b;
        if (Sp) {
            Sl = Sp + (int64_t)i * b * d_in + (int64_t)j * b;
            lds = ldw;
        } else {
            big_mma<NS, false, false, false, false>(sm, tid, p, Ai, b, Cij, ldw, nullptr, NoPre(), [&](int pt, int qt, CH::Acc &acc) {
                for_acc(acc, p, pt, qt, b, [&](uint32_t off, float v, int, int, int) { gst(s0, off, v); });
            });
        }
        float lsum = 0.f;
        Patch wp;
        big_mma<NS, false, false, false, false>(sm, tid, p, Sl, lds, Bj, b, nullptr,
                                                [&](int pt, int qt) { load_patch(wp, Wij, p, pt, qt, ldw); },
                                                [&](int pt, int qt, CH::Acc &acc) {
#pragma unroll
            for (int tm = 0; tm < CH::TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < CH::TN; ++tn) {
                    const float dj = Dj[qt * TB + p.col(tn)];
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        float res = wp.v[tm][tn][r] - acc.v[tm][tn][r];
                        lsum += res * res * dj;
                        acc.v[tm][tn][r] = res * dj;
                    }
                }
            for_acc(acc, p, pt, qt, b, [&](uint32_t off, float v, int, int, int) { gst(s1, off, v); }); // R D
        });
        big_mma<NS, false, true, false, false>(sm, tid, p, s1, b, Bj, b, nullptr, NoPre(), [&](int pt, int qt, CH::Acc &acc) {
            for_acc(acc, p, pt, qt, b, [&](uint32_t off, float v, int, int, int) { gst(s0, off, v); }); // U = (R D) B^T
        });
        float dd = 0.f;
        uint32_t mb[CH::TM][CH::TN][4]; // mask bytes of this lane's elements (four to a register), requested under the last matrix step
        auto load_mask = [&](int pt, int qt) {
#pragma unroll
            for (int tm = 0; tm < CH::TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < CH::TN; ++tn) {
                    const int64_t gcol = (int64_t)j * b + qt * TB + p.col(tn);
                    const uint8_t *mp = mask + ((int64_t)i * b + pt * TB + p.wm0 + p.kh * 4) * mrow + gcol / mask_group;
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        uint32_t w = 0;
#pragma unroll
                        for (int r = 4 * q; r < 4 * q + 4; ++r)
                            w |= (uint32_t)mp[(int64_t)(tm * 32 + (r >> 2) * 8 + (r & 3)) * mrow] << (8 * (r & 3));
                        mb[tm][tn][q] = w;
                    }
                }
        };
        auto pre_G = [&](int pt, int qt) {
            load_patch(wp, Cij, p, pt, qt, ldw);
            load_mask(pt, qt);
        };
        big_mma<NS, true, false, false, false>(sm, tid, p, Ai, b, s0, b, nullptr, pre_G, [&](int pt, int qt, CH::Acc &acc) {
            // G = A^T U: W' step on kept entries; Delta -> s1, raw G -> Gout (fused mode)
            const uint32_t cbase = opaque_u(4u * (uint32_t)((pt * TB + p.wm0 + p.kh * 4) * ldw + qt * TB + p.wn0 + p.l32));
            const uint32_t sbase = opaque_u(4u * (uint32_t)((pt * TB + p.wm0 + p.kh * 4) * b + qt * TB + p.wn0 + p.l32));
#pragma unroll
            for (int tm = 0; tm < CH::TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < CH::TN; ++tn) {
                    const int64_t gcol = (int64_t)j * b + qt * TB + p.col(tn);
                    const int sh = (int)(gcol % mask_group);
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const bool kp = (mb[tm][tn][r >> 2] >> (8 * (r & 3) + sh)) & 1u;
                        const float g = acc.v[tm][tn][r], dl = kp ? g : 0.f;
                        dd += dl * dl;
                        if (kp) gst(Cij, cbase + CH::Pos::unif_boff(tm, tn, r, ldw), wp.v[tm][tn][r] + eta2 * dl);
                        if (FUSED) {
                            gst(s1, sbase + CH::Pos::unif_boff(tm, tn, r, b), dl);
                            gst(Gij, cbase + CH::Pos::unif_boff(tm, tn, r, ldw), g);
                        }
                    }
                }
            asm volatile("" : "+v"(dd)); // formed here: otherwise the masked values stay in registers until the sum is used
        });
        if (FUSED) {
            big_mma<NS, false, false, false, false>(sm, tid, p, s1, b, K + (int64_t)j * b * b, b, nullptr, NoPre(),
                                             [&](int pt, int qt, CH::Acc &acc) {
                for_acc(acc, p, pt, qt, b, [&](uint32_t off, float v, int, int, int) { gst(s0, off, v); }); // V = Delta K
            });
            float dz = 0.f;
            // the raw G of this lane's elements (written by this lane above); Delta is G on the kept entries
            big_mma<NS, false, false, false, false>(sm, tid, p, AtA + (int64_t)i * b * b, b, s0, b, nullptr,
                                             [&](int pt, int qt) {
                                                 load_patch(wp, Gij, p, pt, qt, ldw);
                                                 load_mask(pt, qt);
                                             },
                                             [&](int pt, int qt, CH::Acc &acc) {
                // Z = (A^T A) V:  G_new = G - eta Z;  <Delta, Z>
                const uint32_t cbase = opaque_u(4u * (uint32_t)((pt * TB + p.wm0 + p.kh * 4) * ldw + qt * TB + p.wn0 + p.l32));
#pragma unroll
                for (int tm = 0; tm < CH::TM; ++tm)
#pragma unroll
                    for (int tn = 0; tn < CH::TN; ++tn) {
                        const int sh = (int)(((int64_t)j * b + qt * TB + p.col(tn)) % mask_group);
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const float z = acc.v[tm][tn][r];
                            const bool kp = (mb[tm][tn][r >> 2] >> (8 * (r & 3) + sh)) & 1u;
                            dz += kp ? wp.v[tm][tn][r] * z : 0.f;
                            gst(Gij, cbase + CH::Pos::unif_boff(tm, tn, r, ldw), -2.f * (wp.v[tm][tn][r] - eta2 * z));
                        }
                    }
            });
            float ltot = CH::block_sum(lsum - 2.f * eta2 * dd + eta2 * eta2 * dz, sm.red, tid);
            if (tid == 0) loss_part[blk] = ltot;
        }
    }
}

// ---- joint-Adam forward/backward (see phase_FB_kernel in chain.hip) ----------------------------------
// Per block: S = C B -> s0, R D -> s1, grad_A partial += -2 (R D) S^T, T = A^T (R D) -> s0 (S is dead),
// grad_B partial = -2 C^T T (old core), then T B^T with the Adam update of the core in its epilogue.
template <int NS>
__global__ __launch_bounds__(CH::NT) void big_phase_FB_kernel(
    const float *__restrict__ Wbar, float *__restrict__ C, const float *__restrict__ A,
    const float *__restrict__ Bw, const float *__restrict__ D, const uint8_t *__restrict__ mask, int mask_group,
    float *__restrict__ mC, float *__restrict__ vC, AdamCoef k, int64_t d_in, int nbi, int nbj, int nsplit, int nitems,
    float *__restrict__ gApart, float *__restrict__ gBpart, float *__restrict__ loss_part,
    float *__restrict__ scratch) {
    constexpr int b = NS * TB;
    __shared__ Smem<TB> sm;
    const int tid = threadIdx.x;
    const CH::Pos p(tid);
    const int ldw = (int)d_in;
    const int64_t mrow = d_in / mask_group;
    float *s0 = scratch + (int64_t)blockIdx.x * 2 * b * b, *s1 = s0 + b * b;
    const int chunk = (nbj + nsplit - 1) / nsplit;
    for (int item = blockIdx.x; item < nitems; item += gridDim.x) { // item = (row block i, chunk c)
    const int i = item / nsplit, c = item % nsplit;
    const int j0 = c * chunk, j1 = min(nbj, j0 + chunk);
    float *gp = gApart + (int64_t)item * b * b;
    const float *Ai = A + (int64_t)i * b * b;
    if (j0 >= j1) { // empty chunk: its partial is still summed by the wrapper update
        for (int e = tid; e < b * b; e += CH::NT) gp[e] = 0.f;
        continue;
    }
    for (int j = j0; j < j1; ++j) {
        float *Cij = C + (int64_t)i * b * d_in + (int64_t)j * b;
        const float *Wij = Wbar + (int64_t)i * b * d_in + (int64_t)j * b;
        const float *Bj = Bw + (int64_t)j * b * b, *Dj = D + (int64_t)j * b;
        big_mma<NS, false, false, false, false>(sm, tid, p, Cij, ldw, Bj, b, nullptr, NoPre(), [&](int pt, int qt, CH::Acc &acc) {
            for_acc(acc, p, pt, qt, b, [&](uint32_t off, float v, int, int, int) { gst(s0, off, v); }); // S = C B
        });
        float lsum = 0.f;
        Patch wp;
        big_mma<NS, false, false, false, false>(sm, tid, p, Ai, b, s0, b, nullptr,
                                                [&](int pt, int qt) { load_patch(wp, Wij, p, pt, qt, ldw); },
                                                [&](int pt, int qt, CH::Acc &acc) {
#pragma unroll
            for (int tm = 0; tm < CH::TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < CH::TN; ++tn) {
                    const float dj = Dj[qt * TB + p.col(tn)];
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        float res = wp.v[tm][tn][r] - acc.v[tm][tn][r];
                        lsum += res * res * dj;
                        acc.v[tm][tn][r] = res * dj;
                    }
                }
            for_acc(acc, p, pt, qt, b, [&](uint32_t off, float v, int, int, int) { gst(s1, off, v); }); // R D
        });
        float ltot = CH::block_sum(lsum, sm.red, tid);
        if (tid == 0) loss_part[i * nbj + j] = ltot;
        const bool first = j == j0;
        big_mma<NS, false, true, false, false>(sm, tid, p, s1, b, s0, b, nullptr,
                                               [&](int pt, int qt) { if (!first) load_patch(wp, gp, p, pt, qt, b); },
                                               [&](int pt, int qt, CH::Acc &acc) {
            for_acc(acc, p, pt, qt, b, [&](uint32_t off, float v, int tm, int tn, int r) {
                gst(gp, off, (first ? 0.f : wp.v[tm][tn][r]) - 2.f * v); // += -2 (R D) S^T, same workgroup, fixed order
            });
        });
        big_mma<NS, true, false, false, false>(sm, tid, p, Ai, b, s1, b, nullptr, NoPre(), [&](int pt, int qt, CH::Acc &acc) {
            for_acc(acc, p, pt, qt, b, [&](uint32_t off, float v, int, int, int) { gst(s0, off, v); }); // T = A^T (R D)
        });
        float *gb = gBpart + ((int64_t)j * nbi + i) * b * b;
        big_mma<NS, true, false, false, false>(sm, tid, p, Cij, ldw, s0, b, nullptr, NoPre(), [&](int pt, int qt, CH::Acc &acc) {
            for_acc(acc, p, pt, qt, b, [&](uint32_t off, float v, int, int, int) { gst(gb, off, -2.f * v); }); // C^T T, old core
        });
        float *mij = mC + (int64_t)i * b * d_in + (int64_t)j * b, *vij = vC + (int64_t)i * b * d_in + (int64_t)j * b;
        uint32_t mb[CH::TM][CH::TN][4];
        auto pre_C = [&](int pt, int qt) {
            load_patch(wp, Cij, p, pt, qt, ldw);
#pragma unroll
            for (int tm = 0; tm < CH::TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < CH::TN; ++tn) {
                    const int64_t gcol = (int64_t)j * b + qt * TB + p.col(tn);
                    const uint8_t *mp = mask + ((int64_t)i * b + pt * TB + p.wm0 + p.kh * 4) * mrow + gcol / mask_group;
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        uint32_t w = 0;
#pragma unroll
                        for (int r = 4 * q; r < 4 * q + 4; ++r)
                            w |= (uint32_t)mp[(int64_t)(tm * 32 + (r >> 2) * 8 + (r & 3)) * mrow] << (8 * (r & 3));
                        mb[tm][tn][q] = w;
                    }
                }
        };
        big_mma<NS, false, true, false, false>(sm, tid, p, s0, b, Bj, b, nullptr, pre_C, [&](int pt, int qt, CH::Acc &acc) {
            // T B^T: Adam on the core, g = -2 (T B^T) (.) M; the moments decay on pruned entries too
            const uint32_t cbase = opaque_u(4u * (uint32_t)((pt * TB + p.wm0 + p.kh * 4) * ldw + qt * TB + p.wn0 + p.l32));
#pragma unroll
            for (int tm = 0; tm < CH::TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < CH::TN; ++tn) {
                    const int sh = (int)(((int64_t)j * b + qt * TB + p.col(tn)) % mask_group);
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const uint32_t off = cbase + CH::Pos::unif_boff(tm, tn, r, ldw);
                        const bool kp = (mb[tm][tn][r >> 2] >> (8 * (r & 3) + sh)) & 1u;
                        const float g = kp ? -2.f * acc.v[tm][tn][r] : 0.f;
                        const float mn = k.b1 * gld(mij, off) + k.one_minus_b1 * g;
                        const float vn = k.b2 * gld(vij, off) + k.one_minus_b2 * g * g;
                        gst(mij, off, mn);
                        gst(vij, off, vn);
                        if (kp) gst(Cij, off, wp.v[tm][tn][r] - k.lr * (mn * k.inv_c1) / (sqrtf(vn * k.inv_c2) + k.eps));
                    }
                }
        });
    }
    }
}

// ---- core gradient at the current point (see phase_GS_kernel in chain.hip) ------------------------------
template <int NS>
__global__ __launch_bounds__(CH::NT) void big_phase_GS_kernel(
    const float *__restrict__ Wbar, const float *__restrict__ C, const float *__restrict__ A,
    const float *__restrict__ Bw, const float *__restrict__ D, int64_t d_in, int nbj, int nblocks,
    float *__restrict__ Gout, float *__restrict__ loss_part, float *__restrict__ scratch) {
    constexpr int b = NS * TB;
    __shared__ Smem<TB> sm;
    const int tid = threadIdx.x;
    const CH::Pos p(tid);
    const int ldw = (int)d_in;
    float *s0 = scratch + (int64_t)blockIdx.x * 2 * b * b, *s1 = s0 + b * b;
    for (int blk = blockIdx.x; blk < nblocks; blk += gridDim.x) {
        const int i = blk / nbj, j = blk % nbj;
        const float *Cij = C + (int64_t)i * b * d_in + (int64_t)j * b;
        const float *Wij = Wbar + (int64_t)i * b * d_in + (int64_t)j * b;
        const float *Ai = A + (int64_t)i * b * b, *Bj = Bw + (int64_t)j * b * b, *Dj = D + (int64_t)j * b;
        float *Gij = Gout + (int64_t)i * b * d_in + (int64_t)j * b;
        big_mma<NS, false, false, false, false>(sm, tid, p, Ai, b, Cij, ldw, nullptr, NoPre(), [&](int pt, int qt, CH::Acc &acc) {
            for_acc(acc, p, pt, qt, b, [&](uint32_t off, float v, int, int, int) { gst(s0, off, v); }); // S' = A C
        });
        float lsum = 0.f;
        Patch wp;
        big_mma<NS, false, false, false, false>(sm, tid, p, s0, b, Bj, b, nullptr,
                                                [&](int pt, int qt) { load_patch(wp, Wij, p, pt, qt, ldw); },
                                                [&](int pt, int qt, CH::Acc &acc) {
#pragma unroll
            for (int tm = 0; tm < CH::TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < CH::TN; ++tn) {
                    const float dj = Dj[qt * TB + p.col(tn)];
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        float res = wp.v[tm][tn][r] - acc.v[tm][tn][r];
                        lsum += res * res * dj;
                        acc.v[tm][tn][r] = res * dj;
                    }
                }
            for_acc(acc, p, pt, qt, b, [&](uint32_t off, float v, int, int, int) { gst(s1, off, v); }); // R D
        });
        big_mma<NS, false, true, false, false>(sm, tid, p, s1, b, Bj, b, nullptr, NoPre(), [&](int pt, int qt, CH::Acc &acc) {
            for_acc(acc, p, pt, qt, b, [&](uint32_t off, float v, int, int, int) { gst(s0, off, v); }); // U = (R D) B^T
        });
        big_mma<NS, true, false, false, false>(sm, tid, p, Ai, b, s0, b, nullptr, NoPre(), [&](int pt, int qt, CH::Acc &acc) {
            for_acc(acc, p, pt, qt, ldw, [&](uint32_t off, float v, int, int, int) { gst(Gij, off, -2.f * v); }); // -2 A^T U
        });
        float ltot = CH::block_sum(lsum, sm.red, tid);
        if (tid == 0) loss_part[blk] = ltot;
    }
}

// ---- wrapper Grams -----------------------------------------------------------------------------
template <int NS>
__global__ __launch_bounds__(CH::NT) void big_wrapper_grams_kernel(
    const float *__restrict__ A, const float *__restrict__ Bw, const float *__restrict__ D, int nbi,
    float *__restrict__ colnorm2, float *__restrict__ fro2A, float *__restrict__ AtA, float *__restrict__ K,
    float *__restrict__ fro2K) {
    constexpr int b = NS * TB;
    __shared__ Smem<TB> sm;
    const int tid = threadIdx.x;
    const CH::Pos p(tid);
    const bool isA = (int)blockIdx.x < nbi;
    const int idx = isA ? blockIdx.x : blockIdx.x - nbi;
    const float *src = (isA ? A : Bw) + (int64_t)idx * b * b;
    float *dst = (isA ? AtA : K) + (int64_t)idx * b * b;
    float f2 = 0.f;
    auto epi = [&](int pt, int qt, CH::Acc &acc) {
        for_acc(acc, p, pt, qt, b, [&](uint32_t off, float v, int, int, int) {
            const int e = (int)(off / 4u); // element index in the b x b result
            f2 += v * v;
            gst(dst, off, v);
            if (isA && e / b == e % b) colnorm2[(int64_t)idx * b + e / b] = v;
        });
    };
    if (isA) big_mma<NS, true, false, false, false>(sm, tid, p, src, b, src, b, nullptr, NoPre(), epi);          // A^T A
    else     big_mma<NS, false, true, true, false>(sm, tid, p, src, b, src, b, D + (int64_t)idx * b, NoPre(), epi); // (B D) B^T
    float ftot = CH::block_sum(f2, sm.red, tid);
    if (tid == 0) (isA ? fro2A : fro2K)[idx] = ftot;
}

} // namespace

size_t big_scratch_floats(const Dims &d, int max_wgs) { return (size_t)max_wgs * 2 * d.b * d.b; }

void launch_big_phase_A(const Dims &d, const float *Wbar, const float *C, const float *A, const float *B,
                        const float *D, int nsplit, float *gpart, float *beta_part, float *loss_part, bool loss_only,
                        int grid_cap, float *scratch, hipStream_t s) {
    const int nitems = d.nbi * nsplit;
    dim3 grid(std::min(nitems, grid_cap)), block(CH::NT);
    if (loss_only) // (the kernel's gradient argument doubles as the residual output in this mode: never the partials)
        hipLaunchKernelGGL((big_phase_A_kernel<2, true>), grid, block, 0, s, Wbar, C, A, B, D, d.d_in, d.nbj, nsplit,
                           nitems, (float *)nullptr, beta_part, loss_part, scratch);
    else
        hipLaunchKernelGGL((big_phase_A_kernel<2, false>), grid, block, 0, s, Wbar, C, A, B, D, d.d_in, d.nbj, nsplit,
                           nitems, gpart, beta_part, loss_part, scratch);
}

// Loss-only forward pass at d_block 256 that also leaves the residual R D in Rout (d_out x d_in, leading dimension d_in).
void launch_big_residual(const Dims &d, const float *Wbar, const float *C, const float *A, const float *B,
                         const float *D, int nsplit, float *Rout, float *loss_part, int grid_cap, float *scratch,
                         hipStream_t s) {
    const int nitems = d.nbi * nsplit;
    hipLaunchKernelGGL((big_phase_A_kernel<2, true>), dim3(std::min(nitems, grid_cap)), dim3(CH::NT), 0, s, Wbar, C, A, B, D,
                       d.d_in, d.nbj, nsplit, nitems, Rout, (float *)nullptr, loss_part, scratch);
}

void launch_big_phase_B(const Dims &d, const float *Wbar, const float *C, const float *A, const float *B,
                        const float *D, int nsplit, float *gpart, float *beta_part, float *Sp, int grid_cap,
                        float *scratch, hipStream_t s) {
    const int nitems = d.nbj * nsplit;
    hipLaunchKernelGGL((big_phase_B_kernel<2>), dim3(std::min(nitems, grid_cap)), dim3(CH::NT), 0, s, Wbar, C, A, B, D,
                       d.d_in, d.nbi, d.nbj, nsplit, nitems, gpart, beta_part, Sp, scratch);
}

void launch_big_phase_WS(const Dims &d, const float *Wbar, float *C, const float *A, const float *B, const float *D,
                         const float *AtA, const float *K, const uint8_t *mask, int mask_group, const float *fro2A,
                         const float *fro2K, float *Gout, float *loss_part, const float *Sp, bool fused, int grid_cap, float *scratch,
                         hipStream_t s) {
    dim3 grid(std::min(d.nblocks, grid_cap)), block(CH::NT);
    if (fused)
        hipLaunchKernelGGL((big_phase_WS_kernel<2, true>), grid, block, 0, s, Wbar, C, A, B, D, AtA, K, mask,
                           mask_group, fro2A, d.nbi, fro2K, d.nbj, d.d_in, d.nbj, d.nblocks, Gout, loss_part, Sp, scratch);
    else
        hipLaunchKernelGGL((big_phase_WS_kernel<2, false>), grid, block, 0, s, Wbar, C, A, B, D, AtA, K, mask,
                           mask_group, fro2A, d.nbi, fro2K, d.nbj, d.d_in, d.nbj, d.nblocks, Gout, loss_part, Sp, scratch);
}

void launch_big_phase_FB(const Dims &d, const float *Wbar, float *C, const float *A, const float *B, const float *D,
                         const uint8_t *mask, int mask_group, float *mC, float *vC, double lr, double b1, double b2,
                         double eps, int64_t t, int nsplit, float *gApart, float *gBpart, float *loss_part, int grid_cap,
                         float *scratch, hipStream_t s) {
    const AdamCoef k = make_adam_coef(lr, b1, b2, eps, t);
    const int nitems = d.nbi * nsplit;
    hipLaunchKernelGGL((big_phase_FB_kernel<2>), dim3(std::min(nitems, grid_cap)), dim3(CH::NT), 0, s, Wbar, C, A, B, D,
                       mask, mask_group, mC, vC, k, d.d_in, d.nbi, d.nbj, nsplit, nitems, gApart, gBpart, loss_part,
                       scratch);
}

void launch_big_phase_GS(const Dims &d, const float *Wbar, const float *C, const float *A, const float *B,
                         const float *D, float *Gout, float *loss_part, int grid_cap, float *scratch, hipStream_t s) {
    hipLaunchKernelGGL((big_phase_GS_kernel<2>), dim3(std::min(d.nblocks, grid_cap)), dim3(CH::NT), 0, s, Wbar, C, A, B,
                       D, d.d_in, d.nbj, d.nblocks, Gout, loss_part, scratch);
}

void launch_big_wrapper_grams(const Dims &d, const float *A, const float *B, const float *D, float *colnorm2,
                              float *fro2A, float *AtA, float *K, float *fro2K, hipStream_t s) {
    hipLaunchKernelGGL((big_wrapper_grams_kernel<2>), dim3(d.nbi + d.nbj), dim3(CH::NT), 0, s, A, B, D, d.nbi,
                       colnorm2, fro2A, AtA, K, fro2K);
}

} // namespace armor
