// Proxy loss against the whole Gram matrix:  L_H = tr(R H R^T) = || R X^T ||_F^2  for H = X^T X, with the
// residual R = Wbar - A S B of the factorization (Sec. 2 writes the layer-wise objective with the
// activations themselves; Eq. 2, which the method optimises, keeps only diag(H)).  Evaluation only: the block
// decomposition of Eq. 5 does not hold for a non-diagonal weight, so nothing in Alg. 1-3 uses this value.
//
// One workgroup per T x T tile (pt, qt) of the product Q = R H:  Q_tile = sum_k R[pt, k] H[k, qt] over the
// d_in / T inner tiles, both operand tiles staged global -> registers -> LDS one step ahead of the matrix
// work (the product loop of the d_block 256 chains), then  <R[pt, qt], Q_tile>  as this tile's share of
// the loss.  T = 128 with the products on the bf16 matrix instruction (fp32 operands cut exactly into three
// bf16 pieces, six partial products) when both dimensions are multiples of 128, else T = 32 on the fp32
// instruction.  gfx950 only.
#include "chain_common.h"

#include <algorithm>

namespace armor {

namespace {

struct CfgFull128 { static constexpr int WM = 2, WN = 2, TM = 2, TN = 2; static constexpr bool SPLIT = true; };

template <int T, class CF>
__global__ __launch_bounds__((Chain<T, CF>::NT)) void full_h_loss_kernel(const float *__restrict__ R, int64_t d_in,
                                                                       const float *__restrict__ H, int64_t ldh,
                                                                       int ntr, int ntc, float *__restrict__ part) {
    using CH = Chain<T, CF>;
    __shared__ Smem<T> sm;
    const int tid = threadIdx.x;
    const typename CH::Pos p(tid);
    const int ldr = (int)d_in, ldhh = (int)ldh;
    for (int tile = blockIdx.x; tile < ntr * ntc; tile += gridDim.x) {
        // consecutive workgroups share the row panel of R and walk neighbouring column panels of H
        const int pt = tile / ntc, qt = tile % ntc;
        const float *Rp = R + (int64_t)pt * T * d_in;
        typename CH::TileRegs tx, ty;
        typename CH::Acc acc;
        acc.zero();
        __syncthreads(); // the previous tile's last product is done with the LDS slots
        CH::gload_tile(tx, Rp, ldr, tid);
        CH::gload_tile(ty, H + (int64_t)qt * T, ldhh, tid);
        CH::lstore_tile(sm.X, tx, tid);
        CH::lstore_tile(sm.Y, ty, tid);
        __syncthreads();
        float rp[CH::TM][CH::TN][16]; // R[pt, qt] in the accumulator layout, requested under the last step
        for (int kt = 0; kt < ntc; ++kt) {
            const bool more = kt + 1 < ntc;
            if (more) {
                CH::gload_tile(tx, Rp + (int64_t)(kt + 1) * T, ldr, tid);
                CH::gload_tile(ty, H + (int64_t)(kt + 1) * T * ldh + (int64_t)qt * T, ldhh, tid);
            }
            CH::template mma<false, false, false, true, false>(acc, sm.X, sm.Y, nullptr, p, [&]() {
                if (!more) {
                    const uint32_t lb = opaque_u(p.lane_boff(ldr));
#pragma unroll
                    for (int tm = 0; tm < CH::TM; ++tm)
#pragma unroll
                        for (int tn = 0; tn < CH::TN; ++tn)
#pragma unroll
                            for (int r = 0; r < 16; ++r)
                                rp[tm][tn][r] = gld(Rp + (int64_t)qt * T, lb + CH::Pos::unif_boff(tm, tn, r, ldr));
                }
            });
            __syncthreads();
            if (more) {
                CH::lstore_tile(sm.X, tx, tid);
                CH::lstore_tile(sm.Y, ty, tid);
            }
            __syncthreads();
        }
        float lsum = 0.f;
#pragma unroll
        for (int tm = 0; tm < CH::TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < CH::TN; ++tn)
#pragma unroll
                for (int r = 0; r < 16; ++r) lsum += rp[tm][tn][r] * acc.v[tm][tn][r];
        const float ltot = CH::block_sum(lsum, sm.red, tid);
        if (tid == 0) part[tile] = ltot;
    }
}

} // namespace

int full_h_tile(int64_t d_out, int64_t d_in) { return (d_out % 128 == 0 && d_in % 128 == 0) ? 128 : 32; }

int64_t full_h_parts(int64_t d_out, int64_t d_in) {
    const int t = full_h_tile(d_out, d_in);
    return (d_out / t) * (d_in / t);
}

// R: d_out x d_in fp32 (leading dimension d_in); H: d_in x d_in fp32, leading dimension ldh (symmetric);
// part: full_h_parts() floats, one per tile, every one written.
void launch_full_h_loss(const float *R, int64_t d_out, int64_t d_in, const float *H, int64_t ldh, float *part,
                        int grid_cap, hipStream_t s) {
    const int t = full_h_tile(d_out, d_in);
    const int ntr = (int)(d_out / t), ntc = (int)(d_in / t);
    const int ntiles = ntr * ntc;
    if (t == 128) {
        using CH = Chain<128, CfgFull128>;
        hipLaunchKernelGGL((full_h_loss_kernel<128, CfgFull128>), dim3(std::min(ntiles, grid_cap)), dim3(CH::NT), 0, s, R,
                           d_in, H, ldh, ntr, ntc, part);
    } else {
        using CH = Chain<32>;
        hipLaunchKernelGGL((full_h_loss_kernel<32, Cfg<32>>), dim3(std::min(ntiles, 8 * grid_cap)), dim3(CH::NT), 0, s, R,
                           d_in, H, ldh, ntr, ntc, part);
    }
}

} // namespace armor
