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
#include "armor_internal.h"

namespace armor {

typedef float floatx16 __attribute__((ext_vector_type(16)));

template <int B> struct Cfg;
template <> struct Cfg<32>  { static constexpr int WM = 1, WN = 1, TM = 1, TN = 1; };
template <> struct Cfg<64>  { static constexpr int WM = 2, WN = 2, TM = 1, TN = 1; };
template <> struct Cfg<128> { static constexpr int WM = 2, WN = 4, TM = 2, TN = 1; };

template <int B> struct Chain {
    static constexpr int WM = Cfg<B>::WM, WN = Cfg<B>::WN, TM = Cfg<B>::TM, TN = Cfg<B>::TN;
    static constexpr int NW = WM * WN, NT = NW * 64, P = B + 1;
    static constexpr int TILE_FLOATS = B * P;
    static_assert(WM * TM * 32 == B && WN * TN * 32 == B, "wave tiling must cover the block");

    struct Acc {
        floatx16 v[TM][TN];
        __device__ void zero() {
#pragma unroll
            for (int a = 0; a < TM; ++a)
#pragma unroll
                for (int c = 0; c < TN; ++c)
#pragma unroll
                    for (int r = 0; r < 16; ++r) v[a][c][r] = 0.f;
        }
    };

    // position of this lane's accumulator element r of sub-tile (tm,tn) inside the b x b block
    struct Pos {
        int wm0, wn0, l32, kh;
        __device__ Pos(int tid) {
            int w = tid >> 6, lane = tid & 63;
            wm0 = (w % WM) * TM * 32;
            wn0 = (w / WM) * TN * 32;
            l32 = lane & 31;
            kh = lane >> 5;
        }
        __device__ int row(int tm, int r) const { return wm0 + tm * 32 + (r >> 2) * 8 + kh * 4 + (r & 3); }
        __device__ int col(int tn) const { return wn0 + tn * 32 + l32; }
    };

    // global (row-major, leading dimension ld) -> LDS tile
    __device__ static void load_tile(float *T, const float *__restrict__ g, int64_t ld, int tid) {
        constexpr int V = B * B / 4, PER = V / NT;
        static_assert(V % NT == 0, "tile load must divide evenly");
        float4 v[PER];
#pragma unroll
        for (int it = 0; it < PER; ++it) {
            int idx = it * NT + tid, r = idx / (B / 4), c4 = idx % (B / 4);
            v[it] = *reinterpret_cast<const float4 *>(g + (int64_t)r * ld + c4 * 4);
        }
#pragma unroll
        for (int it = 0; it < PER; ++it) {
            int idx = it * NT + tid, r = idx / (B / 4), c4 = idx % (B / 4);
            float *t = T + r * P + c4 * 4;
            t[0] = v[it].x; t[1] = v[it].y; t[2] = v[it].z; t[3] = v[it].w;
        }
    }

    __device__ static void store_acc(float *T, const Acc &acc, const Pos &p) {
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                for (int r = 0; r < 16; ++r) T[p.row(tm, r) * P + p.col(tn)] = acc.v[tm][tn][r];
    }

    // acc += op(L) * op(R) over the b inner indices.  op(L)(m,k) = LT ? L[k][m] : L[m][k];
    // op(R)(k,n) = RT ? R[n][k] : R[k][n];  SCALE multiplies op(L)(m,k) by Dk[k].
    template <bool LT, bool RT, bool SCALE>
    __device__ static void mma(Acc &acc, const float *__restrict__ L, const float *__restrict__ R,
                               const float *__restrict__ Dk, const Pos &p) {
#pragma unroll 8
        for (int k = 0; k < B; k += 2) {
            int kk = k + p.kh;
            float a[TM], b[TN];
#pragma unroll
            for (int tm = 0; tm < TM; ++tm) {
                int m = p.wm0 + tm * 32 + p.l32;
                a[tm] = LT ? L[kk * P + m] : L[m * P + kk];
                if (SCALE) a[tm] *= Dk[kk];
            }
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) {
                int n = p.wn0 + tn * 32 + p.l32;
                b[tn] = RT ? R[n * P + kk] : R[kk * P + n];
            }
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < TN; ++tn)
                    acc.v[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[tm], b[tn], acc.v[tm][tn], 0, 0, 0);
        }
    }

    // deterministic block-wide sum; result valid in thread 0.  red: NW floats of LDS.
    __device__ static float block_sum(float v, float *red, int tid) {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
        __syncthreads();
        if ((tid & 63) == 0) red[tid >> 6] = v;
        __syncthreads();
        float s = 0.f;
        if (tid == 0)
            for (int w = 0; w < NW; ++w) s += red[w];
        return s;
    }
};

template <int B> struct Smem {
    float X[Chain<B>::TILE_FLOATS];
    float Y[Chain<B>::TILE_FLOATS];
    float Dl[B];
    float red[16];
};

// ------------------------------------------------------------------------------------------------
// A-phase (Alg. 2, first gradient step; App. D.1).  Workgroup (i, c) walks the column blocks j of
// its chunk c and accumulates  sum_j (R D)^(i,j) S^(i,j)T  in registers.
//   gpart[(i*nsplit + c)][b][b] = -2 * that sum          (partial grad_A^(i))
//   beta_part[i*nbj + j] = || S^(i,j) D^(j) S^(i,j)T ||_F (Eq. 9 summand / 2)
//   loss_part[i*nbj + j] = sum (R^(i,j))^2 D^(j)          (Eq. 5 summand)
// LOSS_ONLY stops after the block loss.
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
    const int i = blockIdx.x / nsplit, c = blockIdx.x % nsplit;
    const int chunk = (nbj + nsplit - 1) / nsplit;
    const int j0 = c * chunk, j1 = min(nbj, j0 + chunk);
    typename CH::Acc gacc, acc;
    gacc.zero();
    for (int j = j0; j < j1; ++j) {
        const float *Cij = C + (int64_t)i * B * d_in + (int64_t)j * B;
        const float *Wij = Wbar + (int64_t)i * B * d_in + (int64_t)j * B;
        CH::load_tile(sm.X, Cij, d_in, tid);
        CH::load_tile(sm.Y, Bw + (int64_t)j * B * B, B, tid);
        if (tid < B) sm.Dl[tid] = D[(int64_t)j * B + tid];
        __syncthreads();
        acc.zero();
        CH::template mma<false, false, false>(acc, sm.X, sm.Y, nullptr, p); // S = C B
        __syncthreads();
        CH::store_acc(sm.X, acc, p);
        CH::load_tile(sm.Y, A + (int64_t)i * B * B, B, tid);
        float wb[CH::TM][CH::TN][16];
#pragma unroll
        for (int tm = 0; tm < CH::TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < CH::TN; ++tn)
#pragma unroll
                for (int r = 0; r < 16; ++r) wb[tm][tn][r] = Wij[(int64_t)p.row(tm, r) * d_in + p.col(tn)];
        __syncthreads();
        acc.zero();
        CH::template mma<false, false, false>(acc, sm.Y, sm.X, nullptr, p); // What = A S
        float lsum = 0.f;
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
        float ltot = CH::block_sum(lsum, sm.red, tid); // (has barriers: every wave is done reading Y)
        if (tid == 0) loss_part[i * nbj + j] = ltot;
        if (!LOSS_ONLY) {
            CH::store_acc(sm.Y, acc, p); // R D
            __syncthreads();
            CH::template mma<false, true, false>(gacc, sm.Y, sm.X, nullptr, p); // += (R D) S^T
            acc.zero();
            CH::template mma<false, true, true>(acc, sm.X, sm.X, sm.Dl, p); // (S D) S^T
            float f2 = 0.f;
#pragma unroll
            for (int tm = 0; tm < CH::TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < CH::TN; ++tn)
#pragma unroll
                    for (int r = 0; r < 16; ++r) f2 += acc.v[tm][tn][r] * acc.v[tm][tn][r];
            float ftot = CH::block_sum(f2, sm.red, tid);
            if (tid == 0) beta_part[i * nbj + j] = sqrtf(ftot);
        }
        __syncthreads();
    }
    if (!LOSS_ONLY) {
        float *gp = gpart + (int64_t)blockIdx.x * B * B;
#pragma unroll
        for (int tm = 0; tm < CH::TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < CH::TN; ++tn)
#pragma unroll
                for (int r = 0; r < 16; ++r) gp[p.row(tm, r) * B + p.col(tn)] = -2.f * gacc.v[tm][tn][r];
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
    float *__restrict__ gpart, float *__restrict__ beta_part) {
    using CH = Chain<B>;
    __shared__ Smem<B> sm;
    const int tid = threadIdx.x;
    const typename CH::Pos p(tid);
    const int j = blockIdx.x / nsplit, c = blockIdx.x % nsplit;
    const int chunk = (nbi + nsplit - 1) / nsplit;
    const int i0 = c * chunk, i1 = min(nbi, i0 + chunk);
    typename CH::Acc gacc, acc;
    gacc.zero();
    if (tid < B) sm.Dl[tid] = D[(int64_t)j * B + tid];
    __syncthreads();
    float dn2 = 0.f;
    if (tid == 0)
        for (int q = 0; q < B; ++q) dn2 += sm.Dl[q] * sm.Dl[q];
    for (int i = i0; i < i1; ++i) {
        const float *Cij = C + (int64_t)i * B * d_in + (int64_t)j * B;
        const float *Wij = Wbar + (int64_t)i * B * d_in + (int64_t)j * B;
        CH::load_tile(sm.X, Cij, d_in, tid);
        CH::load_tile(sm.Y, A + (int64_t)i * B * B, B, tid);
        __syncthreads();
        acc.zero();
        CH::template mma<false, false, false>(acc, sm.Y, sm.X, nullptr, p); // S' = A C
        __syncthreads();
        CH::store_acc(sm.X, acc, p);
        CH::load_tile(sm.Y, Bw + (int64_t)j * B * B, B, tid);
        float wb[CH::TM][CH::TN][16];
#pragma unroll
        for (int tm = 0; tm < CH::TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < CH::TN; ++tn)
#pragma unroll
                for (int r = 0; r < 16; ++r) wb[tm][tn][r] = Wij[(int64_t)p.row(tm, r) * d_in + p.col(tn)];
        __syncthreads();
        acc.zero();
        CH::template mma<false, false, false>(acc, sm.X, sm.Y, nullptr, p); // What = S' B
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
        CH::template mma<true, false, false>(gacc, sm.X, sm.Y, nullptr, p); // += S'^T (R D)
        acc.zero();
        CH::template mma<true, false, false>(acc, sm.X, sm.X, nullptr, p); // S'^T S'
        float f2 = 0.f;
#pragma unroll
        for (int tm = 0; tm < CH::TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < CH::TN; ++tn)
#pragma unroll
                for (int r = 0; r < 16; ++r) f2 += acc.v[tm][tn][r] * acc.v[tm][tn][r];
        float ftot = CH::block_sum(f2, sm.red, tid);
        if (tid == 0) beta_part[i * nbj + j] = sqrtf(ftot) * sqrtf(dn2);
        __syncthreads();
    }
    float *gp = gpart + (int64_t)blockIdx.x * B * B;
#pragma unroll
    for (int tm = 0; tm < CH::TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < CH::TN; ++tn)
#pragma unroll
            for (int r = 0; r < 16; ++r) gp[p.row(tm, r) * B + p.col(tn)] = -2.f * gacc.v[tm][tn][r];
}

// ------------------------------------------------------------------------------------------------
// Core gradient (App. D.3 without the mask):  G^(i,j) = A^(i)T ((Wbar - A C B) D)^(i,j) B^(j)T.
//   MODE 0: the W' step of Alg. 2:  C <- C + (2 / beta_W') G on kept entries (Eq. 11).
//   MODE 1: Gout = -2 G for every entry (the selection scores and the q-vectors of Alg. 3 read
//           it), and the block loss (= loss after the continuous step) to loss_part.
// One workgroup per block; blocks are independent.
// ------------------------------------------------------------------------------------------------
template <int B, int MODE>
__global__ __launch_bounds__(Chain<B>::NT) void phase_G_kernel(
    const float *__restrict__ Wbar, float *__restrict__ C, const float *__restrict__ A,
    const float *__restrict__ Bw, const float *__restrict__ D, const uint8_t *__restrict__ mask, int mask_group,
    const double *__restrict__ scalars, int64_t d_in, int nbj, float *__restrict__ Gout,
    float *__restrict__ loss_part) {
    using CH = Chain<B>;
    __shared__ Smem<B> sm;
    const int tid = threadIdx.x;
    const typename CH::Pos p(tid);
    const int i = blockIdx.x / nbj, j = blockIdx.x % nbj;
    float *Cij = C + (int64_t)i * B * d_in + (int64_t)j * B;
    const float *Wij = Wbar + (int64_t)i * B * d_in + (int64_t)j * B;
    typename CH::Acc acc;
    CH::load_tile(sm.X, Cij, d_in, tid);
    CH::load_tile(sm.Y, A + (int64_t)i * B * B, B, tid);
    if (tid < B) sm.Dl[tid] = D[(int64_t)j * B + tid];
    __syncthreads();
    acc.zero();
    CH::template mma<false, false, false>(acc, sm.Y, sm.X, nullptr, p); // S' = A C
    __syncthreads();
    CH::store_acc(sm.X, acc, p);
    CH::load_tile(sm.Y, Bw + (int64_t)j * B * B, B, tid);
    float wb[CH::TM][CH::TN][16];
#pragma unroll
    for (int tm = 0; tm < CH::TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < CH::TN; ++tn)
#pragma unroll
            for (int r = 0; r < 16; ++r) wb[tm][tn][r] = Wij[(int64_t)p.row(tm, r) * d_in + p.col(tn)];
    __syncthreads();
    acc.zero();
    CH::template mma<false, false, false>(acc, sm.X, sm.Y, nullptr, p); // What = S' B
    float lsum = 0.f;
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
    if (MODE == 1) {
        float ltot = CH::block_sum(lsum, sm.red, tid);
        if (tid == 0) loss_part[blockIdx.x] = ltot;
    }
    __syncthreads();
    CH::store_acc(sm.X, acc, p); // R D   (Y still holds B^j)
    __syncthreads();
    acc.zero();
    CH::template mma<false, true, false>(acc, sm.X, sm.Y, nullptr, p); // U = (R D) B^T
    __syncthreads();
    CH::store_acc(sm.X, acc, p);
    CH::load_tile(sm.Y, A + (int64_t)i * B * B, B, tid);
    __syncthreads();
    acc.zero();
    CH::template mma<true, false, false>(acc, sm.Y, sm.X, nullptr, p); // G = A^T U
    if (MODE == 0) {
        const double bw = scalars[2];
        const float eta2 = bw > 0.0 ? (float)(2.0 / bw) : 0.f;
        const int64_t mrow = d_in / mask_group;
#pragma unroll
        for (int tm = 0; tm < CH::TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < CH::TN; ++tn)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    int row = p.row(tm, r), col = p.col(tn);
                    int64_t gcol = (int64_t)j * B + col;
                    uint8_t mb = mask[((int64_t)i * B + row) * mrow + gcol / mask_group];
                    if ((mb >> (gcol % mask_group)) & 1) {
                        float *cp = Cij + (int64_t)row * d_in + col;
                        *cp = *cp + eta2 * acc.v[tm][tn][r];
                    }
                }
    } else {
        float *Gij = Gout + (int64_t)i * B * d_in + (int64_t)j * B;
#pragma unroll
        for (int tm = 0; tm < CH::TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < CH::TN; ++tn)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    Gij[(int64_t)p.row(tm, r) * d_in + p.col(tn)] = -2.f * acc.v[tm][tn][r];
    }
}

// ------------------------------------------------------------------------------------------------
// Small Gram-type products of the wrappers themselves (Eq. 11 and the shortcuts of Alg. 3):
//   blockIdx <  nbi : colnorm2[i*b+p] = ||A^(i)[:,p]||^2 (= ||a||^2 of Eq. 7), fro2A[i] = ||A^iT A^i||_F^2
//   blockIdx >= nbi : K^(j) = B^(j) D^(j) B^(j)T (holds every B' D B'^T of Eq. 7), fro2K[j] = ||K^j||_F^2
// ------------------------------------------------------------------------------------------------
template <int B>
__global__ __launch_bounds__(Chain<B>::NT) void wrapper_grams_kernel(
    const float *__restrict__ A, const float *__restrict__ Bw, const float *__restrict__ D, int nbi,
    float *__restrict__ colnorm2, float *__restrict__ fro2A, float *__restrict__ K, float *__restrict__ fro2K) {
    using CH = Chain<B>;
    __shared__ Smem<B> sm;
    const int tid = threadIdx.x;
    const typename CH::Pos p(tid);
    typename CH::Acc acc;
    acc.zero();
    const bool isA = (int)blockIdx.x < nbi;
    const int idx = isA ? blockIdx.x : blockIdx.x - nbi;
    CH::load_tile(sm.X, (isA ? A : Bw) + (int64_t)idx * B * B, B, tid);
    if (!isA && tid < B) sm.Dl[tid] = D[(int64_t)idx * B + tid];
    __syncthreads();
    if (isA) CH::template mma<true, false, false>(acc, sm.X, sm.X, nullptr, p); // A^T A
    else     CH::template mma<false, true, true>(acc, sm.X, sm.X, sm.Dl, p);    // (B D) B^T
    float f2 = 0.f;
#pragma unroll
    for (int tm = 0; tm < CH::TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < CH::TN; ++tn)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                float v = acc.v[tm][tn][r];
                f2 += v * v;
                int row = p.row(tm, r), col = p.col(tn);
                if (isA) { if (row == col) colnorm2[(int64_t)idx * B + row] = v; }
                else K[(int64_t)idx * B * B + row * B + col] = v;
            }
    float ftot = CH::block_sum(f2, sm.red, tid);
    if (tid == 0) (isA ? fro2A : fro2K)[idx] = ftot;
}

// ------------------------------------------------------------------------------------------------
// host launchers
// ------------------------------------------------------------------------------------------------
int chain_max_nsplit() { return 64; }

#define ARMOR_DISPATCH_B(bval, ...)                      \
    switch (bval) {                                      \
    case 32:  { constexpr int BB = 32;  __VA_ARGS__; } break; \
    case 64:  { constexpr int BB = 64;  __VA_ARGS__; } break; \
    case 128: { constexpr int BB = 128; __VA_ARGS__; } break; \
    default: break;                                      \
    }

void launch_phase_A(const Dims &d, const float *Wbar, const float *C, const float *A, const float *B,
                    const float *D, int nsplit, float *gpart, float *beta_part, float *loss_part,
                    bool loss_only, hipStream_t s) {
    ARMOR_DISPATCH_B(d.b, {
        dim3 grid(d.nbi * nsplit), block(Chain<BB>::NT);
        if (loss_only)
            hipLaunchKernelGGL((phase_A_kernel<BB, true>), grid, block, 0, s, Wbar, C, A, B, D, d.d_in, d.nbj,
                               nsplit, gpart, beta_part, loss_part);
        else
            hipLaunchKernelGGL((phase_A_kernel<BB, false>), grid, block, 0, s, Wbar, C, A, B, D, d.d_in, d.nbj,
                               nsplit, gpart, beta_part, loss_part);
    });
}

void launch_phase_B(const Dims &d, const float *Wbar, const float *C, const float *A, const float *B,
                    const float *D, int nsplit, float *gpart, float *beta_part, hipStream_t s) {
    ARMOR_DISPATCH_B(d.b, {
        dim3 grid(d.nbj * nsplit), block(Chain<BB>::NT);
        hipLaunchKernelGGL((phase_B_kernel<BB>), grid, block, 0, s, Wbar, C, A, B, D, d.d_in, d.nbi, d.nbj, nsplit,
                           gpart, beta_part);
    });
}

void launch_phase_G(const Dims &d, const float *Wbar, float *C, const float *A, const float *B, const float *D,
                    const uint8_t *mask, int mask_group, const double *scalars, float *Gout, float *loss_part,
                    int mode, hipStream_t s) {
    ARMOR_DISPATCH_B(d.b, {
        dim3 grid(d.nblocks), block(Chain<BB>::NT);
        if (mode == 0)
            hipLaunchKernelGGL((phase_G_kernel<BB, 0>), grid, block, 0, s, Wbar, C, A, B, D, mask, mask_group,
                               scalars, d.d_in, d.nbj, Gout, loss_part);
        else
            hipLaunchKernelGGL((phase_G_kernel<BB, 1>), grid, block, 0, s, Wbar, C, A, B, D, mask, mask_group,
                               scalars, d.d_in, d.nbj, Gout, loss_part);
    });
}

void launch_wrapper_grams(const Dims &d, const float *A, const float *B, const float *D, float *colnorm2,
                          float *fro2A, float *K, float *fro2K, hipStream_t s) {
    ARMOR_DISPATCH_B(d.b, {
        dim3 grid(d.nbi + d.nbj), block(Chain<BB>::NT);
        hipLaunchKernelGGL((wrapper_grams_kernel<BB>), grid, block, 0, s, A, B, D, d.nbi, colnorm2, fro2A, K, fro2K);
    });
}

} // namespace armor
