// HBM-bound and small kernels around the contraction chains: normalisation (Sec. 3.2),
// initialisation (Eq. 3), wrapper updates (Alg. 2), the sparse-core step (Alg. 3, Eq. 6-8),
// denormalisation and N:M packing.  gfx950; 64-wide waves; every reduction has a fixed order.
#include "armor_internal.h"
#include "planes.h"

#include <algorithm>
#include <cmath>

namespace armor {

__device__ __forceinline__ float bf16_bits_to_float(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }

template <bool BF16> __device__ __forceinline__ float load_w(const void *W, int64_t idx) {
    if (BF16) return bf16_bits_to_float(reinterpret_cast<const uint16_t *>(W)[idx]);
    return reinterpret_cast<const float *>(W)[idx];
}

// deterministic sum over a 256-thread workgroup; result in every thread
__device__ __forceinline__ double block_sum_256(double v, double *red) {
    const int tid = threadIdx.x;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    __syncthreads();
    if ((tid & 63) == 0) red[tid >> 6] = v;
    __syncthreads();
    return (red[0] + red[1]) + (red[2] + red[3]);
}

// ------------------------------------------------------------------------------------------------
// normalisation (Sec. 3.2)
// ------------------------------------------------------------------------------------------------
// A run of VEC consecutive entries of W as floats: 16 bytes per load (8 bf16 or 4 fp32).
template <bool BF16> struct WVec {
    static constexpr int VEC = BF16 ? 8 : 4;
    float v[VEC];
    __device__ __forceinline__ void load(const void *W, int64_t idx) { // idx: element index, multiple of VEC
        if (BF16) {
            const uint4 q = *reinterpret_cast<const uint4 *>(reinterpret_cast<const uint16_t *>(W) + idx);
            const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                v[2 * e] = __uint_as_float(w[e] << 16);
                v[2 * e + 1] = __uint_as_float(w[e] & 0xffff0000u);
            }
        } else {
            const float4 q = *reinterpret_cast<const float4 *>(reinterpret_cast<const float *>(W) + idx);
            v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
        }
    }
};

// Column sums of squares over one chunk of rows.  Workgroup = 64 column threads (VEC columns each) x 4 row
// lanes; the four row lanes are added in a fixed order through LDS.  Requires d_in % VEC == 0.
template <bool BF16>
__global__ __launch_bounds__(256) void colnorm_partial_kernel(const void *__restrict__ W, int64_t d_out,
                                                              int64_t d_in, int nchunk,
                                                              float *__restrict__ partial) {
    constexpr int VEC = WVec<BF16>::VEC;
    __shared__ float red[3][64][VEC + 1];
    const int cx = threadIdx.x & 63, ry = threadIdx.x >> 6;
    const int64_t j = ((int64_t)blockIdx.x * 64 + cx) * VEC;
    const int c = blockIdx.y;
    const int64_t rows = (d_out + nchunk - 1) / nchunk, r0 = c * rows, r1 = min(d_out, r0 + rows);
    float s[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) s[e] = 0.f;
    if (j < d_in) {
#pragma unroll 4
        for (int64_t i = r0 + ry; i < r1; i += 4) {
            WVec<BF16> w;
            w.load(W, i * d_in + j);
#pragma unroll
            for (int e = 0; e < VEC; ++e) s[e] += w.v[e] * w.v[e];
        }
    }
    if (ry > 0) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) red[ry - 1][cx][e] = s[e];
    }
    __syncthreads();
    if (ry == 0 && j < d_in) {
#pragma unroll
        for (int e = 0; e < VEC; ++e)
            partial[(int64_t)c * d_in + j + e] = (s[e] + red[0][cx][e]) + (red[1][cx][e] + red[2][cx][e]);
    }
}

// scalar form for widths that are not a multiple of the vector length
template <bool BF16>
__global__ __launch_bounds__(256) void colnorm_partial_scalar_kernel(const void *__restrict__ W, int64_t d_out,
                                                                     int64_t d_in, int nchunk,
                                                                     float *__restrict__ partial) {
    int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
    int c = blockIdx.y;
    int64_t rows = (d_out + nchunk - 1) / nchunk, r0 = c * rows, r1 = min(d_out, r0 + rows);
    if (j >= d_in) return;
    float s = 0.f;
    for (int64_t i = r0; i < r1; ++i) {
        float w = load_w<BF16>(W, i * d_in + j);
        s += w * w;
    }
    partial[(int64_t)c * d_in + j] = s;
}

// r1 (zero norms replaced by 1) and its reciprocal.  64 columns x 16 chunk lanes per workgroup: lane y adds
// chunks y, y+16, ... in order (fp64), the 16 lane sums are then added in lane order.
__global__ __launch_bounds__(1024) void colnorm_final_kernel(const float *__restrict__ partial, int64_t d_in,
                                                             int nchunk, float *__restrict__ r1,
                                                             float *__restrict__ r1_inv) {
    __shared__ double red[16][64];
    const int cx = threadIdx.x & 63, cy = threadIdx.x >> 6;
    const int64_t j = (int64_t)blockIdx.x * 64 + cx;
    double s = 0.0;
    if (j < d_in)
        for (int c = cy; c < nchunk; c += 16) s += (double)partial[(int64_t)c * d_in + j];
    red[cy][cx] = s;
    __syncthreads();
    if (cy == 0 && j < d_in) {
        double t = 0.0;
#pragma unroll
        for (int y = 0; y < 16; ++y) t += red[y][cx];
        float r = (float)sqrt(t);
        r = r > 0.f ? r : 1.f;
        r1[j] = r;
        r1_inv[j] = 1.f / r;
    }
}

// One workgroup per row: W1 = W / r1, r2 = its row norm, Wbar = W1 / r2.  The first KEEP vectors of
// a thread stay in registers between the two passes; longer rows are read again (L2).
template <bool BF16, bool VECTOR>
__global__ __launch_bounds__(256) void rownorm_scale_kernel(const void *__restrict__ W, int64_t d_in,
                                                            const float *__restrict__ r1_inv, float *__restrict__ r2,
                                                            float *__restrict__ Wbar) {
    __shared__ double red[4];
    const int64_t i = blockIdx.x;
    const int tid = threadIdx.x;
    if (VECTOR) {
        constexpr int VEC = WVec<BF16>::VEC, KEEP = 4;
        const int64_t nvec = d_in / VEC;
        WVec<BF16> keep[KEEP];
        double s = 0.0;
#pragma unroll
        for (int u = 0; u < KEEP; ++u) {
            const int64_t v = tid + (int64_t)u * 256;
            if (v < nvec) {
                keep[u].load(W, i * d_in + v * VEC);
                float part = 0.f;
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    keep[u].v[e] *= r1_inv[v * VEC + e];
                    part += keep[u].v[e] * keep[u].v[e];
                }
                s += (double)part;
            }
        }
        for (int64_t v = tid + (int64_t)KEEP * 256; v < nvec; v += 256) {
            WVec<BF16> w;
            w.load(W, i * d_in + v * VEC);
            float part = 0.f;
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                const float w1 = w.v[e] * r1_inv[v * VEC + e];
                part += w1 * w1;
            }
            s += (double)part;
        }
        s = block_sum_256(s, red);
        float r = (float)sqrt(s);
        r = r > 0.f ? r : 1.f;
        if (tid == 0) r2[i] = r;
        const float rinv = 1.f / r;
        auto store = [&](int64_t v, const float *w1) {
            float4 *dst = reinterpret_cast<float4 *>(Wbar + i * d_in + v * VEC);
#pragma unroll
            for (int q = 0; q < VEC / 4; ++q)
                dst[q] = make_float4(w1[4 * q] * rinv, w1[4 * q + 1] * rinv, w1[4 * q + 2] * rinv, w1[4 * q + 3] * rinv);
        };
#pragma unroll
        for (int u = 0; u < KEEP; ++u) {
            const int64_t v = tid + (int64_t)u * 256;
            if (v < nvec) store(v, keep[u].v);
        }
        for (int64_t v = tid + (int64_t)KEEP * 256; v < nvec; v += 256) {
            WVec<BF16> w;
            w.load(W, i * d_in + v * VEC);
#pragma unroll
            for (int e = 0; e < VEC; ++e) w.v[e] *= r1_inv[v * VEC + e];
            store(v, w.v);
        }
    } else {
        double s = 0.0;
        for (int64_t j = tid; j < d_in; j += 256) {
            float w1 = load_w<BF16>(W, i * d_in + j) * r1_inv[j];
            s += (double)w1 * (double)w1;
        }
        s = block_sum_256(s, red);
        float r = (float)sqrt(s);
        r = r > 0.f ? r : 1.f;
        if (tid == 0) r2[i] = r;
        const float rinv = 1.f / r;
        for (int64_t j = tid; j < d_in; j += 256) Wbar[i * d_in + j] = (load_w<BF16>(W, i * d_in + j) * r1_inv[j]) * rinv;
    }
}

// partial: [nchunk][d_in] floats followed by d_in floats for the reciprocal column norms
void launch_colnorm(const void *W, int bf16, int64_t d_out, int64_t d_in, float *partial, int nchunk, float *r1,
                    hipStream_t s) {
    float *r1_inv = partial + (int64_t)nchunk * d_in;
    const int vec = bf16 ? 8 : 4;
    if (d_in % vec == 0) {
        dim3 grid((unsigned)((d_in / vec + 63) / 64), nchunk);
        if (bf16) hipLaunchKernelGGL(colnorm_partial_kernel<true>, grid, dim3(256), 0, s, W, d_out, d_in, nchunk, partial);
        else      hipLaunchKernelGGL(colnorm_partial_kernel<false>, grid, dim3(256), 0, s, W, d_out, d_in, nchunk, partial);
    } else {
        dim3 grid((unsigned)((d_in + 255) / 256), nchunk);
        if (bf16) hipLaunchKernelGGL(colnorm_partial_scalar_kernel<true>, grid, dim3(256), 0, s, W, d_out, d_in, nchunk, partial);
        else      hipLaunchKernelGGL(colnorm_partial_scalar_kernel<false>, grid, dim3(256), 0, s, W, d_out, d_in, nchunk, partial);
    }
    hipLaunchKernelGGL(colnorm_final_kernel, dim3((unsigned)((d_in + 63) / 64)), dim3(1024), 0, s, partial, d_in,
                       nchunk, r1, r1_inv);
}

void launch_rownorm_scale(const void *W, int bf16, int64_t d_out, int64_t d_in, const float *r1_inv, float *r2,
                          float *Wbar, hipStream_t s) {
    const bool vec = d_in % (bf16 ? 8 : 4) == 0;
    dim3 grid((unsigned)d_out), block(256);
    if (bf16 && vec)       hipLaunchKernelGGL((rownorm_scale_kernel<true, true>), grid, block, 0, s, W, d_in, r1_inv, r2, Wbar);
    else if (bf16)         hipLaunchKernelGGL((rownorm_scale_kernel<true, false>), grid, block, 0, s, W, d_in, r1_inv, r2, Wbar);
    else if (vec)          hipLaunchKernelGGL((rownorm_scale_kernel<false, true>), grid, block, 0, s, W, d_in, r1_inv, r2, Wbar);
    else                   hipLaunchKernelGGL((rownorm_scale_kernel<false, false>), grid, block, 0, s, W, d_in, r1_inv, r2, Wbar);
}

// ------------------------------------------------------------------------------------------------
// initialisation (Eq. 3)
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void init_identity_kernel(float *__restrict__ A, int64_t total, int b) {
    int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= total) return;
    int64_t within = e % ((int64_t)b * b);
    A[e] = (within / b == within % b) ? 1.f : 0.f;
}

void launch_init_identity(float *A, int nblk, int b, hipStream_t s) {
    int64_t total = (int64_t)nblk * b * b;
    hipLaunchKernelGGL(init_identity_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, A, total, b);
}

// One thread per group of M columns: importance I = (w*w)*D_j in fp32, keep the N largest
// (equal scores: lower column wins), C = Wbar (.) M, one mask byte per group.
template <int M>
__global__ __launch_bounds__(256) void init_nm_kernel(const float *__restrict__ Wbar, const float *__restrict__ D,
                                                      int64_t d_in, int64_t ngroups, int N, float *__restrict__ C,
                                                      uint8_t *__restrict__ mask) {
    int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (g >= ngroups) return;
    int64_t gpr = d_in / M, col0 = (g % gpr) * M, base = (g / gpr) * d_in + col0;
    float w[M], sc[M];
#pragma unroll
    for (int p = 0; p < M; ++p) {
        w[p] = Wbar[base + p];
        float ww = __fmul_rn(w[p], w[p]);
        sc[p] = __fmul_rn(ww, D[col0 + p]);
    }
    uint32_t bits = 0;
#pragma unroll
    for (int p = 0; p < M; ++p) {
        int rank = 0;
#pragma unroll
        for (int q = 0; q < M; ++q) rank += (sc[q] > sc[p] || (sc[q] == sc[p] && q < p)) ? 1 : 0;
        bool keep = rank < N;
        bits |= keep ? (1u << p) : 0u;
        C[base + p] = keep ? w[p] : 0.f;
    }
    mask[g] = (uint8_t)bits;
}

void launch_init_nm(const float *Wbar, const float *D, int64_t d_out, int64_t d_in, int N, int M, float *C,
                    uint8_t *mask, hipStream_t s) {
    int64_t ngroups = d_out * (d_in / M);
    dim3 grid((unsigned)((ngroups + 255) / 256));
    switch (M) {
    case 2: hipLaunchKernelGGL(init_nm_kernel<2>, grid, dim3(256), 0, s, Wbar, D, d_in, ngroups, N, C, mask); break;
    case 4: hipLaunchKernelGGL(init_nm_kernel<4>, grid, dim3(256), 0, s, Wbar, D, d_in, ngroups, N, C, mask); break;
    case 8: hipLaunchKernelGGL(init_nm_kernel<8>, grid, dim3(256), 0, s, Wbar, D, d_in, ngroups, N, C, mask); break;
    default: break;
    }
}

__global__ __launch_bounds__(256) void diag_kernel(const float *__restrict__ H, int64_t d_in, int64_t ldh,
                                                   float *__restrict__ D) {
    int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (j < d_in) D[j] = H[j * ldh + j];
}

void launch_diag(const float *H, int64_t d_in, int64_t ldh, float *D, hipStream_t s) {
    hipLaunchKernelGGL(diag_kernel, dim3((unsigned)((d_in + 255) / 256)), dim3(256), 0, s, H, d_in, ldh, D);
}

// ------------------------------------------------------------------------------------------------
// The weights of Eq. 2 straight from the activations: D[j] (+)= sum_t X[t][j]^2, without forming H.
// This is all the method itself needs of the calibration data (2 n d_in bytes, HBM-bound).
// Chunk c of `rows_per_chunk` tokens -> partial[c][j] in fp32, then a fixed-order fp64 sum over the
// chunks.
// ------------------------------------------------------------------------------------------------
template <bool BF16>
__global__ __launch_bounds__(256) void diag_x_partial_kernel(const void *__restrict__ X, int64_t n, int64_t d_in,
                                                             int64_t ldx, int64_t rows_per_chunk,
                                                             float *__restrict__ partial) {
    // a workgroup reads 256 x 16 consecutive bytes of one token row per load instruction and walks
    // down the rows of its chunk, 8 rows in flight
    constexpr int VEC = WVec<BF16>::VEC;
    const int64_t j = ((int64_t)blockIdx.x * 256 + threadIdx.x) * VEC;
    const int64_t c = blockIdx.y, r0 = c * rows_per_chunk, r1 = min(n, r0 + rows_per_chunk);
    if (j >= d_in) return;
    float s[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) s[e] = 0.f;
    int64_t i = r0;
    for (; i + 8 <= r1; i += 8) {
        WVec<BF16> w[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) w[u].load(X, (i + u) * ldx + j);
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int e = 0; e < VEC; ++e) s[e] += w[u].v[e] * w[u].v[e];
    }
    for (; i < r1; ++i) {
        WVec<BF16> w;
        w.load(X, i * ldx + j);
#pragma unroll
        for (int e = 0; e < VEC; ++e) s[e] += w.v[e] * w.v[e];
    }
#pragma unroll
    for (int e = 0; e < VEC; ++e) partial[c * d_in + j + e] = s[e];
}

// 64 columns x 16 chunk lanes per workgroup: lane y adds chunks y, y+16, ... in order (fp64), the 16
// lane sums are then added in lane order
__global__ __launch_bounds__(1024) void diag_x_final_kernel(const float *__restrict__ partial, int64_t d_in, int nchunk,
                                                            float *__restrict__ D, int accumulate) {
    __shared__ double red[16][64];
    const int cx = threadIdx.x & 63, cy = threadIdx.x >> 6;
    const int64_t j = (int64_t)blockIdx.x * 64 + cx;
    double s = 0.0;
    if (j < d_in) {
        for (int c0 = cy; c0 < nchunk; c0 += 16 * 8) { // eight loads in flight
            float p[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) p[u] = c0 + 16 * u < nchunk ? partial[(int64_t)(c0 + 16 * u) * d_in + j] : 0.f;
#pragma unroll
            for (int u = 0; u < 8; ++u) s += (double)p[u];
        }
    }
    red[cy][cx] = s;
    __syncthreads();
    if (cy == 0 && j < d_in) {
        double t = accumulate ? (double)D[j] : 0.0;
#pragma unroll
        for (int y = 0; y < 16; ++y) t += red[y][cx];
        D[j] = (float)t;
    }
}

int diag_x_chunks(int64_t n) { return (int)std::max<int64_t>(1, std::min<int64_t>(512, (n + 63) / 64)); }

void launch_diag_x(const void *X, int bf16, int64_t n, int64_t d_in, int64_t ldx, float *D, int accumulate,
                   float *partial, hipStream_t s) {
    const int nchunk = diag_x_chunks(n), vec = bf16 ? 8 : 4;
    const int64_t rows_per_chunk = (n + nchunk - 1) / nchunk;
    dim3 grid((unsigned)((d_in / vec + 255) / 256), (unsigned)nchunk);
    if (bf16) hipLaunchKernelGGL(diag_x_partial_kernel<true>, grid, dim3(256), 0, s, X, n, d_in, ldx, rows_per_chunk, partial);
    else      hipLaunchKernelGGL(diag_x_partial_kernel<false>, grid, dim3(256), 0, s, X, n, d_in, ldx, rows_per_chunk, partial);
    hipLaunchKernelGGL(diag_x_final_kernel, dim3((unsigned)((d_in + 63) / 64)), dim3(1024), 0, s, partial, d_in, nchunk, D,
                       accumulate);
}

// ------------------------------------------------------------------------------------------------
// wrapper update (Alg. 2):  X^(k) <- X^(k) - grad^(k) / beta,  beta = 2 * sum of the per-block
// summands of Eq. 9 / Eq. 10, grad^(k) = sum of the nsplit partials the chain kernel left.
// A zero beta leaves X unchanged.  Workgroup (k, q) updates 256 entries of block k, one per thread; every workgroup re-derives beta in the same fixed order.  Workgroup (0,0) also writes the loss of the previous
// iterate (sum of the block losses) when trace_out is given, and the step size 1/beta (0 when beta = 0)
// when eta_out is given.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void update_wrapper_kernel(float *__restrict__ X, int b, const float *__restrict__ gpart,
                                                             int nsplit, const float *__restrict__ beta_part,
                                                             int nblocks, const float *__restrict__ loss_part,
                                                             double *__restrict__ trace_out,
                                                             double *__restrict__ eta_out) {
    __shared__ double red[4];
    const int tid = threadIdx.x, k = blockIdx.x, q = blockIdx.y;
    const int bb = b * b, e = q * 256 + tid;
    // the partial gradients of this element first (independent loads in flight together, summed in
    // chunk order)
    const bool live = e < bb;
    double g = 0.0;
    if (live) {
#pragma unroll 8
        for (int c = 0; c < nsplit; ++c) g += (double)gpart[((int64_t)k * nsplit + c) * bb + e];
    }
    const float xold = live ? X[(int64_t)k * bb + e] : 0.f;
    double s = 0.0;
    for (int i = tid; i < nblocks; i += 256) s += (double)beta_part[i];
    const double beta = 2.0 * block_sum_256(s, red);
    if (eta_out != nullptr && k == 0 && q == 0 && tid == 0) *eta_out = beta > 0.0 ? 1.0 / beta : 0.0;
    if (trace_out != nullptr && k == 0 && q == 0) {
        double l = 0.0;
        for (int i = tid; i < nblocks; i += 256) l += (double)loss_part[i];
        l = block_sum_256(l, red);
        if (tid == 0) *trace_out = l;
    }
    if (!(beta > 0.0) || !live) return;
    X[(int64_t)k * bb + e] = (float)((double)xold - g / beta);
}

// The same update at d_block = 128 for the chains that take the wrapper as bf16 pieces: workgroup (k, q) owns
// the 16-row strip q of block k (thread t: row t / 16, eight columns from 8 (t % 16)), writes the fp32 values
// and, through LDS, the strip's entries of both plane sets: P (op(x, k) = X[x][k]: rows of the strip, all eight
// runs) and PT (op(x, k) = X[k][x]: the strip's rows are run q of every column).  Same sums in the same order
// as update_wrapper_kernel.
__global__ __launch_bounds__(256) void update_wrapper_planes_kernel(float *__restrict__ X, const float *__restrict__ gpart,
                                                                    int nsplit, const float *__restrict__ beta_part,
                                                                    int nblocks, const float *__restrict__ loss_part,
                                                                    double *__restrict__ trace_out,
                                                                    double *__restrict__ eta_out,
                                                                    uint16_t *__restrict__ P, uint16_t *__restrict__ PT) {
    constexpr int b = PLANE_B, bb = b * b;
    __shared__ double red[4];
    __shared__ float T[16][b + 1];
    const int tid = threadIdx.x, k = blockIdx.x, q = blockIdx.y;
    const int row = tid >> 4, col = 8 * (tid & 15);
    const int e = (16 * q + row) * b + col;
    double g[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) g[u] = 0.0;
#pragma unroll 4
    for (int c = 0; c < nsplit; ++c) {
        const float4 *src = reinterpret_cast<const float4 *>(gpart + ((int64_t)k * nsplit + c) * bb + e);
        const float4 lo = src[0], hi = src[1];
        g[0] += (double)lo.x; g[1] += (double)lo.y; g[2] += (double)lo.z; g[3] += (double)lo.w;
        g[4] += (double)hi.x; g[5] += (double)hi.y; g[6] += (double)hi.z; g[7] += (double)hi.w;
    }
    float4 *xp = reinterpret_cast<float4 *>(X + (int64_t)k * bb + e);
    const float4 xlo = xp[0], xhi = xp[1];
    const float xold[8] = {xlo.x, xlo.y, xlo.z, xlo.w, xhi.x, xhi.y, xhi.z, xhi.w};
    double s = 0.0;
    for (int i = tid; i < nblocks; i += 256) s += (double)beta_part[i];
    const double beta = 2.0 * block_sum_256(s, red);
    if (eta_out != nullptr && k == 0 && q == 0 && tid == 0) *eta_out = beta > 0.0 ? 1.0 / beta : 0.0;
    if (trace_out != nullptr && k == 0 && q == 0) {
        double l = 0.0;
        for (int i = tid; i < nblocks; i += 256) l += (double)loss_part[i];
        l = block_sum_256(l, red);
        if (tid == 0) *trace_out = l;
    }
    if (!(beta > 0.0)) return; // X and its pieces stay as they are (uniform over the workgroup)
    float xn[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        xn[u] = (float)((double)xold[u] - g[u] / beta);
        T[row][col + u] = xn[u];
    }
    xp[0] = make_float4(xn[0], xn[1], xn[2], xn[3]);
    xp[1] = make_float4(xn[4], xn[5], xn[6], xn[7]);
    __syncthreads();
    float v[16];
    if (tid < b) { // P: 16 rows x 8 runs; thread -> (x = strip row t % 16, run t / 16)
        const int x = tid & 15, run = tid >> 4;
#pragma unroll
        for (int i = 0; i < 16; ++i) v[i] = T[x][16 * run + i];
        plane_emit(P + (int64_t)k * 3 * bb, run, 16 * q + x, v);
    } else if (PT != nullptr) { // PT: the strip is run q of all 128 columns; thread -> column t - 128
        const int x = tid - b;
#pragma unroll
        for (int i = 0; i < 16; ++i) v[i] = T[i][x];
        plane_emit(PT + (int64_t)k * 3 * bb, q, x, v);
    }
}

void launch_update_wrapper(float *A, int nblk, int b, const float *gpart, int nsplit, const float *beta_part,
                           int nblocks, const float *loss_part, double *trace_out, double *eta_out, uint16_t *P,
                           uint16_t *PT, hipStream_t s) {
    if (P != nullptr && b == PLANE_B) {
        hipLaunchKernelGGL(update_wrapper_planes_kernel, dim3(nblk, b / 16), dim3(256), 0, s, A, gpart, nsplit, beta_part,
                           nblocks, loss_part, trace_out, eta_out, P, PT);
        return;
    }
    int nq = (b * b + 255) / 256;
    hipLaunchKernelGGL(update_wrapper_kernel, dim3(nblk, nq), dim3(256), 0, s, A, b, gpart, nsplit, beta_part, nblocks,
                       loss_part, trace_out, eta_out);
}

// Adam update of a wrapper (joint-Adam variant, Sec. 3.3.1): g = sum of the partial gradients in a
// fixed order, then the published update with bias correction; moments are fp32 state.
// inv_c1 = 1/(1 - b1^t), inv_c2 = 1/(1 - b2^t).
__global__ __launch_bounds__(256) void adam_wrapper_kernel(float *__restrict__ X, float *__restrict__ m,
                                                           float *__restrict__ v, int b, const float *__restrict__ gpart,
                                                           int nsplit, double lr, double b1, double b2, double eps,
                                                           double inv_c1, double inv_c2, int nblocks,
                                                           const float *__restrict__ loss_part,
                                                           double *__restrict__ trace_out) {
    __shared__ double red[4];
    const int tid = threadIdx.x, k = blockIdx.x, q = blockIdx.y;
    const int bb = b * b, e = q * 256 + tid;
    if (trace_out != nullptr && k == 0 && q == 0) {
        double l = 0.0;
        for (int i = tid; i < nblocks; i += 256) l += (double)loss_part[i];
        l = block_sum_256(l, red);
        if (tid == 0) *trace_out = l;
    }
    if (e >= bb) return;
    double g = 0.0;
#pragma unroll 8
    for (int c = 0; c < nsplit; ++c) g += (double)gpart[((int64_t)k * nsplit + c) * bb + e];
    const int64_t idx = (int64_t)k * bb + e;
    const double mn = b1 * (double)m[idx] + (1.0 - b1) * g;
    const double vn = b2 * (double)v[idx] + (1.0 - b2) * g * g;
    m[idx] = (float)mn;
    v[idx] = (float)vn;
    X[idx] = (float)((double)X[idx] - lr * (mn * inv_c1) / (sqrt(vn * inv_c2) + eps));
}

void launch_adam_wrapper(float *X, float *m, float *v, int nblk, int b, const float *gpart, int nsplit, double lr,
                         double b1, double b2, double eps, int64_t t, int nblocks, const float *loss_part,
                         double *trace_out, hipStream_t s) {
    const double inv_c1 = 1.0 / (1.0 - pow(b1, (double)t)), inv_c2 = 1.0 / (1.0 - pow(b2, (double)t));
    hipLaunchKernelGGL(adam_wrapper_kernel, dim3(nblk, (b * b + 255) / 256), dim3(256), 0, s, X, m, v, b, gpart, nsplit,
                       lr, b1, b2, eps, inv_c1, inv_c2, nblocks, loss_part, trace_out);
}

// Input validation (optional): counts NaN/Inf entries of W and NaN/Inf/negative loss weights D_j = ||X_j||^2
// (Eq. 2).  flag must be zero on entry; integer atomics only.
template <bool BF16>
__global__ __launch_bounds__(256) void count_nonfinite_kernel(const void *__restrict__ W, int64_t n,
                                                              const float *__restrict__ D, int64_t d_in,
                                                              int32_t *__restrict__ flag) {
    int bad = 0;
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < n; e += stride) {
        const float w = load_w<BF16>(W, e);
        bad += !(fabsf(w) <= 3.402823466e38f);
    }
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < d_in; e += stride) {
        const float dj = D[e];
        bad += !(dj >= 0.f && dj <= 3.402823466e38f);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) bad += __shfl_xor(bad, off, 64);
    if ((threadIdx.x & 63) == 0 && bad != 0) atomicAdd(flag, bad);
}

void launch_count_nonfinite(const void *W, int bf16, int64_t n, const float *D, int64_t d_in, int32_t *flag,
                            hipStream_t s) {
    const int grid = (int)std::max<int64_t>(1, std::min<int64_t>((n + 255) / 256, 4096));
    if (bf16) hipLaunchKernelGGL(count_nonfinite_kernel<true>, dim3(grid), dim3(256), 0, s, W, n, D, d_in, flag);
    else hipLaunchKernelGGL(count_nonfinite_kernel<false>, dim3(grid), dim3(256), 0, s, W, n, D, d_in, flag);
}

__global__ __launch_bounds__(256) void zero_kernel(float *__restrict__ x, int64_t n) {
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < n; e += (int64_t)gridDim.x * 256) x[e] = 0.f;
}

__global__ __launch_bounds__(256) void fill_kernel(float *__restrict__ x, int64_t n, float v) {
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < n; e += (int64_t)gridDim.x * 256) x[e] = v;
}

void launch_fill(float *x, int64_t n, float v, hipStream_t s) {
    int grid = (int)std::min<int64_t>((n + 255) / 256, 65536);
    if (grid > 0) hipLaunchKernelGGL(fill_kernel, dim3(grid), dim3(256), 0, s, x, n, v);
}

void launch_zero(float *x, int64_t n, hipStream_t s) {
    int grid = (int)std::min<int64_t>((n + 255) / 256, 65536);
    if (n > 0) hipLaunchKernelGGL(zero_kernel, dim3(grid), dim3(256), 0, s, x, n);
}

__global__ __launch_bounds__(256) void sum_to_double_kernel(const float *__restrict__ part, int n,
                                                            double *__restrict__ out) {
    __shared__ double red[4];
    double a = 0.0;
    for (int e = threadIdx.x; e < n; e += 256) a += (double)part[e];
    a = block_sum_256(a, red);
    if (threadIdx.x == 0) *out = a;
}

// dst[0 .. n) = *src (src may be one of them)
__global__ __launch_bounds__(256) void broadcast_double_kernel(double *__restrict__ dst, int64_t n, const double *src) {
    const double v = *src;
    __syncthreads();
    for (int64_t e = threadIdx.x; e < n; e += 256) dst[e] = v;
}

void launch_broadcast_double(double *dst, int64_t n, const double *src, hipStream_t s) {
    if (n > 0) hipLaunchKernelGGL(broadcast_double_kernel, dim3(1), dim3(256), 0, s, dst, n, src);
}

void launch_sum_to_double(const float *part, int n, double *out, hipStream_t s) {
    hipLaunchKernelGGL(sum_to_double_kernel, dim3(1), dim3(256), 0, s, part, n, out);
}

// ------------------------------------------------------------------------------------------------
// sparse-core step (Alg. 3).  One workgroup per block (i,j).
//  1. Scores: g_kappa = L1 (or L2) norm of the M entries of group kappa = i'*(b/M)+k of the
//     unmasked core gradient (Sec. 3.3.2); draw one group by an exponential race on a counter
//     hash: key = -ln(u)/g, smallest key wins, ties to the lower kappa.
//  2. For every N-subset s of the group (lexicographic order), Eq. 7:
//        gain_s = q_s^T (K_ss)^+ q_s / ||a||^2,   w_s = (K_ss)^+ q_s / ||a||^2   (Eq. 8)
//     with K = B^j D^j B^jT (so K_ss = B' D B'^T), a = column i' of A^i, and
//        q_p = B_p D DeltaW^T a = (A^T (R D) B^T)[i', p] + ||a||^2 sum_p' K[p,p'] c_p'
//     because DeltaW = R + a (c^T B_group) (Eq. 6); the first term is -Gfull/2, already in HBM.
//  3. Largest gain wins (first in order on ties); write weights and mask byte.
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ uint64_t mix64(uint64_t z) {
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ULL;
    z ^= z >> 27; z *= 0x94D049BB133111EBULL;
    z ^= z >> 31;
    return z;
}

__device__ __forceinline__ float hash_uniform(uint64_t seed, uint64_t ctr) {
    uint64_t z = mix64(seed + 0x9E3779B97F4A7C15ULL * ctr);
    return (float)((z >> 40) + 1ULL) * (1.0f / 16777216.0f);
}

// -ln(u) for u = m * 2^-24, m = (z >> 40) + 1, to about 2 ulp without the library logarithm.  The race
// is decided by u near 1, where -ln(u) is small: there x = 1 - u is exact in fp32 and the series of
// -ln(1 - x) is used (x < 1/16, 7 terms, truncation below 1e-9 relative); elsewhere the hardware log2
// is accurate relative to a result that is at least 0.06.
__device__ __forceinline__ float neg_log_uniform(uint64_t z) {
    const uint32_t m = (uint32_t)(z >> 40) + 1u;
    const float u = (float)m * (1.0f / 16777216.0f);
    const float x = (float)(16777216u - m) * (1.0f / 16777216.0f);
    float poly = fmaf(x, 1.0f / 7.0f, 1.0f / 6.0f);
    poly = fmaf(x, poly, 0.2f);
    poly = fmaf(x, poly, 0.25f);
    poly = fmaf(x, poly, 1.0f / 3.0f);
    poly = fmaf(x, poly, 0.5f);
    poly = fmaf(x, poly, 1.0f);
    poly *= x;
    const float big = -0.69314718056f * __log2f(u);
    return x < 0.0625f ? poly : big;
}

// w = G^+ q for a symmetric PSD N x N matrix (Moore-Penrose: eigenvalues <= 1e-12 * the largest are
// treated as zero), returns q^T G^+ q.  Everything is unrolled so that it stays in registers.
//   N = 2: eigenvalues from trace and determinant.  lambda_max = h + r with h = (a+d)/2, r = |((a-d)/2, b)|,
//          lambda_min = det / lambda_max (no cancellation).  Both kept: G^+ = adj(G)/det.  Only the larger
//          kept: G is lambda_max v v^T up to the dropped part, so G^+ = G / lambda_max^2.
//   N >= 3: L D L^T when G is provably far from the drop threshold, otherwise a one-sided Jacobi
//          orthogonalisation (Hestenes): plane rotations V make the columns of U = G V mutually orthogonal;
//          then G = U V^T, the column norms sigma_k are the eigenvalues of the PSD matrix, and
//          G^+ q = sum_k v_k (u_k . q) / sigma_k^2 over the kept k.
template <int N> __device__ double pinv_solve(double (&G)[N][N], const double (&q)[N], double (&w)[N]) {
    if (N == 1) {
        w[0] = G[0][0] > 0.0 ? q[0] / G[0][0] : 0.0;
        return w[0] * q[0];
    }
    if (N == 2) {
        const double a = G[0][0], b = G[0][N - 1], d = G[N - 1][N - 1];
        const double h = 0.5 * (a + d), e = 0.5 * (a - d);
        const double lmax = h + sqrt(e * e + b * b);
        w[0] = 0.0;
        w[N - 1] = 0.0;
        if (!(lmax > 0.0)) return 0.0;
        const double det = a * d - b * b, lmin = det / lmax;
        if (lmin > 1e-12 * lmax) {
            const double inv = 1.0 / det;
            w[0] = (d * q[0] - b * q[N - 1]) * inv;
            w[N - 1] = (a * q[N - 1] - b * q[0]) * inv;
        } else {
            const double inv = 1.0 / (lmax * lmax);
            w[0] = (a * q[0] + b * q[N - 1]) * inv;
            w[N - 1] = (b * q[0] + d * q[N - 1]) * inv;
        }
        return q[0] * w[0] + q[N - 1] * w[N - 1];
    }
    {
        // Fast path.  With pivots d_k of G = L D L^T and rho_k = d_k / G_kk (the pivots of the unit-
        // diagonal scaling G' of G):  lambda_min(G) >= lambda_min(G') min_k G_kk,  lambda_min(G') >=
        // det G' / lambda_max(G')^(N-1) >= prod rho_k / N^(N-1),  lambda_max(G) <= trace G.  If that
        // lower bound on lambda_min / lambda_max clears the drop threshold with a factor 10 to spare,
        // no eigenvalue is dropped, G^+ = G^-1, and the triangular solves give the same w (to
        // rounding) without the eigen-decomposition.
        double L[N][N], d[N], dmin = G[0][0], tr = 0.0, rho = 1.0, nn = 1.0;
        bool ok = true;
#pragma unroll
        for (int k = 0; k < N; ++k) {
            dmin = fmin(dmin, G[k][k]);
            tr += G[k][k];
            if (k > 0) nn *= (double)N;
        }
#pragma unroll
        for (int k = 0; k < N; ++k) {
            double dk = G[k][k];
#pragma unroll
            for (int m = 0; m < k; ++m) dk -= L[k][m] * L[k][m] * d[m];
            d[k] = dk;
            ok = ok && dk > 0.0 && G[k][k] > 0.0;
            const double inv = ok ? 1.0 / dk : 0.0;
            rho *= ok ? dk / G[k][k] : 0.0;
#pragma unroll
            for (int r = k + 1; r < N; ++r) {
                double v = G[r][k];
#pragma unroll
                for (int m = 0; m < k; ++m) v -= L[r][m] * L[k][m] * d[m];
                L[r][k] = v * inv;
            }
        }
        if (ok && rho * dmin >= 1e-11 * nn * tr) {
            double y[N];
#pragma unroll
            for (int k = 0; k < N; ++k) { // L y = q
                double v = q[k];
#pragma unroll
                for (int m = 0; m < k; ++m) v -= L[k][m] * y[m];
                y[k] = v;
            }
#pragma unroll
            for (int k = N - 1; k >= 0; --k) { // L^T w = D^-1 y
                double v = y[k] / d[k];
#pragma unroll
                for (int m = k + 1; m < N; ++m) v -= L[m][k] * w[m];
                w[k] = v;
            }
            double gain = 0.0;
#pragma unroll
            for (int k = 0; k < N; ++k) gain += q[k] * w[k];
            return gain;
        }
    }
    // One-sided Jacobi.  U starts as G (its columns), V as the identity; a rotation of columns (i, j) by the
    // angle that zeroes their inner product is applied to both, so U = G V throughout.
    double V[N][N];
#pragma unroll
    for (int i = 0; i < N; ++i)
#pragma unroll
        for (int j = 0; j < N; ++j) V[i][j] = i == j ? 1.0 : 0.0;
    for (int pass = 0; pass < 40; ++pass) {
        bool turned = false;
#pragma unroll
        for (int i = 0; i < N - 1; ++i)
#pragma unroll
            for (int j = i + 1; j < N; ++j) {
                double nii = 0.0, njj = 0.0, nij = 0.0;
#pragma unroll
                for (int k = 0; k < N; ++k) {
                    nii += G[k][i] * G[k][i];
                    njj += G[k][j] * G[k][j];
                    nij += G[k][i] * G[k][j];
                }
                if (nij * nij > 1e-30 * nii * njj) { // columns not yet orthogonal to working precision
                    const double zeta = (njj - nii) / (2.0 * nij);
                    const double tn = copysign(1.0, zeta) / (fabs(zeta) + sqrt(1.0 + zeta * zeta));
                    const double cs = 1.0 / sqrt(1.0 + tn * tn), sn = cs * tn;
#pragma unroll
                    for (int k = 0; k < N; ++k) {
                        const double ui = G[k][i], uj = G[k][j], vi = V[k][i], vj = V[k][j];
                        G[k][i] = cs * ui - sn * uj;
                        G[k][j] = sn * ui + cs * uj;
                        V[k][i] = cs * vi - sn * vj;
                        V[k][j] = sn * vi + cs * vj;
                    }
                    turned = true;
                }
            }
        if (!turned) break;
    }
    double sig2[N], smax2 = 0.0;
#pragma unroll
    for (int j = 0; j < N; ++j) {
        double n2 = 0.0;
#pragma unroll
        for (int k = 0; k < N; ++k) n2 += G[k][j] * G[k][j];
        sig2[j] = n2;
        smax2 = fmax(smax2, n2);
    }
#pragma unroll
    for (int i = 0; i < N; ++i) w[i] = 0.0;
    if (!(smax2 > 0.0)) return 0.0;
    double gain = 0.0;
#pragma unroll
    for (int j = 0; j < N; ++j)
        if (sig2[j] > 1e-24 * smax2) { // sigma_j > 1e-12 sigma_max
            double uq = 0.0, vq = 0.0;
#pragma unroll
            for (int k = 0; k < N; ++k) {
                uq += G[k][j] * q[k];
                vq += V[k][j] * q[k];
            }
            const double coef = uq / sig2[j];
#pragma unroll
            for (int i = 0; i < N; ++i) w[i] += V[i][j] * coef;
            gain += vq * coef;
        }
    return gain;
}

constexpr int binom(int n, int k) { return (k == 0 || k == n) ? 1 : binom(n - 1, k - 1) + binom(n - 1, k); }
// n, k <= 7 at run time: C(n, k) by the product formula (exact in integers at every step)
__device__ __forceinline__ int binom_rt(int n, int k) {
    if (k < 0 || k > n) return 0;
    int c = 1;
    for (int t = 1; t <= k; ++t) c = c * (n - k + t) / t;
    return c;
}

// SEL = the selection heuristic (a template argument: the pass over the groups then has no branches)
template <int N, int M, int SEL>
__global__ __launch_bounds__(256) void sparse_step_kernel(const float *__restrict__ G, float *__restrict__ C,
                                                          uint8_t *__restrict__ mask, const float *__restrict__ K,
                                                          const float *__restrict__ colnorm2, int64_t d_in, int b,
                                                          int nbj, int nblocks, uint64_t seed,
                                                          int64_t t, const float *__restrict__ loss_part,
                                                          double *__restrict__ loss_cont_out,
                                                          int32_t *__restrict__ changes_out) {
    constexpr int NPAT = binom(M, N);
    __shared__ float s_key[4];
    __shared__ int s_kap[4];
    __shared__ float s_gain[NPAT];
    __shared__ double s_q[M], s_K[M][M], s_red[4];
    __shared__ int s_best;
    const int tid = threadIdx.x, blk = blockIdx.x, i = blk / nbj, j = blk % nbj;
    // groups per block row: b and M are powers of two, so rows and columns of a group index come from
    // a shift and a mask (an integer division per group was a quarter of the selection pass)
    const int gpr = b / M, gpb = b * gpr, gsh = 31 - __clz(gpr);

    if (blk == 0 && loss_cont_out != nullptr) { // loss after the continuous step = sum of block losses
        double l = 0.0;
        for (int e = tid; e < nblocks; e += 256) l += (double)loss_part[e];
        l = block_sum_256(l, s_red);
        if (tid == 0) *loss_cont_out = l;
    }

    // ---- 1. selection ----
    float best_key = INFINITY;
    int best_kap = 0x7fffffff;
    const float *Gij = G + (int64_t)i * b * d_in + (int64_t)j * b;
    constexpr int U = 4; // groups per thread whose loads are in flight together (more in flight measured slower)
    // counter hash input of this thread's first group; consecutive groups of a thread are 256 apart,
    // so the 64-bit product by the odd constant is replaced by a running sum
    constexpr uint64_t PHI = 0x9E3779B97F4A7C15ULL;
    uint64_t zin = seed + PHI * ((uint64_t)(((int64_t)t * nblocks + blk) * gpb + tid) + 1ULL);
    for (int kap0 = tid; kap0 < gpb; kap0 += 256 * U) {
        float v[U][M];
#pragma unroll
        for (int u = 0; u < U; ++u) { // unconditional loads (index clamped): a group past the end is dropped below
            const int kap = min(kap0 + u * 256, gpb - 1);
            const float *g = Gij + (int64_t)(kap >> gsh) * d_in + (kap & (gpr - 1)) * M;
            if constexpr (M % 4 == 0) { // 16-byte loads (a group starts at a multiple of M columns)
#pragma unroll
                for (int h = 0; h < M / 4; ++h) {
                    const float4 x = reinterpret_cast<const float4 *>(g)[h];
                    v[u][4 * h] = x.x; v[u][4 * h + 1] = x.y; v[u][4 * h + 2] = x.z; v[u][4 * h + 3] = x.w;
                }
            } else {
                const float2 x = *reinterpret_cast<const float2 *>(g);
                v[u][0] = x.x; v[u][1] = x.y;
                static_assert(M % 4 == 0 || M == 2, "group sizes are 2, 4 or 8");
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int kap = kap0 + u * 256;
            const uint64_t z = mix64(zin);
            zin += PHI * 256ULL;
            float score = 0.f;
            if (SEL == 2) {
#pragma unroll
                for (int p = 0; p < M; ++p) score = fmaf(v[u][p], v[u][p], score);
                score = sqrtf(score);
            } else if (SEL == 3) {
                score = 1.f;
            } else {
#pragma unroll
                for (int p = 0; p < M; ++p) score += fabsf(v[u][p]);
            }
            float key;
            if (SEL == 1) key = -score;
            else key = score > 0.f ? __fdividef(neg_log_uniform(z), score) : INFINITY;
            if (kap >= gpb) key = INFINITY; // (a NaN key never wins either: the comparison below is false)
            if (key < best_key) { best_key = key; best_kap = kap; }
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        float ok = __shfl_xor(best_key, off, 64);
        int oa = __shfl_xor(best_kap, off, 64);
        if (ok < best_key || (ok == best_key && oa < best_kap)) { best_key = ok; best_kap = oa; }
    }
    if ((tid & 63) == 0) { s_key[tid >> 6] = best_key; s_kap[tid >> 6] = best_kap; }
    __syncthreads();
    best_key = s_key[0]; best_kap = s_kap[0];
#pragma unroll
    for (int w = 1; w < 4; ++w)
        if (s_key[w] < best_key || (s_key[w] == best_key && s_kap[w] < best_kap)) { best_key = s_key[w]; best_kap = s_kap[w]; }
    if (best_kap == 0x7fffffff) best_kap = 0; // every key was +inf (or NaN): the first group
    const int ip = best_kap >> gsh, k0 = (best_kap & (gpr - 1)) * M;

    // ---- 2. operands of Eq. 7 for the drawn group: one round of independent loads ----
    float *crow = C + ((int64_t)i * b + ip) * d_in + (int64_t)j * b + k0;
    const float *Kj = K + (int64_t)j * b * b;
    __shared__ double s_c[M], s_g[M], s_a2;
    if (tid < M * M) s_K[tid / M][tid % M] = (double)Kj[(k0 + tid / M) * b + k0 + tid % M];
    if (tid >= 64 && tid < 64 + M) {
        s_c[tid - 64] = (double)crow[tid - 64];
        s_g[tid - 64] = (double)Gij[(int64_t)ip * d_in + k0 + tid - 64];
    }
    if (tid == 128) s_a2 = (double)colnorm2[(int64_t)i * b + ip];
    __syncthreads();
    const double a2 = s_a2;
    if (!(a2 > 0.0)) return; // a = 0: the block cannot move (uniform across the workgroup)
    if (tid < M) {
        double acc = 0.0;
#pragma unroll
        for (int pp = 0; pp < M; ++pp) acc += s_K[tid][pp] * s_c[pp];
        s_q[tid] = -0.5 * s_g[tid] + a2 * acc;
    }
    __syncthreads();

    // ---- 3. sweep: thread x handles the x-th subset in lexicographic order ----
    // (the sweep threads sit in wave blk % 4, so that co-resident workgroups do not all queue their
    // fp64 work on the same SIMD)
    int sub[N];
    double w[N];
    static_assert(NPAT <= 128, "the sweep threads must fit in the workgroup from any wave offset");
    const int sw = (tid - 64 * (blk & 3)) & 255; // sweep-thread index
    if (sw < NPAT) {
        // the sw-th N-subset of {0..M-1} in lexicographic order, by the combinatorial number system: at
        // position x take the smallest admissible element e for which the subsets that start with it,
        // C(M-1-e, N-1-x) of them, cover the remaining rank
        int rank = sw, e = 0;
#pragma unroll
        for (int x = 0; x < N; ++x) {
            for (;; ++e) {
                const int below = binom_rt(M - 1 - e, N - 1 - x);
                if (rank < below) break;
                rank -= below;
            }
            sub[x] = e++;
        }
        double Gs[N][N], qs[N];
#pragma unroll
        for (int x = 0; x < N; ++x) {
            qs[x] = s_q[sub[x]];
#pragma unroll
            for (int y = 0; y < N; ++y) Gs[x][y] = s_K[sub[x]][sub[y]];
        }
        double gain = pinv_solve<N>(Gs, qs, w) / a2;
        s_gain[sw] = (float)gain;
    }
    __syncthreads();
    if (tid == 0) {
        int bi = 0;
        float bg = s_gain[0];
        for (int x = 1; x < NPAT; ++x)
            if (s_gain[x] > bg) { bg = s_gain[x]; bi = x; }
        s_best = bi;
    }
    __syncthreads();
    if (sw == s_best) {
        float out[M];
        uint32_t bits = 0;
#pragma unroll
        for (int p = 0; p < M; ++p) out[p] = 0.f;
#pragma unroll
        for (int x = 0; x < N; ++x) {
            out[sub[x]] = (float)(w[x] / a2);
            bits |= 1u << sub[x];
        }
#pragma unroll
        for (int p = 0; p < M; ++p) crow[p] = out[p];
        uint8_t *mbyte = mask + ((int64_t)i * b + ip) * (d_in / M) + ((int64_t)j * b + k0) / M;
        // groups whose kept set moved in this iteration (an integer count: the order of the adds does not matter)
        if (changes_out != nullptr && *mbyte != (uint8_t)bits) atomicAdd(changes_out, 1);
        *mbyte = (uint8_t)bits;
    }
}

void launch_sparse_step(const Dims &d, const float *G, float *C, uint8_t *mask, const float *K,
                        const float *colnorm2, int N, int M, int selection, uint64_t seed, int64_t t,
                        const float *loss_part, double *loss_cont_out, int32_t *changes_out, hipStream_t s) {
#define ARMOR_SPARSE_LAUNCH(n, m, sel)                                                                        \
    hipLaunchKernelGGL((sparse_step_kernel<n, m, sel>), dim3(d.nblocks), dim3(256), 0, s, G, C, mask, K, colnorm2,  \
                       d.d_in, d.b, d.nbj, d.nblocks, seed, t, loss_part, loss_cont_out, changes_out)
#define ARMOR_SPARSE_CASE(n, m)                                                                               \
    if (N == n && M == m) {                                                                                   \
        switch (selection) {                                                                                  \
        case 1: ARMOR_SPARSE_LAUNCH(n, m, 1); break;                                                          \
        case 2: ARMOR_SPARSE_LAUNCH(n, m, 2); break;                                                          \
        case 3: ARMOR_SPARSE_LAUNCH(n, m, 3); break;                                                          \
        default: ARMOR_SPARSE_LAUNCH(n, m, 0); break;                                                         \
        }                                                                                                     \
        return;                                                                                               \
    }
    ARMOR_SPARSE_CASE(1, 2)
    ARMOR_SPARSE_CASE(1, 4) ARMOR_SPARSE_CASE(2, 4) ARMOR_SPARSE_CASE(3, 4)
    ARMOR_SPARSE_CASE(1, 8) ARMOR_SPARSE_CASE(2, 8) ARMOR_SPARSE_CASE(3, 8) ARMOR_SPARSE_CASE(4, 8)
    ARMOR_SPARSE_CASE(5, 8) ARMOR_SPARSE_CASE(6, 8) ARMOR_SPARSE_CASE(7, 8)
#undef ARMOR_SPARSE_CASE
#undef ARMOR_SPARSE_LAUNCH
}

// ------------------------------------------------------------------------------------------------
// unstructured initial mask (Sec. 4.5; the count-budget optimum of Eq. 2 for the plain core):
// keep the `keep` largest importances (w*w)*D_j of the whole matrix, equal importances going to
// the lower linear index.  Exact selection without sorting: the fp32 bit pattern of a
// non-negative score orders like an unsigned integer, so three histogram passes (11 + 11 + 10
// bits, integer atomics only) find the bit-exact threshold T and the number r of entries equal
// to T to admit; an ordered prefix count over the ties admits the r first ones.
// state[0] = prefix value, state[1] = remaining k, state[2] = r (ties to admit), state[3] = T.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void us_score_kernel(const float *__restrict__ Wbar, const float *__restrict__ D,
                                                       int64_t P, int64_t d_in, uint32_t *__restrict__ score) {
    int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= P) return;
    float w = Wbar[e];
    score[e] = __float_as_uint(__fmul_rn(__fmul_rn(w, w), D[e % d_in]));
}

__global__ __launch_bounds__(256) void us_zero_kernel(uint32_t *__restrict__ hist, int n, uint32_t *__restrict__ state,
                                                      int64_t keep) {
    int e = blockIdx.x * 256 + threadIdx.x;
    if (e < n) hist[e] = 0u;
    if (e == 0) { state[0] = 0u; state[1] = 0u; state[2] = 0u; state[3] = 0u;
                  reinterpret_cast<unsigned long long *>(state + 4)[0] = (unsigned long long)keep; }
}

// histogram of bits [shift, shift+nbits) over the entries whose higher bits equal the prefix
__global__ __launch_bounds__(256) void us_hist_kernel(const uint32_t *__restrict__ score, int64_t P, int shift,
                                                      int nbits, const uint32_t *__restrict__ state,
                                                      uint32_t *__restrict__ hist) {
    __shared__ uint32_t lh[2048];
    for (int e = threadIdx.x; e < 2048; e += 256) lh[e] = 0u;
    __syncthreads();
    const uint32_t prefix = state[0];
    const int hi = shift + nbits;
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < P; e += (int64_t)gridDim.x * 256) {
        uint32_t v = score[e];
        bool match = hi >= 32 ? true : ((v >> hi) == (prefix >> hi));
        if (match) atomicAdd(&lh[(v >> shift) & ((1u << nbits) - 1u)], 1u);
    }
    __syncthreads();
    for (int e = threadIdx.x; e < (1 << nbits); e += 256)
        if (lh[e]) atomicAdd(&hist[e], lh[e]);
}

// walk the bins from the top until the remaining budget is met; fix those bits of the threshold
__global__ void us_select_kernel(uint32_t *__restrict__ hist, int shift, int nbits, uint32_t *__restrict__ state,
                                 int last) {
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    unsigned long long k = reinterpret_cast<unsigned long long *>(state + 4)[0];
    uint32_t prefix = state[0];
    int bin = (1 << nbits) - 1;
    for (; bin > 0; --bin) {
        if ((unsigned long long)hist[bin] >= k) break;
        k -= hist[bin];
    }
    prefix |= (uint32_t)bin << shift;
    state[0] = prefix;
    reinterpret_cast<unsigned long long *>(state + 4)[0] = k; // budget left inside this bin
    if (last) {
        state[3] = prefix;                                       // T
        unsigned long long ties = hist[bin];
        state[2] = (uint32_t)(k < ties ? k : ties);              // r: ties to admit (k <= ties unless keep > P)
    }
    for (int e = 0; e < (1 << nbits); ++e) hist[e] = 0u;
}

// one byte of mask (8 consecutive entries) per thread; chunk = 2048 entries per workgroup
__global__ __launch_bounds__(256) void us_tie_count_kernel(const uint32_t *__restrict__ score, int64_t P,
                                                           const uint32_t *__restrict__ state,
                                                           uint32_t *__restrict__ tie_count) {
    __shared__ uint32_t cnt;
    if (threadIdx.x == 0) cnt = 0u;
    __syncthreads();
    const uint32_t T = state[3];
    int64_t e0 = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 8;
    uint32_t c = 0;
    for (int q = 0; q < 8; ++q)
        if (e0 + q < P && score[e0 + q] == T) ++c;
    if (c) atomicAdd(&cnt, c);
    __syncthreads();
    if (threadIdx.x == 0) tie_count[blockIdx.x] = cnt;
}

__global__ __launch_bounds__(256) void us_tie_scan_kernel(const uint32_t *__restrict__ tie_count, int64_t nchunks,
                                                          unsigned long long *__restrict__ tie_offset) {
    // exclusive prefix sum by one workgroup: each thread owns a contiguous slice
    __shared__ unsigned long long part[256];
    const int64_t per = (nchunks + 255) / 256, a = threadIdx.x * per, b = min(nchunks, a + per);
    unsigned long long s = 0;
    for (int64_t e = a; e < b; ++e) s += tie_count[e];
    part[threadIdx.x] = s;
    __syncthreads();
    unsigned long long base = 0;
    for (int t = 0; t < (int)threadIdx.x; ++t) base += part[t];
    for (int64_t e = a; e < b; ++e) { tie_offset[e] = base; base += tie_count[e]; }
}

__global__ __launch_bounds__(256) void us_apply_kernel(const float *__restrict__ Wbar, const uint32_t *__restrict__ score,
                                                       int64_t P, const uint32_t *__restrict__ state,
                                                       const unsigned long long *__restrict__ tie_offset,
                                                       float *__restrict__ C, uint8_t *__restrict__ mask) {
    __shared__ uint32_t wsum[4];
    const uint32_t T = state[3], r = state[2];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int64_t e0 = ((int64_t)blockIdx.x * 256 + tid) * 8;
    uint32_t sc[8], c = 0;
#pragma unroll
    for (int q = 0; q < 8; ++q) {
        sc[q] = e0 + q < P ? score[e0 + q] : 0xffffffffu;
        c += (e0 + q < P && sc[q] == T) ? 1u : 0u;
    }
    // ordered exclusive prefix of the tie counts inside the workgroup
    uint32_t incl = c;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        uint32_t o = __shfl_up(incl, off, 64);
        if (lane >= off) incl += o;
    }
    if (lane == 63) wsum[w] = incl;
    __syncthreads();
    unsigned long long rank = tie_offset[blockIdx.x] + (incl - c);
    for (int t = 0; t < w; ++t) rank += wsum[t];
    if (e0 >= P) return;
    uint32_t bits = 0;
#pragma unroll
    for (int q = 0; q < 8; ++q) {
        if (e0 + q >= P) break;
        bool keep = sc[q] > T;
        if (sc[q] == T) { keep = rank < (unsigned long long)r; ++rank; }
        bits |= keep ? (1u << q) : 0u;
        C[e0 + q] = keep ? Wbar[e0 + q] : 0.f;
    }
    mask[e0 / 8] = (uint8_t)bits;
}

size_t unstructured_init_ws_bytes(int64_t d_out, int64_t d_in) {
    int64_t P = d_out * d_in, nchunks = (P + 2047) / 2048;
    return (size_t)(2048 + 16) * 4 + (size_t)nchunks * (4 + 8) + 1024;
}

// score_buf: P uint32 of scratch (the caller lends the core-gradient buffer); ws: unstructured_init_ws_bytes
void launch_unstructured_init(const float *Wbar, const float *D, int64_t d_out, int64_t d_in, int64_t keep,
                              float *C, uint8_t *mask, uint32_t *score_buf, void *ws, hipStream_t s) {
    const int64_t P = d_out * d_in, nchunks = (P + 2047) / 2048;
    char *base = reinterpret_cast<char *>(ws);
    uint32_t *hist = reinterpret_cast<uint32_t *>(base);
    uint32_t *state = hist + 2048; // 8 words: [0] prefix [2] r [3] T [4..5] 64-bit budget
    size_t off = ((size_t)(2048 + 16) * 4 + 255) & ~size_t(255);
    unsigned long long *tie_offset = reinterpret_cast<unsigned long long *>(base + off);
    uint32_t *tie_count = reinterpret_cast<uint32_t *>(base + off + (size_t)nchunks * 8);
    hipLaunchKernelGGL(us_zero_kernel, dim3(8), dim3(256), 0, s, hist, 2048, state, keep);
    hipLaunchKernelGGL(us_score_kernel, dim3((unsigned)((P + 255) / 256)), dim3(256), 0, s, Wbar, D, P, d_in, score_buf);
    const int grid = (int)std::min<int64_t>((P + 255) / 256, 4096);
    const int shifts[3] = {21, 10, 0}, nbits[3] = {11, 11, 10};
    for (int pass = 0; pass < 3; ++pass) {
        hipLaunchKernelGGL(us_hist_kernel, dim3(grid), dim3(256), 0, s, score_buf, P, shifts[pass], nbits[pass], state, hist);
        hipLaunchKernelGGL(us_select_kernel, dim3(1), dim3(64), 0, s, hist, shifts[pass], nbits[pass], state, pass == 2);
    }
    hipLaunchKernelGGL(us_tie_count_kernel, dim3((unsigned)nchunks), dim3(256), 0, s, score_buf, P, state, tie_count);
    hipLaunchKernelGGL(us_tie_scan_kernel, dim3(1), dim3(256), 0, s, tie_count, nchunks, tie_offset);
    hipLaunchKernelGGL(us_apply_kernel, dim3((unsigned)nchunks), dim3(256), 0, s, Wbar, score_buf, P, state, tie_offset, C,
                       mask);
}

// ------------------------------------------------------------------------------------------------
// epilogue: denormalisation (Sec. 3.2) and compressed N:M storage
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void denormalize_kernel(float *__restrict__ A, float *__restrict__ B,
                                                          const float *__restrict__ r1, const float *__restrict__ r2,
                                                          int64_t na, int64_t nb, int b) {
    int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e < na) {
        int64_t blk = e / ((int64_t)b * b), p = (e / b) % b;
        A[e] = (float)((double)A[e] * (double)r2[blk * b + p]);
    } else if (e < na + nb) {
        int64_t f = e - na, blk = f / ((int64_t)b * b), q = f % b;
        B[f] = (float)((double)B[f] * (double)r1[blk * b + q]);
    }
}

void launch_denormalize(float *A, float *B, const float *r1, const float *r2, int64_t d_out, int64_t d_in, int b,
                        hipStream_t s) {
    int64_t na = d_out * b, nb = d_in * b;
    hipLaunchKernelGGL(denormalize_kernel, dim3((unsigned)((na + nb + 255) / 256)), dim3(256), 0, s, A, B, r1, r2, na,
                       nb, b);
}

__device__ __forceinline__ uint16_t float_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40); // NaN stays NaN
    return (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}

// Compressed N:M storage.  A thread packs G consecutive groups of one row, G chosen so that its index
// fields fill whole bytes: the kept values in increasing column order, and per kept entry its column
// inside the group in a field of W_BITS bits (1, 2 or 4 for M = 2, 4, 8), fields filling each byte
// from bit 0 upwards; a row of meta starts on a byte boundary.
template <int N, int M> struct PackGeom {
    static constexpr int W_BITS = M == 2 ? 1 : (M == 4 ? 2 : 4);
    static constexpr int NW = N * W_BITS; // index bits per group
    static constexpr int G = (NW % 8 == 0) ? 1 : (NW % 4 == 0) ? 2 : (NW % 2 == 0) ? 4 : 8;
    static constexpr int BYTES = G * NW / 8; // meta bytes per thread
};

template <int N, int M, bool BF16>
__global__ __launch_bounds__(256) void pack_nm_kernel(const float *__restrict__ S, const uint8_t *__restrict__ mask,
                                                      int64_t d_out, int64_t d_in, void *__restrict__ values,
                                                      uint8_t *__restrict__ meta) {
    using PG = PackGeom<N, M>;
    constexpr int G = PG::G;
    const int64_t gpr = d_in / M, tpr = (gpr + G - 1) / G; // groups, threads per row
    const int64_t meta_row = (gpr * PG::NW + 7) / 8;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= d_out * tpr) return;
    const int64_t i = idx / tpr, g0 = (idx % tpr) * G;
    const int ng = (int)min((int64_t)G, gpr - g0);
    float v[G][M];
    uint32_t bits[G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        bits[g] = 0;
        if (g < ng) {
            bits[g] = mask[i * gpr + g0 + g];
            const float *src = S + i * d_in + (g0 + g) * M;
            if (M == 2) {
                const float2 q = *reinterpret_cast<const float2 *>(src);
                v[g][0] = q.x; v[g][1] = q.y;
            } else {
#pragma unroll
                for (int q4 = 0; q4 < M / 4; ++q4) {
                    const float4 q = reinterpret_cast<const float4 *>(src)[q4];
                    v[g][4 * q4] = q.x; v[g][4 * q4 + 1] = q.y; v[g][4 * q4 + 2] = q.z; v[g][4 * q4 + 3] = q.w;
                }
            }
        }
    }
    float kept[G][N];
    uint64_t field = 0; // G * NW <= 56 bits
#pragma unroll
    for (int g = 0; g < G; ++g) {
        int x = 0;
#pragma unroll
        for (int e = 0; e < N; ++e) kept[g][e] = 0.f;
#pragma unroll
        for (int p = 0; p < M; ++p) {
            const bool on = ((bits[g] >> p) & 1u) && x < N;
#pragma unroll
            for (int e = 0; e < N; ++e)
                if (on && x == e) kept[g][e] = v[g][p];
            if (on) {
                field |= (uint64_t)p << (g * PG::NW + x * PG::W_BITS);
                ++x;
            }
        }
    }
    const int64_t vbase = (i * gpr + g0) * N;
#pragma unroll
    for (int g = 0; g < G; ++g)
        if (g < ng) {
#pragma unroll
            for (int e = 0; e < N; ++e) {
                if (BF16) reinterpret_cast<uint16_t *>(values)[vbase + g * N + e] = float_to_bf16_rne(kept[g][e]);
                else      reinterpret_cast<float *>(values)[vbase + g * N + e] = kept[g][e];
            }
        }
    uint8_t *mrow = meta + i * meta_row + (g0 / G) * PG::BYTES;
    const int nbytes = (ng * PG::NW + 7) / 8;
#pragma unroll
    for (int q = 0; q < PG::BYTES; ++q)
        if (q < nbytes) mrow[q] = (uint8_t)(field >> (8 * q));
}

void launch_pack_nm(const float *S, const uint8_t *mask, int64_t d_out, int64_t d_in, int N, int M, void *values,
                    int bf16, uint8_t *meta, hipStream_t s) {
#define ARMOR_PACK_CASE(n, m)                                                                                      \
    if (N == n && M == m) {                                                                                        \
        const int64_t gpr = d_in / m, tpr = (gpr + PackGeom<n, m>::G - 1) / PackGeom<n, m>::G;                     \
        dim3 grid((unsigned)((d_out * tpr + 255) / 256));                                                          \
        if (bf16) hipLaunchKernelGGL((pack_nm_kernel<n, m, true>), grid, dim3(256), 0, s, S, mask, d_out, d_in, values, meta);  \
        else      hipLaunchKernelGGL((pack_nm_kernel<n, m, false>), grid, dim3(256), 0, s, S, mask, d_out, d_in, values, meta); \
        return;                                                                                                    \
    }
    ARMOR_PACK_CASE(1, 2)
    ARMOR_PACK_CASE(1, 4) ARMOR_PACK_CASE(2, 4) ARMOR_PACK_CASE(3, 4)
    ARMOR_PACK_CASE(1, 8) ARMOR_PACK_CASE(2, 8) ARMOR_PACK_CASE(3, 8) ARMOR_PACK_CASE(4, 8)
    ARMOR_PACK_CASE(5, 8) ARMOR_PACK_CASE(6, 8) ARMOR_PACK_CASE(7, 8)
#undef ARMOR_PACK_CASE
}

} // namespace armor
