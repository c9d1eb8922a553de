// Gram matrix of the calibration activations, H (+)= X^T X (Sec. 2; Eq. 2 uses its diagonal).
// X is [n_tokens x d_in] row-major, so the token index is the contraction index and both MFMA
// operands are read "k-major" straight from a row-major chunk of X staged in LDS.
// Only tile pairs (ta <= tb) are computed; the mirror tile is written from the same accumulators.
#include "armor_internal.h"

namespace armor {

typedef float floatx16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ float gram_bf16_to_float(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }

template <int T> struct GramCfg;
template <> struct GramCfg<32>  { static constexpr int WM = 1, WN = 1, TM = 1, TN = 1; };
template <> struct GramCfg<64>  { static constexpr int WM = 2, WN = 2, TM = 1, TN = 1; };
template <> struct GramCfg<128> { static constexpr int WM = 2, WN = 4, TM = 2, TN = 1; };

// fp32 MFMA path (exact products of the inputs, fp32 accumulation); bf16 inputs are widened on load.
template <int T, bool BF16>
__global__ __launch_bounds__(GramCfg<T>::WM *GramCfg<T>::WN * 64) void gram_f32_kernel(
    const void *__restrict__ X, int64_t n, int64_t ldx, int ntile, float *__restrict__ H, int64_t ldh,
    int accumulate) {
    using G = GramCfg<T>;
    constexpr int NT = G::WM * G::WN * 64, KC = 16, TM = G::TM, TN = G::TN;
    __shared__ float Xa[KC][T];
    __shared__ float Xb[KC][T];
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, l32 = lane & 31, kh = lane >> 5;
    int ta = 0, rem = blockIdx.x;
    while (rem >= ntile - ta) { rem -= ntile - ta; ++ta; }
    const int tb = ta + rem;
    const int wm0 = (w % G::WM) * TM * 32, wn0 = (w / G::WM) * TN * 32;
    floatx16 acc[TM][TN];
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int c = 0; c < TN; ++c)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][c][r] = 0.f;

    for (int64_t t0 = 0; t0 < n; t0 += KC) {
        __syncthreads();
        for (int e = tid; e < KC * T; e += NT) {
            int k = e / T, c = e % T;
            int64_t t = t0 + k;
            float va = 0.f, vb = 0.f;
            if (t < n) {
                if (BF16) {
                    const uint16_t *x = reinterpret_cast<const uint16_t *>(X) + t * ldx;
                    va = gram_bf16_to_float(x[(int64_t)ta * T + c]);
                    vb = gram_bf16_to_float(x[(int64_t)tb * T + c]);
                } else {
                    const float *x = reinterpret_cast<const float *>(X) + t * ldx;
                    va = x[(int64_t)ta * T + c];
                    vb = x[(int64_t)tb * T + c];
                }
            }
            Xa[k][c] = va;
            Xb[k][c] = vb;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < KC; k += 2) {
            float a[TM], b[TN];
#pragma unroll
            for (int tm = 0; tm < TM; ++tm) a[tm] = Xa[k + kh][wm0 + tm * 32 + l32];
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) b[tn] = Xb[k + kh][wn0 + tn * 32 + l32];
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < TN; ++tn)
                    acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[tm], b[tn], acc[tm][tn], 0, 0, 0);
        }
    }
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < TN; ++tn)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                int64_t row = (int64_t)ta * T + wm0 + tm * 32 + (r >> 2) * 8 + kh * 4 + (r & 3);
                int64_t col = (int64_t)tb * T + wn0 + tn * 32 + l32;
                float v = acc[tm][tn][r];
                float *h = H + row * ldh + col;
                *h = accumulate ? *h + v : v;
                if (ta != tb) {
                    float *hm = H + col * ldh + row;
                    *hm = accumulate ? *hm + v : v;
                }
            }
}

// ------------------------------------------------------------------------------------------------
// bf16 MFMA path (v_mfma_f32_32x32x16_bf16, fp32 accumulation) for bf16 activations.
// Workgroup = 8 waves, output tile 256 x 256 (wave patch 128 x 64 = 4 x 2 accumulator tiles), so a
// token contributes 2 * 256 * 256 flops per 1 KB read: the kernel is bounded by MFMA issue and L2
// bandwidth, not HBM.  The MFMA operands want 8 consecutive *tokens* of one channel per lane, while
// X is channel-contiguous: each thread transposes an 8 token x 8 channel patch in registers
// (v_perm_b32) on its way from global memory to LDS.  LDS holds [channel][64 tokens] bf16 per
// operand and stage (128 B rows, no padding); the 16-byte token group g of channel ch sits in slot
// g ^ ((ch ^ (ch >> 3)) & 7), which keeps both the transposed writes (lanes vary ch >> 3) and the
// operand reads (lanes vary ch & 7) spread over all banks.  Two LDS stages + a register prefetch
// of the next 64-token chunk overlap global loads with MFMA work.
// ------------------------------------------------------------------------------------------------
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// blockIdx.y = token slice (split-K): slice s covers tokens [s*slice_len, (s+1)*slice_len) and, when
// part != nullptr, writes its upper-triangular tile to part[s] ([d_in x d_in], no mirror) for the
// fixed-order reduction below; with part == nullptr (one slice) it writes / accumulates H directly.
__global__ __launch_bounds__(512) void gram_bf16_kernel(const uint16_t *__restrict__ X, int64_t ldx, int ntile,
                                                        float *__restrict__ H, int64_t ldh, int accumulate,
                                                        int64_t n_tokens, int64_t slice_len,
                                                        float *__restrict__ part, int64_t d_in) {
    constexpr int T = 256, KC = 64, TM = 4, TN = 2;
    const int64_t t_begin = (int64_t)blockIdx.y * slice_len, t_end = min(n_tokens, t_begin + slice_len);
    if (part != nullptr) {
        H = part + (int64_t)blockIdx.y * d_in * d_in;
        ldh = d_in;
        accumulate = 0;
    }
    __shared__ uint4 lds[2][2][T * 8]; // [stage][operand][channel * 8 + slot]
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, l32 = lane & 31, kh = lane >> 5;
    int ta = 0, rem = blockIdx.x;
    while (rem >= ntile - ta) { rem -= ntile - ta; ++ta; }
    const int tb = ta + rem;
    const bool diag = ta == tb;
    const int wm0 = (w & 1) * 128, wn0 = (w >> 1) * 64;

    // loader role: operand, 8-channel column, 8-token row group
    const int op = tid >> 8, lr = tid & 255, chblk = lr & 31, tokblk = lr >> 5;
    const bool loader = !(diag && op == 1);
    const uint16_t *xcol = X + (int64_t)(op ? tb : ta) * T + chblk * 8;
    uint4 pre[8];
    auto gload = [&](int64_t t0) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            int64_t row = t0 + tokblk * 8 + i;
            pre[i] = make_uint4(0u, 0u, 0u, 0u);
            if (loader && row < t_end) pre[i] = *reinterpret_cast<const uint4 *>(xcol + row * ldx);
        }
    };
    auto lstore = [&](int stage) {
        if (!loader) return;
        const uint32_t *r[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) r[i] = reinterpret_cast<const uint32_t *>(&pre[i]);
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            const uint32_t sel = (c & 1) ? 0x07060302u : 0x05040100u;
            uint4 o;
            o.x = __builtin_amdgcn_perm(r[1][c >> 1], r[0][c >> 1], sel);
            o.y = __builtin_amdgcn_perm(r[3][c >> 1], r[2][c >> 1], sel);
            o.z = __builtin_amdgcn_perm(r[5][c >> 1], r[4][c >> 1], sel);
            o.w = __builtin_amdgcn_perm(r[7][c >> 1], r[6][c >> 1], sel);
            int ch = chblk * 8 + c;
            int slot = tokblk ^ ((ch ^ (ch >> 3)) & 7);
            lds[stage][op][ch * 8 + slot] = o;
        }
    };

    floatx16 acc[TM][TN];
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int c = 0; c < TN; ++c)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][c][r] = 0.f;

    const int64_t nchunks = (t_end - t_begin + KC - 1) / KC;
    if (nchunks > 0) {
        gload(t_begin);
        lstore(0);
    }
    __syncthreads();
    for (int64_t ci = 0; ci < nchunks; ++ci) {
        const int st = (int)(ci & 1);
        if (ci + 1 < nchunks) gload(t_begin + (ci + 1) * KC);
        const uint4 *La = lds[st][0];
        const uint4 *Lb = lds[st][diag ? 0 : 1];
#pragma unroll
        for (int ks = 0; ks < KC / 16; ++ks) {
            const int g = ks * 2 + kh;
            bf16x8 a[TM], b[TN];
#pragma unroll
            for (int tm = 0; tm < TM; ++tm) {
                int ch = wm0 + tm * 32 + l32;
                a[tm] = __builtin_bit_cast(bf16x8, La[ch * 8 + (g ^ ((ch ^ (ch >> 3)) & 7))]);
            }
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) {
                int ch = wn0 + tn * 32 + l32;
                b[tn] = __builtin_bit_cast(bf16x8, Lb[ch * 8 + (g ^ ((ch ^ (ch >> 3)) & 7))]);
            }
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < TN; ++tn)
                    acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[tm], b[tn], acc[tm][tn], 0, 0, 0);
        }
        if (ci + 1 < nchunks) lstore(st ^ 1);
        __syncthreads();
    }
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < TN; ++tn)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                int64_t row = (int64_t)ta * T + wm0 + tm * 32 + (r >> 2) * 8 + kh * 4 + (r & 3);
                int64_t col = (int64_t)tb * T + wn0 + tn * 32 + l32;
                float v = acc[tm][tn][r];
                float *h = H + row * ldh + col;
                *h = accumulate ? *h + v : v;
                if (!diag && part == nullptr) {
                    float *hm = H + col * ldh + row;
                    *hm = accumulate ? *hm + v : v;
                }
            }
}

// H (+)= sum over slices, in slice order, of the upper-triangular tiles in part[]; mirror tiles are
// written through an LDS transpose so both stores are row-contiguous.  One workgroup per 32 x 32
// sub-block: blockIdx.x = tile pair, blockIdx.y = sub-block inside the 256 x 256 tile.
__global__ __launch_bounds__(256) void gram_reduce_kernel(const float *__restrict__ part, int nslices, int64_t d_in,
                                                          int ntile, float *__restrict__ H, int64_t ldh,
                                                          int accumulate) {
    __shared__ float tr[32][33];
    int ta = 0, rem = blockIdx.x;
    while (rem >= ntile - ta) { rem -= ntile - ta; ++ta; }
    const int tb = ta + rem;
    const int sr = blockIdx.y / 8, sc = blockIdx.y % 8;
    const int64_t row0 = (int64_t)ta * 256 + sr * 32, col0 = (int64_t)tb * 256 + sc * 32;
    const int c = threadIdx.x & 31, r0 = threadIdx.x >> 5; // 8 rows per pass
#pragma unroll
    for (int pass = 0; pass < 4; ++pass) {
        const int r = pass * 8 + r0;
        float v = 0.f;
        for (int sl = 0; sl < nslices; ++sl) v += part[((int64_t)sl * d_in + row0 + r) * d_in + col0 + c];
        tr[r][c] = v;
        float *h = H + (row0 + r) * ldh + col0 + c;
        *h = accumulate ? *h + v : v;
    }
    if (ta == tb) return; // a diagonal tile holds both of its triangles already
    __syncthreads();
#pragma unroll
    for (int pass = 0; pass < 4; ++pass) {
        const int r = pass * 8 + r0;
        float *hm = H + (col0 + r) * ldh + row0 + c;
        const float v = tr[c][r];
        *hm = accumulate ? *hm + v : v;
    }
}

// Split-K plan for the bf16 kernel: with one 128 KB-LDS workgroup per CU, `pairs` tile pairs alone
// leave CUs idle (136 pairs at d_in = 4096); slicing the tokens S ways gives pairs * S workgroups.
// Cost model: rounds * (tokens per slice + a fixed per-workgroup overhead).
static int gram_slices(int64_t n, int64_t d_in, size_t ws_bytes) {
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
        cus = 256;
    const int64_t nt = d_in / 256, pairs = nt * (nt + 1) / 2;
    int best = 1;
    double best_cost = 1e300;
    for (int S = 1; S <= 32; ++S) {
        if (S > 1 && (size_t)S * d_in * d_in * sizeof(float) > ws_bytes) break;
        int64_t len = ((n + S - 1) / S + 63) / 64 * 64;
        if (S > 1 && len < 2048) break;
        int64_t rounds = (pairs * S + cus - 1) / cus;
        double cost = (double)rounds * ((double)len + 768.0);
        if (cost < best_cost * 0.97) { best_cost = cost; best = S; }
    }
    return best;
}

size_t gram_workspace_bytes(int64_t n, int64_t d_in, int bf16) {
    if (!bf16 || d_in % 256 != 0) return 0;
    int S = gram_slices(n, d_in, (size_t)4 << 30);
    return S > 1 ? (size_t)S * d_in * d_in * sizeof(float) : 0;
}

void launch_gram(const void *X, int bf16, int64_t n, int64_t d_in, int64_t ldx, float *H, int64_t ldh,
                 int accumulate, void *ws, size_t ws_bytes, hipStream_t s) {
    if (bf16 && d_in % 256 == 0 && ldx % 8 == 0) {
        int nt = (int)(d_in / 256), pairs = nt * (nt + 1) / 2;
        int S = ws ? gram_slices(n, d_in, ws_bytes) : 1;
        int64_t len = S > 1 ? ((n + S - 1) / S + 63) / 64 * 64 : n;
        float *part = S > 1 ? reinterpret_cast<float *>(ws) : nullptr;
        hipLaunchKernelGGL(gram_bf16_kernel, dim3((unsigned)pairs, (unsigned)S), dim3(512), 0, s,
                           reinterpret_cast<const uint16_t *>(X), ldx, nt, H, ldh, accumulate, n, len, part, d_in);
        if (S > 1)
            hipLaunchKernelGGL(gram_reduce_kernel, dim3((unsigned)pairs, 64), dim3(256), 0, s, part, S, d_in, nt, H, ldh,
                               accumulate);
        return;
    }
    int T = (d_in % 128 == 0) ? 128 : (d_in % 64 == 0) ? 64 : 32;
    int ntile = (int)(d_in / T);
    dim3 grid((unsigned)(ntile * (ntile + 1) / 2));
#define ARMOR_GRAM_CASE(tt)                                                                                        \
    if (T == tt) {                                                                                                 \
        dim3 block(GramCfg<tt>::WM * GramCfg<tt>::WN * 64);                                                        \
        if (bf16) hipLaunchKernelGGL((gram_f32_kernel<tt, true>), grid, block, 0, s, X, n, ldx, ntile, H, ldh, accumulate);  \
        else      hipLaunchKernelGGL((gram_f32_kernel<tt, false>), grid, block, 0, s, X, n, ldx, ntile, H, ldh, accumulate); \
        return;                                                                                                    \
    }
    ARMOR_GRAM_CASE(128) ARMOR_GRAM_CASE(64) ARMOR_GRAM_CASE(32)
#undef ARMOR_GRAM_CASE
}

} // namespace armor
