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

// ------------------------------------------------------------------------------------------------
// The same product with the gfx950 data path: token-major tiles go from global memory straight
// into LDS (global_load_lds_dwordx4: 16 B per lane, 1 KB = two 512-byte token rows per
// instruction, no register staging, no shuffles), four LDS slots of 32 tokens, up to three stages
// in flight; the matrix-core operands (8 consecutive tokens of one channel per lane) are read with
// the transposing LDS load ds_read_b64_tr_b16: inside each group of 16 lanes, lane j supplies 8
// bytes and lane i receives element i % 4 of the data of lanes i/4, 4 + i/4, 8 + i/4, 12 + i/4.
// Lane j therefore points at token row j/4 and channels 4 (j % 4) .. +3 of a 16-channel group, and
// lane i receives channel i at four consecutive tokens.  LDS rows are unpadded (512 B); the 64-byte
// segments of row r are stored at segment s ^ (r & 3) (applied to the global address of the loading
// lane), so the four rows a half-wave reads together fall on distinct banks.
// Rows past the end of the slice are read from a page of zeros.
// ------------------------------------------------------------------------------------------------
__device__ __attribute__((aligned(16))) uint4 g_gram_zero_row[32]; // 512 zero bytes

typedef short short4v __attribute__((ext_vector_type(4)));
typedef short short8v __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) short4v *lds_short4_ptr;
typedef __attribute__((address_space(3))) void *lds_void_ptr;

__device__ __forceinline__ void gram_dma16(const void *g, uint32_t lds_byte_addr) {
    // issued as assembly so that the compiler keeps no book on these loads: completion is waited for
    // explicitly (s_waitcnt vmcnt) before the barrier that publishes a stage
    asm volatile("s_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "{m0}"(lds_byte_addr) : "memory");
}

#define GRAM_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(0x0f70 | ((n) & 15) | (((n) >> 4) << 14))

constexpr int GD_T = 256, GD_K = 32, GD_SLOTS = 4; // (a fifth slot, all of the LDS, measured slower)
constexpr int GD_TILE_BYTES = GD_K * GD_T * 2; // 16 KB: 32 token rows of 256 channels
constexpr int GD_SLOT_BYTES = 2 * GD_TILE_BYTES;

// Tile pairs (ta <= tb) in an order that keeps neighbours close: blocks of 4 row tiles x 8 column
// tiles, row-major over the blocks, row-major inside.  32 consecutive pairs then touch about 12
// channel blocks instead of 17 to 33.
__device__ __forceinline__ void gram_pair_from_index(int idx, int ntile, int &ta, int &tb) {
    for (int bi = 0; bi * 4 < ntile; ++bi)
        for (int bj = (bi * 4) / 8; bj * 8 < ntile; ++bj) {
            int cnt = 0;
            for (int r = bi * 4; r < min(bi * 4 + 4, ntile); ++r) {
                const int c_lo = max(bj * 8, r), c_hi = min(bj * 8 + 8, ntile);
                cnt += max(0, c_hi - c_lo);
            }
            if (idx >= cnt) { idx -= cnt; continue; }
            for (int r = bi * 4; r < min(bi * 4 + 4, ntile); ++r) {
                const int c_lo = max(bj * 8, r), c_hi = min(bj * 8 + 8, ntile);
                const int m = max(0, c_hi - c_lo);
                if (idx < m) { ta = r; tb = c_lo + idx; return; }
                idx -= m;
            }
        }
    ta = tb = 0; // not reached for idx < ntile (ntile + 1) / 2
}

// Work item = (token slice, tile pair).  Workgroups go to the 8 XCDs round-robin (each XCD has its
// own L2; all share the memory-side cache).  The pairs, in the order above, are cut into 8 runs of
// `cl`, one per XCD, and an XCD works on its run for `gs` slices at a time (gs * cl >= 32 resident
// workgroups): the workgroups resident on one XCD share tokens and neighbouring tiles (L2), and at
// any time the whole chip works on the same gs slices, so a row of X is fetched from HBM about once
// and found in the memory-side cache by the other XCDs that need it.
__global__ __launch_bounds__(512) void gram_bf16_dma_kernel(const uint16_t *__restrict__ X, int64_t ldx, int ntile,
                                                            float *__restrict__ H, int64_t ldh, int accumulate,
                                                            int64_t n_tokens, int64_t slice_len,
                                                            float *__restrict__ part, int64_t d_in, int npairs,
                                                            int nslices, int cl, int gs) {
    constexpr int TM = 4, TN = 2;
    const int xcd = (int)(blockIdx.x & 7), q = (int)(blockIdx.x >> 3);
    const int grp = q / (gs * cl), in_grp = q % (gs * cl);
    const int slice = grp * gs + in_grp / cl, pidx = xcd * cl + in_grp % cl;
    if (slice >= nslices || pidx >= npairs) return; // uniform for the workgroup
    const int64_t t_begin = (int64_t)slice * slice_len, t_end = min(n_tokens, t_begin + slice_len);
    if (part != nullptr) {
        H = part + (int64_t)slice * d_in * d_in;
        ldh = d_in;
        accumulate = 0;
    }
    __shared__ __attribute__((aligned(16))) uint8_t lds[GD_SLOTS * GD_SLOT_BYTES];
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, l32 = lane & 31, kh = lane >> 5;
    int ta, tb;
    gram_pair_from_index(pidx, ntile, ta, tb);
    const bool diag = ta == tb;
    const int wm = w & 1, wn = w >> 1, wm0 = wm * 128, wn0 = wn * 64;
    const uint32_t lds0 = (uint32_t)(size_t)(lds_void_ptr)lds;

    // loader role: per stage and operand this wave brings token rows 4w .. 4w+3 (two 1 KB loads);
    // lane -> (row 2c + lane/32, stored segment (lane%32)/4, 16-byte part lane%4)
    const int lrow = lane >> 5, lseg = (lane & 31) >> 2, lpart = lane & 3;
    auto issue = [&](int64_t st) {
        const uint32_t sb = lds0 + (uint32_t)(st % GD_SLOTS) * GD_SLOT_BYTES;
#pragma unroll
        for (int op = 0; op < 2; ++op) {
            if (op == 1 && diag) break;
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                const int r = 4 * w + 2 * c + lrow;                 // token row inside the stage
                const int64_t tok = t_begin + st * GD_K + r;
                const int sseg = lseg ^ (r & 3);                    // source segment stored at lseg
                const uint8_t *src = tok < t_end
                    ? reinterpret_cast<const uint8_t *>(X + tok * ldx + (int64_t)(op ? tb : ta) * GD_T) + sseg * 64 + lpart * 16
                    : reinterpret_cast<const uint8_t *>(g_gram_zero_row) + (lane & 31) * 16;
                gram_dma16(src, sb + op * GD_TILE_BYTES + (4 * w + 2 * c) * 512);
            }
        }
    };

    floatx16 acc[TM][TN];
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int c = 0; c < TN; ++c)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][c][r] = 0.f;

    // reader offsets: lane j of a 16-lane group points at token row (8 kh + j/4) and channels
    // 16 (l32/16) + 4 (j%4) .. +3 of the 32-channel segment of its accumulator tile
    const int j16 = lane & 15, rq = j16 >> 2;
    const int within = (16 * (l32 >> 4) + 4 * (j16 & 3)) * 2;
    int a_off[TM], b_off[TN];
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) a_off[tm] = (8 * kh + rq) * 512 + (((4 * wm + tm) ^ rq) * 64) + within;
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) b_off[tn] = (8 * kh + rq) * 512 + (((2 * wn + tn) ^ rq) * 64) + within;

    const int64_t nstages = (t_end - t_begin + GD_K - 1) / GD_K;
    const int per = diag ? 2 : 4; // load instructions per wave per stage

    // operand fragments of one 16-token step: 4 row tiles + 2 column tiles, two transposing reads each
    struct Frags { short4v a[TM][2], b[TN][2]; };
    auto read_frags = [&](Frags &f, int64_t st, int ks) {
        const uint8_t *La = lds + (st % GD_SLOTS) * GD_SLOT_BYTES;
        const uint8_t *Lb = La + (diag ? 0 : GD_TILE_BYTES);
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) {
            f.a[tm][0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(La + a_off[tm] + (16 * ks) * 512));
            f.a[tm][1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(La + a_off[tm] + (16 * ks + 4) * 512));
        }
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) {
            f.b[tn][0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(Lb + b_off[tn] + (16 * ks) * 512));
            f.b[tn][1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(Lb + b_off[tn] + (16 * ks + 4) * 512));
        }
    };
    auto mma = [&](const Frags &f) {
        bf16x8 a[TM], b[TN];
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
            a[tm] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(f.a[tm][0], f.a[tm][1], 0, 1, 2, 3, 4, 5, 6, 7));
#pragma unroll
        for (int tn = 0; tn < TN; ++tn)
            b[tn] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(f.b[tn][0], f.b[tn][1], 0, 1, 2, 3, 4, 5, 6, 7));
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
                acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[tm], b[tn], acc[tm][tn], 0, 0, 0);
    };
    // wait until this wave's loads of stage `st` have landed (at most the loads of `later` younger stages
    // may still be outstanding), then meet the other waves
    auto publish = [&](int later) {
        if (later <= 0) { GRAM_WAIT_VMCNT(0); }
        else if (per == 2) { if (later == 1) { GRAM_WAIT_VMCNT(2); } else if (later == 2) { GRAM_WAIT_VMCNT(4); } else { GRAM_WAIT_VMCNT(6); } }
        else { if (later == 1) { GRAM_WAIT_VMCNT(4); } else if (later == 2) { GRAM_WAIT_VMCNT(8); } else { GRAM_WAIT_VMCNT(12); } }
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    };

    // Software pipeline over half-stages: the operand reads of a 16-token step are issued one step
    // before its MFMAs, across stage boundaries too.  The barrier that publishes stage st+1 sits in
    // the middle of stage st; after it every wave has finished stage st-1, whose slot then takes the
    // loads of stage st + GD_SLOTS - 1.
    static_assert(GD_K == 32, "two 16-token steps per stage");
    Frags f0, f1;
    if (nstages > 0) {
        for (int64_t st = 0; st < GD_SLOTS - 1 && st < nstages; ++st) issue(st);
        publish((int)min((int64_t)(GD_SLOTS - 2), nstages - 1));
        read_frags(f0, 0, 0);
    }
    // (the last stage is peeled: with the second half under a condition, the paths that meet in front
    // of mma(f1) differ in their outstanding LDS reads and the compiler makes that product wait for
    // the reads of f0 that were issued a moment ago)
    int64_t st = 0;
    // steady state: a new stage is issued every trip and exactly one younger stage is in flight at the
    // barrier, so the wait is a constant and the trip has no branches
    static_assert(GD_SLOTS == 4, "one younger stage in flight in the steady state");
    if (diag) {
        for (; st + GD_SLOTS - 1 < nstages; ++st) {
            read_frags(f1, st, 1);
            mma(f0);
            GRAM_WAIT_VMCNT(2);
            asm volatile("" ::: "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            issue(st + GD_SLOTS - 1);
            read_frags(f0, st + 1, 0);
            mma(f1);
        }
    } else {
        for (; st + GD_SLOTS - 1 < nstages; ++st) {
            read_frags(f1, st, 1);
            mma(f0);
            GRAM_WAIT_VMCNT(4);
            asm volatile("" ::: "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            issue(st + GD_SLOTS - 1);
            read_frags(f0, st + 1, 0);
            mma(f1);
        }
    }
    for (; st + 1 < nstages; ++st) { // the last stages: nothing left to issue
        read_frags(f1, st, 1);
        mma(f0);
        publish((int)min((int64_t)(GD_SLOTS - 3), nstages - 2 - st)); // stage st+1 landed; younger ones may be in flight
        read_frags(f0, st + 1, 0);
        mma(f1);
    }
    if (nstages > 0) {
        read_frags(f1, nstages - 1, 1);
        mma(f0);
        mma(f1);
    }
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < TN; ++tn)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                int64_t row = (int64_t)ta * GD_T + wm0 + tm * 32 + (r >> 2) * 8 + kh * 4 + (r & 3);
                int64_t col = (int64_t)tb * GD_T + wn0 + tn * 32 + l32;
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
        if ((reinterpret_cast<uintptr_t>(X) & 15) == 0) { // the LDS-direct loads want 16-byte aligned rows
            const int cl = (pairs + 7) / 8, gs = std::min(S, std::max(1, (32 + cl - 1) / cl));
            const int per_xcd = ((S + gs - 1) / gs) * gs * cl;
            hipLaunchKernelGGL(gram_bf16_dma_kernel, dim3((unsigned)(per_xcd * 8)), dim3(512), 0, s,
                               reinterpret_cast<const uint16_t *>(X), ldx, nt, H, ldh, accumulate, n, len, part, d_in,
                               pairs, S, cl, gs);
        }
        else
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
