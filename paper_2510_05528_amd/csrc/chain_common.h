// Building blocks shared by the chain kernels: wave tiling, LDS tile movement and the LDS-resident
// fp32 MFMA product (v_mfma_f32_32x32x2_f32) on b x (b+1) tiles.  gfx950 only.
#pragma once
#include "armor_internal.h"
#include "planes.h"

namespace armor {

typedef float floatx16 __attribute__((ext_vector_type(16)));

// Adam coefficients of iteration t as the kernels use them (Sec. 3.3.1); inv_c = 1 / (1 - beta^t).
struct AdamCoef {
    float b1, b2, one_minus_b1, one_minus_b2, inv_c1, inv_c2, lr, eps;
};
inline AdamCoef make_adam_coef(double lr, double b1, double b2, double eps, int64_t t) {
    AdamCoef k;
    k.b1 = (float)b1; k.b2 = (float)b2; k.one_minus_b1 = (float)(1.0 - b1); k.one_minus_b2 = (float)(1.0 - b2);
    k.inv_c1 = (float)(1.0 / (1.0 - pow(b1, (double)t))); k.inv_c2 = (float)(1.0 / (1.0 - pow(b2, (double)t)));
    k.lr = (float)lr; k.eps = (float)eps;
    return k;
}

// Hides a per-lane offset from loop-invariant code motion: without it the compiler hoists every
// unrolled address of the epilogues out of the block loop and keeps hundreds of them live across
// the matrix products (spilling accumulators), instead of re-deriving each with one add.
__device__ __forceinline__ int opaque(int x) {
    asm volatile("" : "+v"(x));
    return x;
}

__device__ __forceinline__ uint32_t opaque_u(uint32_t x) {
    asm volatile("" : "+v"(x));
    return x;
}

// Global access at a wave-uniform base pointer plus a 32-bit unsigned byte offset.  This is the form
// that maps onto the scalar-base addressing mode of the global instructions (one vector add per
// access); a signed element index instead costs a sign extension and a 64-bit pointer sum each time,
// which made address arithmetic the bulk of the epilogues' vector instructions.  The offsets stay
// inside one b x b block of a matrix, far below 4 GB.
template <class T> __device__ __forceinline__ T gld(const T *base, uint32_t boff) {
    return *reinterpret_cast<const T *>(reinterpret_cast<const char *>(base) + boff);
}
template <class T> __device__ __forceinline__ void gst(T *base, uint32_t boff, T v) {
    *reinterpret_cast<T *>(reinterpret_cast<char *>(base) + boff) = v;
}

__device__ __forceinline__ floatx16 mfma_bf16(const uintx4 &a, const uintx4 &b, const floatx16 &c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// A configuration's SPLIT chooses the matrix instruction of the LDS-resident products (Chain::mma):
// true = bf16 pieces as above, false = v_mfma_f32_32x32x2_f32.
template <int B> struct Cfg;
template <> struct Cfg<32>  { static constexpr int WM = 1, WN = 1, TM = 1, TN = 1; static constexpr bool SPLIT = false; };
template <> struct Cfg<64>  { static constexpr int WM = 2, WN = 2, TM = 1, TN = 1; static constexpr bool SPLIT = false; };
// 8 waves at b = 128, each owning a 64 x 32 patch: two waves share a SIMD, so one wave's LDS reads
// and address arithmetic overlap the other's MFMA issue (measured: same loop rate as 4 waves of
// 64 x 64 or 16 waves of 32 x 32, but the only shape that leaves registers for operand prefetch).
template <> struct Cfg<128> { static constexpr int WM = 2, WN = 4, TM = 2, TN = 1; static constexpr bool SPLIT = false; };

template <int B, class C = Cfg<B>> struct Chain {
    static constexpr int WM = C::WM, WN = C::WN, TM = C::TM, TN = C::TN;
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
        // 32-bit element offset of accumulator element (tm,tn,r) in a row-major matrix of leading
        // dimension ld, split into a per-lane part and a wave-uniform part so that the address is
        // "uniform base + one VGPR" and nothing 64-bit per element stays live.
        __device__ int lane_off(int ld) const { return (wm0 + kh * 4) * ld + wn0 + l32; }
        __device__ static int unif_off(int tm, int tn, int r, int ld) {
            return (tm * 32 + (r >> 2) * 8 + (r & 3)) * ld + tn * 32;
        }
        // the same as byte offsets of fp32 elements, for gld / gst
        __device__ uint32_t lane_boff(int ld) const { return 4u * (uint32_t)lane_off(ld); }
        __device__ static uint32_t unif_boff(int tm, int tn, int r, int ld) { return 4u * (uint32_t)unif_off(tm, tn, r, ld); }
    };

    // global (row-major, leading dimension ld) -> registers -> LDS tile, in two halves so that the
    // global loads of the next operand can stay in flight underneath a matrix product.
    static constexpr int PER = B * B / 4 / NT;
    static_assert((B * B / 4) % NT == 0, "tile load must divide evenly");
    struct TileRegs { float4 v[PER]; };

    // Loader lane mapping: every group of 32 lanes covers 4 rows x 8 float4 columns, so a global
    // load instruction still reads whole 128-byte lines while the four scalar LDS writes of a
    // float4 (stride 16 B across lanes of a row, +1 bank per row with the odd pitch) hit 32
    // different banks.
    static constexpr int ROWS_PER_IT = NT / (B / 4); // tile rows covered by one pass of the workgroup
    __device__ static __forceinline__ int loader_row(int tid) { return ((tid >> 5) / (B / 32)) * 4 + ((tid & 31) >> 3); }
    __device__ static __forceinline__ int loader_c4(int tid) { return ((tid >> 5) % (B / 32)) * 8 + (tid & 7); }

    __device__ static __forceinline__ void gload_tile(TileRegs &t, const float *__restrict__ g, int ld, int tid) {
        const int off0 = opaque(loader_row(tid) * ld + loader_c4(tid) * 4);
#pragma unroll
        for (int it = 0; it < PER; ++it)
            t.v[it] = *reinterpret_cast<const float4 *>(g + (off0 + it * ROWS_PER_IT * ld));
    }

    __device__ static __forceinline__ void lstore_tile(float *T, const TileRegs &t, int tid) {
        float *d0 = T + opaque(loader_row(tid) * P + loader_c4(tid) * 4);
#pragma unroll
        for (int it = 0; it < PER; ++it) {
            float *d = d0 + it * ROWS_PER_IT * P;
            d[0] = t.v[it].x; d[1] = t.v[it].y; d[2] = t.v[it].z; d[3] = t.v[it].w;
        }
    }

    __device__ static void load_tile(float *T, const float *__restrict__ g, int ld, int tid) {
        TileRegs t;
        gload_tile(t, g, ld, tid);
        lstore_tile(T, t, tid);
    }

    __device__ static void store_acc(float *T, const Acc &acc, const Pos &p) {
        float *d0 = T + opaque(p.lane_off(P));
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                for (int r = 0; r < 16; ++r) d0[Pos::unif_off(tm, tn, r, P)] = acc.v[tm][tn][r];
    }

    // acc += op(L) * op(R) over the b inner indices.  op(L)(m,k) = LT ? L[k][m] : L[m][k];
    // op(R)(k,n) = RT ? R[n][k] : R[k][n];  SCALE multiplies op(L)(m,k) by Dk[k].
    // Operands are fetched one group of G k-steps ahead of the MFMAs that consume them (two
    // register sets), so LDS latency is covered by the wave's own matrix work.
    static constexpr int G = 2;
    struct Frag { float a[G][TM], b[G][TN]; };

    template <bool LT, bool RT, bool SCALE>
    __device__ static __forceinline__ void fetch(Frag &f, int k0, const float *__restrict__ L,
                                                 const float *__restrict__ R, const float *__restrict__ Dk,
                                                 const Pos &p) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
            int kk = k0 + 2 * g + p.kh;
#pragma unroll
            for (int tm = 0; tm < TM; ++tm) {
                int m = p.wm0 + tm * 32 + p.l32;
                f.a[g][tm] = LT ? L[kk * P + m] : L[m * P + kk];
            }
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) {
                int n = p.wn0 + tn * 32 + p.l32;
                f.b[g][tn] = RT ? R[n * P + kk] : R[kk * P + n];
            }
            if (SCALE) {
                float dk = Dk[kk];
#pragma unroll
                for (int tm = 0; tm < TM; ++tm) f.a[g][tm] *= dk;
            }
        }
    }

    // FIRST: the first matrix instruction of every accumulator tile takes a zero C operand, i.e. the
    // product overwrites acc and nobody has to clear 16 registers per tile beforehand.
    template <bool FIRST = false> __device__ static __forceinline__ void issue(Acc &acc, const Frag &f) {
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < TN; ++tn) {
                    if (FIRST && g == 0) {
                        const floatx16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                        acc.v[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x2f32(f.a[g][tm], f.b[g][tn], zero, 0, 0, 0);
                    } else {
                        acc.v[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x2f32(f.a[g][tm], f.b[g][tn], acc.v[tm][tn], 0, 0, 0);
                    }
                }
    }

    // acc (+)= op(L) * op(R); ZERO: acc = op(L) * op(R) (see issue).
    // PEEL: the last trip is peeled off the loop.  A fetch under a condition inside the loop splits it
    // into blocks, and the wait in front of the next matrix instructions then has to cover the path
    // without the fetch, i.e. it also waits for operands requested a moment ago (LDS-fed loop alone:
    // 83 % of the fp32 matrix peak with the condition, 91 % peeled).  Inside a kernel the better form
    // depends on what else is live around the product, so call sites choose by measurement.
    // The same product on the bf16 matrix instruction: the fp32 LDS operands are cut into their three
    // bf16 pieces as they are read.  One lane supplies eight consecutive inner indices of a group of 16
    // (lane half kh: 8 kh .. 8 kh + 7); the pieces of group g + 1 are cut underneath the 6 TM TN matrix
    // instructions of group g and the raw values of group g + 2 are read underneath those as well.
    template <bool LT, bool RT, bool SCALE>
    __device__ static __forceinline__ void fetch16(float (&a)[TM][8], float (&b)[TN][8], int g,
                                                   const float *__restrict__ L, const float *__restrict__ R,
                                                   const float *__restrict__ Dk, const Pos &p) {
        const int k0 = 16 * g + 8 * p.kh;
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) {
            const int m = p.wm0 + tm * 32 + p.l32;
#pragma unroll
            for (int e = 0; e < 8; ++e) a[tm][e] = LT ? L[(k0 + e) * P + m] : L[m * P + k0 + e];
        }
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) {
            const int n = p.wn0 + tn * 32 + p.l32;
#pragma unroll
            for (int e = 0; e < 8; ++e) b[tn][e] = RT ? R[n * P + k0 + e] : R[(k0 + e) * P + n];
        }
        if (SCALE) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float dk = Dk[k0 + e];
#pragma unroll
                for (int tm = 0; tm < TM; ++tm) a[tm][e] *= dk;
            }
        }
    }

    template <bool LT, bool RT, bool SCALE, bool ZERO, class Late>
    __device__ static __forceinline__ void mma_split(Acc &acc, const float *__restrict__ L, const float *__restrict__ R,
                                                     const float *__restrict__ Dk, const Pos &p, Late &&late) {
        static_assert(B % 16 == 0, "groups of 16 inner indices");
        constexpr int NG = B / 16;
        float ra[TM][8], rb[TN][8];
        Pieces pa[2][TM], pb[2][TN];
        fetch16<LT, RT, SCALE>(ra, rb, 0, L, R, Dk, p);
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) cut3(ra[tm], pa[0][tm]);
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) cut3(rb[tn], pb[0][tn]);
        if (NG > 1) fetch16<LT, RT, SCALE>(ra, rb, 1, L, R, Dk, p);
#pragma unroll
        for (int g = 0; g < NG; ++g) {
            const int cur = g & 1;
            if (g + 1 < NG) {
#pragma unroll
                for (int tm = 0; tm < TM; ++tm) cut3(ra[tm], pa[cur ^ 1][tm]);
#pragma unroll
                for (int tn = 0; tn < TN; ++tn) cut3(rb[tn], pb[cur ^ 1][tn]);
            }
            if (g + 2 < NG) fetch16<LT, RT, SCALE>(ra, rb, g + 2, L, R, Dk, p);
            if (g == (NG > 2 ? NG - 2 : 0)) late();
            // small partial products first: (3,1) (1,3) (2,2) (2,1) (1,2) (1,1)
#pragma unroll
            for (int c = 0; c < 6; ++c)
#pragma unroll
                for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                    for (int tn = 0; tn < TN; ++tn) {
                        const Pieces &x = pa[cur][tm], &y = pb[cur][tn];
                        const uintx4 a = c == 0 ? vec4(x.p3) : (c == 2 || c == 3) ? vec4(x.p2) : vec4(x.p1);
                        const uintx4 b = c == 1 ? vec4(y.p3) : (c == 2 || c == 4) ? vec4(y.p2) : vec4(y.p1);
                        if (ZERO && g == 0 && c == 0) {
                            const floatx16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                            acc.v[tm][tn] = mfma_bf16(a, b, zero);
                        } else {
                            acc.v[tm][tn] = mfma_bf16(a, b, acc.v[tm][tn]);
                        }
                    }
            // issue order: a matrix instruction, then its share of the cuts and of the LDS reads
            constexpr int NM = 6 * TM * TN, NV = 11 * 4 * (TM + TN) + (SCALE ? 8 * TM : 0), ND = 8 * (TM + TN) + (SCALE ? 8 : 0);
#pragma unroll
            for (int m = 0; m < NM; ++m) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, (NV + NM - 1) / NM, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, (ND + NM - 1) / NM, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }

    // late(): requests whose results are wanted right after the product (what an epilogue reads from
    // global memory); issued two groups before the end of the bf16 form, where the registers of the
    // operand pipeline start to free up, and in front of the fp32 form.
    struct NoLate {
        __device__ void operator()() const {}
    };
    template <bool LT, bool RT, bool SCALE, bool PEEL = true, bool ZERO = false, class Late = NoLate>
    __device__ static void mma(Acc &acc, const float *__restrict__ L, const float *__restrict__ R,
                               const float *__restrict__ Dk, const Pos &p, Late &&late = Late()) {
        if constexpr (C::SPLIT) {
            mma_split<LT, RT, SCALE, ZERO>(acc, L, R, Dk, p, late);
            return;
        }
        late();
        static_assert(B % (4 * G) == 0 && B >= 12 * G, "two groups per trip; head, loop and tail trips");
        Frag f0, f1;
        fetch<LT, RT, SCALE>(f0, 0, L, R, Dk, p);
        int k = 0;
        // The scheduling fences keep the order "request the next group, then the matrix instructions of
        // the current one": left alone, the scheduler sinks the LDS reads to just in front of their
        // first use inside the kernels, and every group then waits for its own operands.
#define ARMOR_MMA_FENCE() __builtin_amdgcn_sched_barrier(0)
        if constexpr (ZERO) { // head trip
            fetch<LT, RT, SCALE>(f1, 2 * G, L, R, Dk, p);
            ARMOR_MMA_FENCE();
            issue<true>(acc, f0);
            ARMOR_MMA_FENCE();
            fetch<LT, RT, SCALE>(f0, 4 * G, L, R, Dk, p);
            ARMOR_MMA_FENCE();
            issue(acc, f1);
            ARMOR_MMA_FENCE();
            k = 4 * G;
        }
        if constexpr (PEEL) {
#pragma unroll 1
            for (; k < B - 4 * G; k += 4 * G) {
                fetch<LT, RT, SCALE>(f1, k + 2 * G, L, R, Dk, p);
                ARMOR_MMA_FENCE();
                issue(acc, f0);
                ARMOR_MMA_FENCE();
                fetch<LT, RT, SCALE>(f0, k + 4 * G, L, R, Dk, p);
                ARMOR_MMA_FENCE();
                issue(acc, f1);
                ARMOR_MMA_FENCE();
            }
            fetch<LT, RT, SCALE>(f1, B - 2 * G, L, R, Dk, p);
            ARMOR_MMA_FENCE();
            issue(acc, f0);
            issue(acc, f1);
        } else {
#pragma unroll 1
            for (; k < B; k += 4 * G) {
                fetch<LT, RT, SCALE>(f1, k + 2 * G, L, R, Dk, p);
                ARMOR_MMA_FENCE();
                issue(acc, f0);
                ARMOR_MMA_FENCE();
                if (k + 4 * G < B) fetch<LT, RT, SCALE>(f0, k + 4 * G, L, R, Dk, p);
                ARMOR_MMA_FENCE();
                issue(acc, f1);
                ARMOR_MMA_FENCE();
            }
        }
#undef ARMOR_MMA_FENCE
    }

    // Squared Frobenius norm of the symmetric product X X^T (XT = false; rows of the tile) or X^T X
    // (XT = true), as this lane's share of the sum.  At b = 128 only the 10 upper-triangular 32 x 32
    // tiles of the 4 x 4 grid are formed, off-diagonal ones counted twice; the two SIMDs that carry
    // a two-tile wave and a one-tile wave set the time, 3 tile-products instead of the 4 every SIMD
    // does for the full product.  Wave -> tiles: w0 (0,0)(0,1), w1 (1,1)(1,2), w2 (2,2), w3 (3,3),
    // w4 (0,2), w5 (0,3), w6 (1,3), w7 (2,3).
    template <bool XT> __device__ static float sym_frob2(const float *__restrict__ X, const Pos &p, int tid) {
        if constexpr (B != 128) {
            Acc acc;
            acc.zero();
            mma<XT, !XT, false>(acc, X, X, nullptr, p);
            float f2 = 0.f;
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                    for (int r = 0; r < 16; ++r) f2 += acc.v[tm][tn][r] * acc.v[tm][tn][r];
            return f2;
        } else {
            const int w = tid >> 6;
            const int rt = w < 4 ? w : (w < 6 ? 0 : w - 5);
            const int ct = w < 4 ? w : (w == 4 ? 2 : 3);
            const bool two = w < 2;
            const int ra = XT ? 32 * rt + p.l32 : (32 * rt + p.l32) * P;
            const int cb = XT ? 32 * ct + p.l32 : (32 * ct + p.l32) * P;
            const int cstep = XT ? 32 : 32 * P;     // to the next column tile
            const int kstride = XT ? P : 1;         // one k step
            const float *xa = X + ra + p.kh * kstride, *xb = X + cb + p.kh * kstride;
            floatx16 a0, a1;
#pragma unroll
            for (int r = 0; r < 16; ++r) { a0[r] = 0.f; a1[r] = 0.f; }
            if (two) {
#pragma unroll 8
                for (int k = 0; k < B; k += 2) {
                    const float fa = xa[k * kstride], fb0 = xb[k * kstride], fb1 = xb[k * kstride + cstep];
                    a0 = __builtin_amdgcn_mfma_f32_32x32x2f32(fa, fb0, a0, 0, 0, 0);
                    a1 = __builtin_amdgcn_mfma_f32_32x32x2f32(fa, fb1, a1, 0, 0, 0);
                }
            } else {
#pragma unroll 8
                for (int k = 0; k < B; k += 2) {
                    const float fa = xa[k * kstride], fb0 = xb[k * kstride];
                    a0 = __builtin_amdgcn_mfma_f32_32x32x2f32(fa, fb0, a0, 0, 0, 0);
                }
            }
            float s0 = 0.f, s1 = 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) { s0 += a0[r] * a0[r]; s1 += a1[r] * a1[r]; }
            return (rt == ct ? s0 : 2.f * s0) + 2.f * s1;
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

// eta = 2 / beta_W' with beta_W' = 2 ||A^T A||_F ||B D B^T||_F (Eq. 11), from the squared Frobenius
// norms of the parts of the two block-diagonal matrices (nA and nK partial sums).  One wave per
// workgroup evaluates the sums, every workgroup in the same fixed order (fp64), so all take the
// same step and no separate reduction launch is needed (one wave only: thousands of waves reading
// the same few cache lines at kernel start queue up on one L2 channel).  Call with a whole wave;
// publish_eta_W / read_eta_W move the value through LDS to the rest of the workgroup.
__device__ __forceinline__ float wave_eta_W(const float *__restrict__ fro2A, int nA, const float *__restrict__ fro2K,
                                            int nK) {
    const int lane = threadIdx.x & 63;
    // the first 256 values of each array are requested together: one memory round trip, not one per value
    float va[4], vk[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int e = lane + 64 * q; // clamped, unconditional loads: a lane-predicated load would wait for its own data
        va[q] = 0.f;
        vk[q] = 0.f;
        if (64 * q < nA) va[q] = fro2A[min(e, nA - 1)];
        if (64 * q < nK) vk[q] = fro2K[min(e, nK - 1)];
        if (e >= nA) va[q] = 0.f;
        if (e >= nK) vk[q] = 0.f;
    }
    double a = 0.0, k = 0.0;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        a += (double)va[q];
        k += (double)vk[q];
    }
    for (int e = lane + 256; e < nA; e += 64) a += (double)fro2A[e];
    for (int e = lane + 256; e < nK; e += 64) k += (double)fro2K[e];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        a += __shfl_xor(a, off, 64);
        k += __shfl_xor(k, off, 64);
    }
    const double bw = 2.0 * sqrt(a) * sqrt(k);
    const float eta = bw > 0.0 ? (float)(2.0 / bw) : 0.f;
    // every lane holds the same value: keep it in a scalar register like any other uniform
    return __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(eta)));
}

template <int B> struct Smem {
    float X[Chain<B>::TILE_FLOATS];
    float Y[Chain<B>::TILE_FLOATS];
    float Dl[B];
    float red[16];
    float eta;
};

template <class SM>
__device__ __forceinline__ void publish_eta_W(SM &sm, int tid, const float *__restrict__ fro2A, int nA,
                                              const float *__restrict__ fro2K, int nK) {
    if (tid < 64) { // wave 0; visible to the others after the next barrier
        const float e = wave_eta_W(fro2A, nA, fro2K, nK);
        if (tid == 0) sm.eta = e;
    }
}
template <class SM> __device__ __forceinline__ float read_eta_W(const SM &sm) {
    return __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(sm.eta))); // uniform: scalar register
}

} // namespace armor
