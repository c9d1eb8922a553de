// Per-block contraction chains at b = 128 with one operand resident in LDS and the other streamed
// from global memory straight into matrix-instruction fragments (same mathematics as chain.hip:
// Alg. 2 / App. D, Alg. 3's gradient; that file states what each phase computes).
//
// Why a second form.  With both operand tiles of a product staged in LDS (chain.hip) a workgroup
// holds 2 x 66 KB, so one workgroup owns a CU, and everything that is not a matrix instruction
// (LDS hand-over of a result, tile staging, barriers, the epilogue arithmetic, waiting for Wbar)
// leaves the matrix pipes idle.  Here only the operand that was just computed on the CU sits in LDS
// (66 KB); the other one comes from L2 / HBM as fragments: a lane asks for exactly the elements the
// matrix instruction wants from it, a few k-groups ahead of their use.  Two 256-thread workgroups
// then share a CU (2 x 75 KB of LDS, at most 256 VGPRs per wave), and one's epilogue runs
// underneath the other's products.  Nothing is staged, so a product has no barrier inside it.
//
// k-slot map.  v_mfma_f32_32x32x2_f32 takes from lane (x = lane % 32, h = lane / 32) the operand
// element (x, k-slot h) of the step.  Which k of the inner dimension a slot stands for is free as
// long as both operands agree.  Steps come in groups of four (8 inner indices); step i of group q
// gives lane half h the index k = 8 q + 4 h + i.  A lane of a k-contiguous operand then needs four
// consecutive floats per group: one 16-byte load.
#include "chain_common.h"

#include <algorithm>

namespace armor {

namespace stream { // (named: profilers print the kernels' names)

struct CfgStream { static constexpr int WM = 2, WN = 2, TM = 2, TN = 2; static constexpr bool SPLIT = false; };
constexpr int SB = 128;
using CS = Chain<SB, CfgStream>;
typedef float floatx4 __attribute__((ext_vector_type(4)));

// Matrix instruction of the products.  0: v_mfma_f32_32x32x2_f32 on the fp32 operands.  1: every fp32
// operand value is cut EXACTLY into three bf16 pieces (x = x1 + x2 + x3: the top 8 significant bits,
// the next 8, the last 8, by truncation) and a product x y is formed as the six partial products
// x1 y1 + x1 y2 + x2 y1 + x1 y3 + x2 y2 + x3 y1 on v_mfma_f32_32x32x16_bf16 (fp32 accumulation); the
// three dropped ones are below 2^-23 |x y|, the size of one fp32 rounding.  Sixteen inner indices
// then cost six 8-pass instructions instead of eight 16-pass ones.
#ifndef ARMOR_STREAM_BF16X3
#define ARMOR_STREAM_BF16X3 1
#endif
constexpr bool SPLIT_BF16 = ARMOR_STREAM_BF16X3 != 0;
// Workgroups per CU, and how far ahead (in groups of 8 inner indices) a product on the bf16 instruction
// requests its global operands: pre-cut wrapper pieces are used as they arrive (one pair of groups ahead);
// block data is cut one pair before it is used, so it is requested two pairs ahead.  (One workgroup per CU
// with all 512 registers and requests three to four pairs ahead measured 8 % slower: the second workgroup's
// products cover this one's epilogues.)
constexpr int SEQ_WGS = 2;
constexpr int SPLIT_DEPTH_PIECES = 2, SPLIT_DEPTH_DATA = 4;
struct SmemStream {
    float X[CS::TILE_FLOATS];
    float red[16];
    float eta;
    uint2 M[SB * 64 / 8]; // the block's mask bytes, rows of 64 bytes (at most one byte per two columns)
};

// Where an operand op(x, k) of a product lives (x: its row index for the left operand, its column
// index for the right one; k: the inner index):
enum class Src {
    GK, // global memory, k contiguous: g[x * ld + k]
    GX, // global memory, x contiguous: g[k * ld + x]
    LK, // LDS tile of pitch P, k contiguous: T[x * P + k]
    LX, // LDS tile of pitch P, x contiguous: T[k * P + x]
    GP, // global memory, a wrapper-sized matrix already cut into its three bf16 pieces (make_planes_kernel),
        // stored in the order the lanes ask for it: P[piece][run of 16 inner indices][lane half h][x][8], 16-bit
        // elements, the eight being k = 16 run + 4 h + i and 16 run + 8 + 4 h + i (i = 0..3): what lane (x, h)
        // supplies for that run.  One load instruction of a wave then reads two contiguous 512-byte stretches.
};
constexpr bool is_global(Src s) { return s == Src::GK || s == Src::GX || s == Src::GP; }

constexpr int NGROUP = SB / 8;

// One operand's fragments: f[q][i][t] for group q, step i, 32-wide tile t of this wave.  Indices are
// compile-time everywhere (the product is fully unrolled), so only the groups in flight hold registers.
template <Src S> struct Operand {
    const float *base;
    uint32_t lane; // byte offset (global) or float index (LDS) of this lane's element (x0, k = 4 h)
    uint32_t tile; // the same kind of offset from tile 0 to tile 1
    uint32_t ld4;  // bytes per k step (GX)
    float f[NGROUP][4][2];
    uintx4 pc[NGROUP / 2][3][2]; // GP: pieces of a pair of groups, [pair][piece][tile]

    __device__ __forceinline__ Operand(const float *b, int ld, int x0, int kh) : base(b) {
        if constexpr (S == Src::GK) { lane = opaque_u(4u * (uint32_t)(x0 * ld + 4 * kh)); tile = 4u * 32u * (uint32_t)ld; ld4 = 0; }
        if constexpr (S == Src::GX) { lane = opaque_u(4u * (uint32_t)(4 * kh * ld + x0)); tile = 4u * 32u; ld4 = 4u * (uint32_t)ld; }
        if constexpr (S == Src::LK) { lane = opaque_u((uint32_t)(x0 * CS::P + 4 * kh)); tile = 32u * CS::P; ld4 = 0; }
        if constexpr (S == Src::LX) { lane = opaque_u((uint32_t)(4 * kh * CS::P + x0)); tile = 32u; ld4 = 0; }
        if constexpr (S == Src::GP) { lane = opaque_u(16u * (uint32_t)(kh * SB + x0)); tile = 16u * 32u; ld4 = 0; }
    }
    // a quarter of group q's requests (part 0..3), or all of them (part < 0)
    __device__ __forceinline__ void request(int q, int part = -1) {
        if constexpr (S == Src::GP) { // one 16-byte load per piece and tile for the pair of groups (q, q + 1), q even
            if (q % 2 == 0) {
#pragma unroll
                for (int pi = 0; pi < 3; ++pi)
#pragma unroll
                    for (int t = 0; t < 2; ++t) {
                        if (part >= 0 && part != pi) continue;
                        pc[q / 2][pi][t] = gld(reinterpret_cast<const uintx4 *>(base),
                                               lane + t * tile + (uint32_t)pi * (2u * SB * SB) + (32u * SB) * (uint32_t)(q / 2));
                    }
            }
            return;
        }
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            if constexpr (S == Src::GK) {
                if (part >= 0 && part != t) continue;
                const floatx4 v = gld(reinterpret_cast<const floatx4 *>(base), lane + t * tile + 32u * q);
#pragma unroll
                for (int i = 0; i < 4; ++i) f[q][i][t] = v[i];
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    if (part >= 0 && part != i) continue;
                    if constexpr (S == Src::GX) f[q][i][t] = gld(base, lane + t * tile + (uint32_t)(8 * q + i) * ld4);
                    if constexpr (S == Src::LK) f[q][i][t] = base[lane + t * tile + 8 * q + i];
                    if constexpr (S == Src::LX) f[q][i][t] = base[lane + t * tile + (8 * q + i) * CS::P];
                }
            }
        }
    }
};

// acc (+)= opL * opR over the 128 inner indices; ZERO: acc = opL * opR (the first matrix instruction
// of every tile takes a zero C operand); NEGR: opR enters negated.  Global operands are requested
// DEPTH groups ahead (a group's matrix instructions take ~0.43 us per wave: 3 groups cover an L2
// hit; measured 2 and 3 alike, 4 and 5 slower; 2 leaves more registers), LDS operands one group ahead.
// tail() runs once, TAIL_BACK groups before the end: at or behind the product's last global request.
// Loads return in issue order, so a request that goes to HBM holds up every later one: what the
// caller wants from HBM next is asked for there and travels underneath the remaining matrix
// instructions and the hand-over that follows (a smaller TAIL_BACK when registers are short: fewer
// operand groups are still held).
constexpr int STREAM_DEPTH = 2;

struct NoTail {
    __device__ void operator()() const {}
};
// A product: begin() asks for the global operands' first groups, run() does the rest.  (Starting the
// requests of the next product in front of an epilogue's stores was measured: no gain.)
template <Src LS, Src RS> struct Product {
    static constexpr int DEPTH = STREAM_DEPTH;
    Operand<LS> l;
    Operand<RS> r;
    __device__ __forceinline__ Product(const float *L, int ldl, const float *R, int ldr, const CS::Pos &p)
        : l(L, ldl, p.wm0 + p.l32, p.kh), r(R, ldr, p.wn0 + p.l32, p.kh) {}
    // the global operands' first DEPTH groups
    __device__ __forceinline__ void begin() {
        if constexpr (SPLIT_BF16) {
#pragma unroll
            for (int q = 0; q < NGROUP; ++q) {
                if (is_global(LS) && q < depth_of(LS)) l.request(q);
                if (is_global(RS) && q < depth_of(RS)) r.request(q);
            }
            return;
        }
#pragma unroll
        for (int q = 0; q < DEPTH; ++q) {
            if constexpr (is_global(LS)) l.request(q);
            if constexpr (is_global(RS)) r.request(q);
        }
    }
    // The same product on the bf16 matrix instruction (see SPLIT_BF16), two groups (16 inner indices) per trip,
    // six rounds of four matrix instructions each (one per 32 x 32 tile of the wave's patch).  Cutting is plain
    // vector arithmetic, about four instructions per matrix instruction, and the matrix pipe is a separate
    // unit: the pieces of pair q + 1 are cut in rounds 2..5 of pair q, one instruction group between two
    // matrix instructions, so both units stay busy from one wave.  Block data from global memory is therefore
    // requested two pairs ahead (it is cut one pair ahead), pre-cut wrapper pieces one pair ahead, LDS operands
    // in rounds 0..1 of the pair before.
    static constexpr int depth_of(Src s) { return s == Src::GP ? SPLIT_DEPTH_PIECES : SPLIT_DEPTH_DATA; }
    static __device__ __forceinline__ void cut_pair(float a, float b, bool neg, uint32_t &o1, uint32_t &o2, uint32_t &o3) {
        if (neg) { a = -a; b = -b; }
        const uint32_t ua = __float_as_uint(a), ub = __float_as_uint(b);
        o1 = __builtin_amdgcn_perm(ub, ua, 0x07060302u);
        const float ra = a - __uint_as_float(ua & 0xffff0000u), rb = b - __uint_as_float(ub & 0xffff0000u);
        const uint32_t va = __float_as_uint(ra), vb = __float_as_uint(rb);
        o2 = __builtin_amdgcn_perm(vb, va, 0x07060302u);
        const float sa = ra - __uint_as_float(va & 0xffff0000u), sb = rb - __uint_as_float(vb & 0xffff0000u);
        o3 = __builtin_amdgcn_perm(__float_as_uint(sb), __float_as_uint(sa), 0x07060302u);
    }
    template <bool ZERO, bool NEGR, int TAIL_BACK, class Tail>
    __device__ __forceinline__ void run_split(CS::Acc &acc, Tail &&tail) {
        static_assert(NGROUP % 2 == 0, "groups are taken in pairs");
        static_assert(!(LS == Src::GP && RS == Src::GP), "one operand of a product is block data");
        constexpr bool CUT_L = LS != Src::GP, CUT_R = RS != Src::GP;
        constexpr bool NEG_L = NEGR && !CUT_R, NEG_R = NEGR && CUT_R; // a negated product negates a cut operand
        constexpr int DL = depth_of(LS), DR = depth_of(RS);
        constexpr int UNITS = (CUT_L ? 8 : 0) + (CUT_R ? 8 : 0), PER_ROUND = UNITS / 4; // (tile, element pair) units
        Pieces cl[2][2], cr[2][2]; // cut pieces, [pair parity][tile]
        // unit u of the pieces of pair q (groups q, q + 1)
        auto cut_unit = [&](int q, int u) {
            const int buf = (q / 2) & 1;
            if (CUT_L && u < 8) {
                const int t = u >> 2, e = u & 3;
                cut_pair(l.f[q + (2 * e) / 4][(2 * e) % 4][t], l.f[q + (2 * e + 1) / 4][(2 * e + 1) % 4][t], NEG_L,
                         cl[buf][t].p1[e], cl[buf][t].p2[e], cl[buf][t].p3[e]);
            } else {
                const int v = CUT_L ? u - 8 : u, t = v >> 2, e = v & 3;
                cut_pair(r.f[q + (2 * e) / 4][(2 * e) % 4][t], r.f[q + (2 * e + 1) / 4][(2 * e + 1) % 4][t], NEG_R,
                         cr[buf][t].p1[e], cr[buf][t].p2[e], cr[buf][t].p3[e]);
            }
        };
        if constexpr (!is_global(LS)) { l.request(0); l.request(1); }
        if constexpr (!is_global(RS)) { r.request(0); r.request(1); }
#pragma unroll
        for (int u = 0; u < UNITS; ++u) cut_unit(0, u);
#pragma unroll
        for (int q = 0; q < NGROUP; q += 2) {
            const int buf = (q / 2) & 1;
            constexpr int NC = 6;
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                // requests of later pairs, spread over the rounds
                if (c < 4) {
#pragma unroll
                    for (int g = 0; g < 2; ++g) {
                        if (is_global(LS) && q + g + DL < NGROUP) l.request(q + g + DL, c);
                        if (is_global(RS) && q + g + DR < NGROUP) r.request(q + g + DR, c);
                    }
                }
                if (c < 2 && q + 2 < NGROUP) { // LDS operands of the next pair: half of each group per round
#pragma unroll
                    for (int g = 0; g < 2; ++g)
#pragma unroll
                        for (int part = 2 * c; part < 2 * c + 2; ++part) {
                            if constexpr (!is_global(LS)) l.request(q + g + 2, part);
                            if constexpr (!is_global(RS)) r.request(q + g + 2, part);
                        }
                }
                if (c == NC - 1 && q <= NGROUP - 1 - TAIL_BACK && q + 2 > NGROUP - 1 - TAIL_BACK) tail();
                // the next pair's pieces
                if (c >= 2 && q + 2 < NGROUP) {
#pragma unroll
                    for (int u = (c - 2) * PER_ROUND; u < (c - 1) * PER_ROUND; ++u) cut_unit(q + 2, u);
                }
#pragma unroll
                for (int tm = 0; tm < 2; ++tm)
#pragma unroll
                    for (int tn = 0; tn < 2; ++tn) {
                        // small partial products first: (3,1) (1,3) (2,2) (2,1) (1,2) (1,1)
                        uintx4 a, b;
                        if constexpr (CUT_L) a = c == 0 ? vec4(cl[buf][tm].p3) : (c == 2 || c == 3) ? vec4(cl[buf][tm].p2) : vec4(cl[buf][tm].p1);
                        else a = l.pc[q / 2][c == 0 ? 2 : (c == 2 || c == 3) ? 1 : 0][tm];
                        if constexpr (CUT_R) b = c == 1 ? vec4(cr[buf][tn].p3) : (c == 2 || c == 4) ? vec4(cr[buf][tn].p2) : vec4(cr[buf][tn].p1);
                        else b = r.pc[q / 2][c == 1 ? 2 : (c == 2 || c == 4) ? 1 : 0][tn];
                        if (ZERO && q == 0 && c == 0) {
                            const floatx16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                            acc.v[tm][tn] = mfma_bf16(a, b, zero);
                        } else {
                            acc.v[tm][tn] = mfma_bf16(a, b, acc.v[tm][tn]);
                        }
                    }
                // issue order inside the round: a matrix instruction, then a share of the vector and memory
                // instructions, four times
#pragma unroll
                for (int m = 0; m < 4; ++m) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                         // one matrix instruction
                    __builtin_amdgcn_sched_group_barrier(0x002, (11 * PER_ROUND + 3) / 4, 0);  // vector arithmetic
                    __builtin_amdgcn_sched_group_barrier(0x120, 4, 0);                         // memory / LDS reads
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }
    template <bool ZERO, bool NEGR = false, int TAIL_BACK = STREAM_DEPTH, class Tail = NoTail>
    __device__ __forceinline__ void run(CS::Acc &acc, Tail &&tail = Tail()) {
        if constexpr (SPLIT_BF16) {
            run_split<ZERO, NEGR, TAIL_BACK>(acc, tail);
            return;
        }
        if constexpr (!is_global(LS)) l.request(0);
        if constexpr (!is_global(RS)) r.request(0);
#pragma unroll
        for (int q = 0; q < NGROUP; ++q) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if (q + DEPTH < NGROUP) {
                    if constexpr (is_global(LS)) l.request(q + DEPTH, i);
                    if constexpr (is_global(RS)) r.request(q + DEPTH, i);
                }
                if (i == 3 && q == NGROUP - 1 - TAIL_BACK) tail();
                if (q + 1 < NGROUP) {
                    if constexpr (!is_global(LS)) l.request(q + 1, i);
                    if constexpr (!is_global(RS)) r.request(q + 1, i);
                }
                // A quarter of a later group's requests, then one step's matrix instructions: the requests
                // issue while the matrix pipe works off the step before (measured 3 % faster than whole groups
                // of requests in front of whole groups of matrix instructions).  The fences keep that order:
                // left alone, the scheduler sinks the requests to just in front of their first use.
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int tm = 0; tm < 2; ++tm)
#pragma unroll
                    for (int tn = 0; tn < 2; ++tn) {
                        const float rv = NEGR ? -r.f[q][i][tn] : r.f[q][i][tn];
                        if (ZERO && q == 0 && i == 0) {
                            const floatx16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                            acc.v[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x2f32(l.f[q][i][tm], rv, zero, 0, 0, 0);
                        } else {
                            acc.v[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x2f32(l.f[q][i][tm], rv, acc.v[tm][tn], 0, 0, 0);
                        }
                    }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }
};

template <Src LS, Src RS, bool ZERO, bool NEGR = false, int TAIL_BACK = STREAM_DEPTH, class Tail = NoTail>
__device__ __forceinline__ void mma_stream(CS::Acc &acc, const float *L, int ldl, const float *R, int ldr,
                                           const CS::Pos &p, Tail &&tail = Tail()) {
    Product<LS, RS> pr(L, ldl, R, ldr, p);
    pr.begin();
    pr.template run<ZERO, NEGR, TAIL_BACK>(acc, tail);
}

// A reduction variable is evaluated where this stands.  Without it the compiler is free to form the
// sum where it is used, after later products, and keeps every addend in a register until then.
__device__ __forceinline__ void settle(float &v) { asm volatile("" : "+v"(v)); }

// A wrapper-sized operand (A^i, B^j, K^j, A^iT A^i: shared by a whole row or column of blocks) is cut into
// its bf16 pieces once per iteration by make_planes_kernel and streamed as pieces; block data is cut where
// it is used.  With the fp32 matrix instruction the same operand is streamed as fp32.
template <Src FP32_FORM> constexpr Src wrapper_src() { return SPLIT_BF16 ? Src::GP : FP32_FORM; }
__device__ __forceinline__ const float *wrapper_ptr(const float *fp32, const uint16_t *planes, int blk) {
    if constexpr (SPLIT_BF16) return reinterpret_cast<const float *>(planes + (int64_t)blk * 3 * SB * SB);
    else return fp32 + (int64_t)blk * SB * SB;
}

// X [nblk][128][128] fp32 -> P = pieces of op(x, k) = X[x][k] (k = column: stands in for the GK form) and
// PT = pieces of op(x, k) = X[k][x] (k = row: the GX form; optional), both in the GP layout.
// Workgroup (blk, 32 values of x); thread -> (x, run of 16 inner indices), x fastest so stores are contiguous.
// Up to three matrices per launch (blockIdx.x runs over all their blocks).
struct PlaneJobs {
    const float *X[3];
    uint16_t *P[3], *PT[3];
    int first[4]; // first[j] .. first[j + 1]: the blocks of job j
};
__global__ __launch_bounds__(256) void make_planes_kernel(PlaneJobs jobs) {
    const int tid = threadIdx.x;
    const int job = (int)blockIdx.x >= jobs.first[2] ? 2 : ((int)blockIdx.x >= jobs.first[1] ? 1 : 0);
    const int blk = blockIdx.x - jobs.first[job];
    const float *__restrict__ X = jobs.X[job];
    uint16_t *__restrict__ P = jobs.P[job], *__restrict__ PT = jobs.PT[job];
    const int x = 32 * blockIdx.y + (tid & 31), run = tid >> 5;
    const float *Xb = X + (int64_t)blk * SB * SB;
    auto emit = [&](uint16_t *out, const float (&v)[16]) { plane_emit(out + (int64_t)blk * 3 * SB * SB, run, x, v); };
    float v[16];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const floatx4 q = *reinterpret_cast<const floatx4 *>(Xb + x * SB + 16 * run + 4 * e);
        v[4 * e] = q[0]; v[4 * e + 1] = q[1]; v[4 * e + 2] = q[2]; v[4 * e + 3] = q[3];
    }
    emit(P, v);
    if (PT != nullptr) {
#pragma unroll
        for (int e = 0; e < 16; ++e) v[e] = Xb[(16 * run + e) * SB + x];
        emit(PT, v);
    }
}

// ------------------------------------------------------------------------------------------------
// W' step fused with the core gradient at the updated core (see phase_WS_kernel in chain.hip for the
// identities).  Per block, with S' = A C handed over by the B step:
//   R = Wbar - S' B      both operands streamed (S' k-contiguous, B^j column-contiguous); Wbar is
//                        loaded into the accumulator and the product runs as Wbar + S' (-B)
//   U = (R D) B^T        R D resident, B^j streamed k-contiguous
//   G = A^T U            U resident, A^i streamed row-contiguous
//   V = Delta K          Delta = G (.) M resident, K^j streamed
//   Z = (A^T A) V        V resident, A^T A streamed
// FUSED = false stops after the W' step itself (unstructured mode, where no sparse-core step follows).
// ------------------------------------------------------------------------------------------------
template <bool FUSED>
__global__ __launch_bounds__(CS::NT, SEQ_WGS) void phase_WS_stream_kernel(
    const float *__restrict__ Wbar, float *__restrict__ C, const float *__restrict__ A,
    const float *__restrict__ Bw, const float *__restrict__ D, const float *__restrict__ AtA,
    const float *__restrict__ K, const uint8_t *__restrict__ mask, int mask_group,
    const float *__restrict__ fro2A, int nA, const float *__restrict__ fro2K, int nK, int64_t d_in, int nbj,
    int nblocks, float *__restrict__ Gout, float *__restrict__ loss_part, const float *__restrict__ Sp,
    WrapperPlanes pl) {
    constexpr int B = SB;
    __shared__ SmemStream sm;
    const int tid = threadIdx.x;
    const CS::Pos p(tid);
    const int ldw = (int)d_in;
    const uint32_t wboff = p.lane_boff(ldw);
    const int64_t mrow = d_in / mask_group;
    CS::Acc acc, acc2;
    publish_eta_W(sm, tid, fro2A, nA, fro2K, nK);
    __syncthreads();
    const float eta2 = read_eta_W(sm);
    const int nb = B / mask_group; // mask bytes per block row: 16, 32 or 64
    const uint32_t mhalf = (uint32_t)((tid >> 1) * 64 + (tid & 1) * (nb >> 1));
    // Wbar of a block and its mask bytes (thread t: half of row t / 2, 8 bytes at a time) are requested
    // at the end of the block before.  Wbar lands in the accumulator of the block's first product: no
    // second set of registers holds it.  The mask bytes wait in LDS for the W' step.
    CS::Acc accw;
    uint2 mreg[4];
    auto request_block = [&](int blk) {
        const int i = blk / nbj, j = blk % nbj;
        const float *Wij = Wbar + (int64_t)i * B * d_in + (int64_t)j * B;
        const uint8_t *mb = mask + (int64_t)i * B * mrow + (int64_t)j * nb;
        const uint32_t mo = (uint32_t)((tid >> 1) * (int)mrow + (tid & 1) * (nb >> 1));
        const uint32_t lb = opaque_u(wboff);
#pragma unroll
        for (int it = 0; it < 4; ++it)
            if (it * 16 < nb) mreg[it] = gld(reinterpret_cast<const uint2 *>(mb), mo + 8u * it);
#pragma unroll
        for (int tm = 0; tm < 2; ++tm)
#pragma unroll
            for (int tn = 0; tn < 2; ++tn)
#pragma unroll
                for (int r = 0; r < 16; ++r) accw.v[tm][tn][r] = gld(Wij, lb + CS::Pos::unif_boff(tm, tn, r, ldw));
    };
    if ((int)blockIdx.x < nblocks) request_block(blockIdx.x);
    for (int blk = blockIdx.x; blk < nblocks; blk += gridDim.x) {
        const int i = blk / nbj, j = blk % nbj;
        float *Cij = C + (int64_t)i * B * d_in + (int64_t)j * B;
        const float *Sij = Sp + (int64_t)i * B * d_in + (int64_t)j * B;
        const float *Dj = D + (int64_t)j * B;
        float lsum = 0.f;
        mma_stream<Src::GK, wrapper_src<Src::GX>(), false, true>(accw, Sij, ldw, wrapper_ptr(Bw, pl.BT, j), B, p); // R = Wbar - S' B
#pragma unroll
        for (int tn = 0; tn < 2; ++tn) {
            const float dj = Dj[p.col(tn)];
#pragma unroll
            for (int tm = 0; tm < 2; ++tm)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float res = accw.v[tm][tn][r];
                    lsum += res * res * dj;
                    accw.v[tm][tn][r] = res * dj;
                }
        }
        settle(lsum);
        // (a product's first wrapper pieces are asked for in front of the hand-over that precedes it: they travel
        // underneath the LDS stores and the barrier)
        Product<Src::LK, wrapper_src<Src::GK>()> prU(sm.X, 0, wrapper_ptr(Bw, pl.B, j), B, p);
        prU.begin();
        CS::store_acc(sm.X, accw, p); // R D   (the previous block is done with X and M: barriers at its end)
#pragma unroll
        for (int it = 0; it < 4; ++it)
            if (it * 16 < nb) *reinterpret_cast<uint2 *>(reinterpret_cast<char *>(sm.M) + mhalf + 8u * it) = mreg[it];
        __syncthreads();
        prU.template run<true>(acc); // U = (R D) B^T
        Product<wrapper_src<Src::GX>(), Src::LX> prG(wrapper_ptr(A, pl.AT, i), B, sm.X, 0, p);
        prG.begin();
        __syncthreads();
        CS::store_acc(sm.X, acc, p);
        __syncthreads();
        // current core values in the accumulator layout, requested behind the product's last operands
        float cv[2][2][16];
        prG.template run<true, false, STREAM_DEPTH>(acc, [&]() { // G = A^T U   (stays in acc)
            const uint32_t lb = opaque_u(wboff);
#pragma unroll
            for (int tm = 0; tm < 2; ++tm)
#pragma unroll
                for (int tn = 0; tn < 2; ++tn)
#pragma unroll
                    for (int r = 0; r < 16; ++r) cv[tm][tn][r] = gld(Cij, lb + CS::Pos::unif_boff(tm, tn, r, ldw));
        });
        __syncthreads();
        // W' step on kept entries; Delta = G (.) M goes to LDS for the two extra products
        uint32_t keep[2][2];
        float dd = 0.f;
        {
            float *d0 = sm.X + opaque(p.lane_off(CS::P));
            const uint32_t lb = opaque_u(wboff);
            const uint8_t *ml = reinterpret_cast<const uint8_t *>(sm.M);
#pragma unroll
            for (int tn = 0; tn < 2; ++tn) {
                const uint32_t mo = opaque_u((uint32_t)((p.wm0 + p.kh * 4) * 64 + p.col(tn) / mask_group));
                const int sh = p.col(tn) % mask_group;
#pragma unroll
                for (int tm = 0; tm < 2; ++tm) {
                    keep[tm][tn] = 0u;
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const uint32_t mbyte = ml[mo + (uint32_t)((tm * 32 + (r >> 2) * 8 + (r & 3)) * 64)];
                        const bool kp = (mbyte >> sh) & 1u;
                        keep[tm][tn] |= (kp ? 1u : 0u) << r;
                        const float dl = kp ? acc.v[tm][tn][r] : 0.f;
                        if (FUSED) {
                            dd += dl * dl;
                            d0[CS::Pos::unif_off(tm, tn, r, CS::P)] = dl;
                        }
                        // (pruned entries are written back as they were: no branch around the store, same lines)
                        gst(Cij, lb + CS::Pos::unif_boff(tm, tn, r, ldw), cv[tm][tn][r] + eta2 * dl);
                    }
                    keep[tm][tn] = opaque_u(keep[tm][tn]); // the masked values themselves are not kept in registers
                }
            }
        }
        if constexpr (!FUSED) {
            request_block(min(blk + (int)gridDim.x, nblocks - 1));
            __syncthreads(); // X and M are free again
            continue;
        }
        settle(dd);
        Product<Src::LK, wrapper_src<Src::GX>()> prV(sm.X, 0, wrapper_ptr(K, pl.K, j), B, p);
        prV.begin();
        __syncthreads();
        prV.template run<true>(acc2); // V = Delta K
        Product<wrapper_src<Src::GK>(), Src::LX> prZ(wrapper_ptr(AtA, pl.AtA, i), B, sm.X, 0, p);
        prZ.begin();
        __syncthreads();
        CS::store_acc(sm.X, acc2, p);
        __syncthreads();
        prZ.template run<true>(acc2); // Z = (A^T A) V
        request_block(min(blk + (int)gridDim.x, nblocks - 1)); // (the last block asks for itself again: harmless)
        float dz = 0.f;
        {
            float *Gij = Gout + (int64_t)i * B * d_in + (int64_t)j * B;
            const uint32_t lb = opaque_u(wboff);
#pragma unroll
            for (int tm = 0; tm < 2; ++tm)
#pragma unroll
                for (int tn = 0; tn < 2; ++tn)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const float g = acc.v[tm][tn][r], z = acc2.v[tm][tn][r];
                        if ((keep[tm][tn] >> r) & 1u) dz += g * z;
                        gst(Gij, lb + CS::Pos::unif_boff(tm, tn, r, ldw), -2.f * (g - eta2 * z));
                    }
        }
        float ltot = CS::block_sum(lsum - 2.f * eta2 * dd + eta2 * eta2 * dz, sm.red, tid); // (barriers: X is free again)
        if (tid == 0) loss_part[blk] = ltot;
    }
}

// deterministic workgroup-wide sums of two values at once; results valid in thread 0
__device__ __forceinline__ void block_sum2(float &a, float &b, float *red, int tid) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        a += __shfl_xor(a, off, 64);
        b += __shfl_xor(b, off, 64);
    }
    __syncthreads();
    if ((tid & 63) == 0) { red[tid >> 6] = a; red[8 + (tid >> 6)] = b; }
    __syncthreads();
    if (tid == 0) {
        a = 0.f; b = 0.f;
        for (int w = 0; w < CS::NW; ++w) { a += red[w]; b += red[8 + w]; }
    }
}

__device__ __forceinline__ float frob2(const CS::Acc &acc) {
    float f2 = 0.f;
#pragma unroll
    for (int tm = 0; tm < 2; ++tm)
#pragma unroll
        for (int tn = 0; tn < 2; ++tn)
#pragma unroll
            for (int r = 0; r < 16; ++r) f2 += acc.v[tm][tn][r] * acc.v[tm][tn][r];
    return f2;
}

// Squared Frobenius norm of the symmetric product X X^T (XT = false) or X^T X (XT = true) of the
// resident tile, as this lane's share of the sum: only the 10 upper-triangular 32 x 32 tiles of the
// 4 x 4 grid are formed, off-diagonal ones counted twice.  Both operands of a tile are 32-row slices of
// the same matrix, so a wave cuts each slice it needs once per 16 inner indices and uses it on either side:
//   wave 0: slices 0, 1    -> tiles (0,0) (0,1) (1,1)        wave 2: slices 0, 2, 3 -> tiles (0,2) (0,3)
//   wave 1: slices 2, 3    -> tiles (2,2) (2,3) (3,3)        wave 3: slices 1, 2, 3 -> tiles (1,2) (1,3)
// (three tiles from two slices, or two tiles from three: 18 / 12 matrix instructions and 88 / 132 cutting
// instructions per 16 inner indices).  `flip` swaps the two kinds (callers pass it for the second half of
// the grid, which is what lands in the CUs' second slots), so that the two workgroups of a CU put their
// heavy waves on different SIMDs.  Both operands come from LDS: no global request is outstanding behind
// this.  The slices of the next 16 inner indices are read and cut underneath the current matrix instructions.
template <bool XT> __device__ __forceinline__ float sym_frob2_stream(const float *X, const CS::Pos &p, int tid, bool flip) {
    const int w = (tid >> 6) ^ (flip ? 2 : 0);
    const int xs = XT ? 1 : CS::P, ks = XT ? CS::P : 1; // strides of the slice row index and of k
    const float *base = X + p.l32 * xs;
    if constexpr (SPLIT_BF16) {
        const bool tri = w < 2;                       // triangle on two slices, or a row of two tiles on three
        const int s0 = tri ? 2 * w : w - 2, s1 = tri ? 2 * w + 1 : 2, s2 = 3;
        const float *sl[3] = {base + 32 * s0 * xs, base + 32 * s1 * xs, base + 32 * s2 * xs};
        floatx16 t0, t1, t2;
#pragma unroll
        for (int r = 0; r < 16; ++r) { t0[r] = 0.f; t1[r] = 0.f; t2[r] = 0.f; }
        float raw[2][3][8];
        Pieces pc[2][3];
        // lane half h supplies indices 16 kb + 8 h .. + 7 of every slice
        auto read = [&](int kb, int g) {
#pragma unroll
            for (int e = 0; e < 8; ++e) raw[kb & 1][g][e] = sl[g][(16 * kb + 8 * p.kh + e) * ks];
        };
        auto six = [&](floatx16 &t, const Pieces &a, const Pieces &b) {
            t = mfma_bf16(vec4(a.p3), vec4(b.p1), t);
            t = mfma_bf16(vec4(a.p1), vec4(b.p3), t);
            t = mfma_bf16(vec4(a.p2), vec4(b.p2), t);
            t = mfma_bf16(vec4(a.p2), vec4(b.p1), t);
            t = mfma_bf16(vec4(a.p1), vec4(b.p2), t);
            t = mfma_bf16(vec4(a.p1), vec4(b.p1), t);
        };
        if (tri) {
            read(0, 0); read(0, 1);
            cut3(raw[0][0], pc[0][0]); cut3(raw[0][1], pc[0][1]);
            read(1, 0); read(1, 1);
#pragma unroll
            for (int kb = 0; kb < SB / 16; ++kb) {
                const int cur = kb & 1, nxt = cur ^ 1;
                if (kb + 1 < SB / 16) { cut3(raw[nxt][0], pc[nxt][0]); cut3(raw[nxt][1], pc[nxt][1]); }
                if (kb + 2 < SB / 16) { read(kb + 2, 0); read(kb + 2, 1); }
                six(t0, pc[cur][0], pc[cur][0]);
                six(t1, pc[cur][0], pc[cur][1]);
                six(t2, pc[cur][1], pc[cur][1]);
#pragma unroll
                for (int m = 0; m < 18; ++m) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x002, 5, 0);
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        } else {
            read(0, 0); read(0, 1); read(0, 2);
            cut3(raw[0][0], pc[0][0]); cut3(raw[0][1], pc[0][1]); cut3(raw[0][2], pc[0][2]);
            read(1, 0); read(1, 1); read(1, 2);
#pragma unroll
            for (int kb = 0; kb < SB / 16; ++kb) {
                const int cur = kb & 1, nxt = cur ^ 1;
                if (kb + 1 < SB / 16) { cut3(raw[nxt][0], pc[nxt][0]); cut3(raw[nxt][1], pc[nxt][1]); cut3(raw[nxt][2], pc[nxt][2]); }
                if (kb + 2 < SB / 16) { read(kb + 2, 0); read(kb + 2, 1); read(kb + 2, 2); }
                six(t0, pc[cur][0], pc[cur][1]);
                six(t1, pc[cur][0], pc[cur][2]);
#pragma unroll
                for (int m = 0; m < 12; ++m) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x002, 11, 0);
                    __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        float q0 = 0.f, q1 = 0.f, q2 = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) { q0 += t0[r] * t0[r]; q1 += t1[r] * t1[r]; q2 += t2[r] * t2[r]; }
        // triangle: two diagonal tiles and one off-diagonal; row: two off-diagonal tiles (t2 stays zero)
        return tri ? q0 + 2.f * q1 + q2 : 2.f * (q0 + q1);
    } else {
        // wave -> tiles (row tile, column tile): w0 (0,0)(0,1)(1,1), w1 (0,2)(0,3)(1,2), w2 (1,3)(2,3), w3 (2,2)(3,3)
        const int r0 = w == 0 ? 0 : w == 1 ? 0 : w == 2 ? 1 : 2, c0 = w == 0 ? 0 : w == 1 ? 2 : w == 2 ? 3 : 2;
        const int r1 = w == 0 ? 0 : w == 1 ? 0 : w == 2 ? 2 : 3, c1 = w == 0 ? 1 : w == 1 ? 3 : 3;
        const int r2 = 1, c2 = w == 0 ? 1 : 2;
        const bool three = w < 2;
        const float *bk = base + p.kh * ks;
        const float *a0 = bk + 32 * r0 * xs, *b0 = bk + 32 * c0 * xs;
        const float *a1 = bk + 32 * r1 * xs, *b1 = bk + 32 * c1 * xs;
        const float *a2 = bk + 32 * r2 * xs, *b2 = bk + 32 * c2 * xs;
        floatx16 t0, t1, t2;
#pragma unroll
        for (int r = 0; r < 16; ++r) { t0[r] = 0.f; t1[r] = 0.f; t2[r] = 0.f; }
        if (three) {
#pragma unroll 8
            for (int k = 0; k < SB; k += 2) {
                t0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a0[k * ks], b0[k * ks], t0, 0, 0, 0);
                t1 = __builtin_amdgcn_mfma_f32_32x32x2f32(a1[k * ks], b1[k * ks], t1, 0, 0, 0);
                t2 = __builtin_amdgcn_mfma_f32_32x32x2f32(a2[k * ks], b2[k * ks], t2, 0, 0, 0);
            }
        } else {
#pragma unroll 8
            for (int k = 0; k < SB; k += 2) {
                t0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a0[k * ks], b0[k * ks], t0, 0, 0, 0);
                t1 = __builtin_amdgcn_mfma_f32_32x32x2f32(a1[k * ks], b1[k * ks], t1, 0, 0, 0);
            }
        }
        float s0 = 0.f, s1 = 0.f, s2 = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) { s0 += t0[r] * t0[r]; s1 += t1[r] * t1[r]; s2 += t2[r] * t2[r]; }
        return (r0 == c0 ? s0 : 2.f * s0) + (r1 == c1 ? s1 : 2.f * s1) + (r2 == c2 ? s2 : 2.f * s2);
    }
}

struct SmemGrad {
    float X[CS::TILE_FLOATS];
    float red[16];
};

// ------------------------------------------------------------------------------------------------
// A-phase (see phase_A_kernel in chain.hip).  Per block:
//   S sqrt(D) = (C B) sqrt(D)        both operands streamed; result resident
//   R sqrt(D) = Wbar sqrt(D) - A (S sqrt D)    A^i streamed; Wbar, scaled, is the accumulator's start
//   gacc += (R sqrt D)(S sqrt D)^T   R sqrt(D) goes through the workgroup's 64 KB of global scratch
//                                    (it stays in L2) and comes back as the streamed operand
//   || (S sqrt D)(S sqrt D)^T ||_F   both operands resident
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(CS::NT, SEQ_WGS) void phase_A_stream_kernel(
    const float *__restrict__ Wbar, const float *__restrict__ C, const float *__restrict__ A,
    const float *__restrict__ Bw, const float *__restrict__ D, int64_t d_in, int nbj, int nsplit,
    float *__restrict__ gpart, float *__restrict__ beta_part, float *__restrict__ loss_part,
    float *__restrict__ scratch, WrapperPlanes pl) {
    constexpr int B = SB;
    __shared__ SmemGrad sm;
    const int tid = threadIdx.x;
    const CS::Pos p(tid);
    const int ldw = (int)d_in;
    const uint32_t wboff = p.lane_boff(ldw);
    const int i = blockIdx.x / nsplit, c = blockIdx.x % nsplit;
    const int chunk = (nbj + nsplit - 1) / nsplit;
    const int j0 = c * chunk, j1 = min(nbj, j0 + chunk);
    float *sc = scratch + (int64_t)blockIdx.x * B * B;
    const float *Ai = wrapper_ptr(A, pl.A, i);
    CS::Acc gacc, acc, accw;
    gacc.zero();
    float *gp = gpart + (int64_t)blockIdx.x * B * B;
    const uint32_t gb = p.lane_boff(B);
    for (int j = j0; j < j1; ++j) {
        const float *Cij = C + (int64_t)i * B * d_in + (int64_t)j * B;
        const float *Wij = Wbar + (int64_t)i * B * d_in + (int64_t)j * B;
        const float *Bj = wrapper_ptr(Bw, pl.BT, j);
        const bool first = j == j0;
        auto reqW = [&]() {
            const uint32_t lb = opaque_u(wboff);
#pragma unroll
            for (int tm = 0; tm < 2; ++tm)
#pragma unroll
                for (int tn = 0; tn < 2; ++tn)
#pragma unroll
                    for (int r = 0; r < 16; ++r) accw.v[tm][tn][r] = gld(Wij, lb + CS::Pos::unif_boff(tm, tn, r, ldw));
        };
        mma_stream<Src::GK, wrapper_src<Src::GX>(), true, false, STREAM_DEPTH>(acc, Cij, ldw, Bj, B, p, reqW); // S = C B; Wbar requested behind it
        float sq[2];
#pragma unroll
        for (int tn = 0; tn < 2; ++tn) {
            sq[tn] = sqrtf(D[(int64_t)j * B + p.col(tn)]);
#pragma unroll
            for (int tm = 0; tm < 2; ++tm)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc.v[tm][tn][r] *= sq[tn];
        }
        CS::store_acc(sm.X, acc, p); // S sqrt(D)   (the previous block is done with X: barriers at its end)
        __syncthreads();
#pragma unroll
        for (int tn = 0; tn < 2; ++tn)
#pragma unroll
            for (int tm = 0; tm < 2; ++tm)
#pragma unroll
                for (int r = 0; r < 16; ++r) accw.v[tm][tn][r] *= sq[tn];
        mma_stream<wrapper_src<Src::GK>(), Src::LX, false, true>(accw, Ai, B, sm.X, 0, p); // R sqrt(D)
        float lsum = frob2(accw);
        settle(lsum);
        {
            const uint32_t lb = opaque_u(gb);
#pragma unroll
            for (int tm = 0; tm < 2; ++tm)
#pragma unroll
                for (int tn = 0; tn < 2; ++tn)
#pragma unroll
                    for (int r = 0; r < 16; ++r) gst(sc, lb + CS::Pos::unif_boff(tm, tn, r, B), accw.v[tm][tn][r]);
        }
        __syncthreads(); // scratch written by the whole workgroup (same CU, same L1: in order)
        mma_stream<Src::GK, Src::LK, false>(gacc, sc, B, sm.X, 0, p); // += (R sqrt D)(S sqrt D)^T
        float f2 = sym_frob2_stream<false>(sm.X, p, tid, 2 * blockIdx.x >= gridDim.x); // || (S sqrt D)(S sqrt D)^T ||_F^2
        block_sum2(lsum, f2, sm.red, tid); // (barriers: X and the scratch are free again)
        if (tid == 0) {
            loss_part[i * nbj + j] = lsum;
            beta_part[i * nbj + j] = sqrtf(f2);
        }
    }
    const uint32_t lb = opaque_u(gb);
#pragma unroll
    for (int tm = 0; tm < 2; ++tm)
#pragma unroll
        for (int tn = 0; tn < 2; ++tn)
#pragma unroll
            for (int r = 0; r < 16; ++r) gst(gp, lb + CS::Pos::unif_boff(tm, tn, r, B), -2.f * gacc.v[tm][tn][r]);
}

// ------------------------------------------------------------------------------------------------
// B-phase (see phase_B_kernel in chain.hip).  Per block:
//   S' = A C                     both operands streamed; result resident, and written out for the W' step
//   R D = (Wbar - S' B) D        B^j streamed; Wbar is the accumulator's start
//   gacc += S'^T (R D)           R D through the workgroup's global scratch
//   || S'^T S' ||_F              both operands resident
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(CS::NT, SEQ_WGS) void phase_B_stream_kernel(
    const float *__restrict__ Wbar, const float *__restrict__ C, const float *__restrict__ A,
    const float *__restrict__ Bw, const float *__restrict__ D, int64_t d_in, int nbi, int nbj, int nsplit,
    float *__restrict__ gpart, float *__restrict__ beta_part, float *__restrict__ Sp,
    float *__restrict__ scratch, WrapperPlanes pl) {
    constexpr int B = SB;
    __shared__ SmemGrad sm;
    const int tid = threadIdx.x;
    const CS::Pos p(tid);
    const int ldw = (int)d_in;
    const uint32_t wboff = p.lane_boff(ldw);
    const int j = blockIdx.x / nsplit, c = blockIdx.x % nsplit;
    const int chunk = (nbi + nsplit - 1) / nsplit;
    const int i0 = c * chunk, i1 = min(nbi, i0 + chunk);
    float *sc = scratch + (int64_t)blockIdx.x * B * B;
    const float *Bj = wrapper_ptr(Bw, pl.BT, j), *Dj = D + (int64_t)j * B;
    float dj[2];
#pragma unroll
    for (int tn = 0; tn < 2; ++tn) dj[tn] = Dj[p.col(tn)];
    float dn2 = 0.f;
    if (tid == 0)
        for (int q = 0; q < B; ++q) dn2 += Dj[q] * Dj[q];
    CS::Acc gacc, acc, accw;
    gacc.zero();
    float *gp = gpart + (int64_t)blockIdx.x * B * B;
    const uint32_t gb = p.lane_boff(B);
    for (int i = i0; i < i1; ++i) {
        const float *Cij = C + (int64_t)i * B * d_in + (int64_t)j * B;
        const float *Wij = Wbar + (int64_t)i * B * d_in + (int64_t)j * B;
        const float *Ai = wrapper_ptr(A, pl.A, i);
        const bool first = i == i0;
        auto reqW = [&]() {
            const uint32_t lb = opaque_u(wboff);
#pragma unroll
            for (int tm = 0; tm < 2; ++tm)
#pragma unroll
                for (int tn = 0; tn < 2; ++tn)
#pragma unroll
                    for (int r = 0; r < 16; ++r) accw.v[tm][tn][r] = gld(Wij, lb + CS::Pos::unif_boff(tm, tn, r, ldw));
        };
        mma_stream<wrapper_src<Src::GK>(), Src::GX, true, false, STREAM_DEPTH>(acc, Ai, B, Cij, ldw, p, reqW); // S' = A C; Wbar requested behind it
        CS::store_acc(sm.X, acc, p); // (the previous block is done with X: barriers at its end)
        __syncthreads();
        mma_stream<Src::LK, wrapper_src<Src::GX>(), false, true>(accw, sm.X, 0, Bj, B, p); // R = Wbar - S' B
        {
            const uint32_t lb = opaque_u(gb);
#pragma unroll
            for (int tm = 0; tm < 2; ++tm)
#pragma unroll
                for (int tn = 0; tn < 2; ++tn)
#pragma unroll
                    for (int r = 0; r < 16; ++r) gst(sc, lb + CS::Pos::unif_boff(tm, tn, r, B), accw.v[tm][tn][r] * dj[tn]); // R D
        }
        __syncthreads(); // scratch written by the whole workgroup (same CU, same L1: in order)
        mma_stream<Src::LX, Src::GX, false>(gacc, sm.X, 0, sc, B, p); // += S'^T (R D)
        // A and C do not change until the W' step: that step takes S' from here.  Stores complete in
        // issue order with the loads, so S' leaves from its LDS copy here, where the next global
        // request is a whole product away (the symmetric product reads LDS only).
        if (Sp != nullptr) {
            float *Sij = Sp + (int64_t)i * B * d_in + (int64_t)j * B;
            const uint32_t lb = opaque_u(wboff);
            const float *x0 = sm.X + opaque(p.lane_off(CS::P));
#pragma unroll
            for (int tm = 0; tm < 2; ++tm)
#pragma unroll
                for (int tn = 0; tn < 2; ++tn)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        gst(Sij, lb + CS::Pos::unif_boff(tm, tn, r, ldw), x0[CS::Pos::unif_off(tm, tn, r, CS::P)]);
        }
        float f2 = sym_frob2_stream<true>(sm.X, p, tid, 2 * blockIdx.x >= gridDim.x), unused = 0.f; // || S'^T S' ||_F^2
        block_sum2(f2, unused, sm.red, tid); // (barriers: X and the scratch are free again)
        if (tid == 0) beta_part[i * nbj + j] = sqrtf(f2) * sqrtf(dn2);
    }
    const uint32_t lb = opaque_u(gb);
#pragma unroll
    for (int tm = 0; tm < 2; ++tm)
#pragma unroll
        for (int tn = 0; tn < 2; ++tn)
#pragma unroll
            for (int r = 0; r < 16; ++r) gst(gp, lb + CS::Pos::unif_boff(tm, tn, r, B), -2.f * gacc.v[tm][tn][r]);
}

// ------------------------------------------------------------------------------------------------
// Core gradient at the current point (see phase_GS_kernel in chain.hip; after the joint-Adam step).
// Per block:  S' = A C (both streamed), R = Wbar - S' B, U = (R D) B^T, G = A^T U; Gout = -2 G.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(CS::NT, 2) void phase_GS_stream_kernel(
    const float *__restrict__ Wbar, const float *__restrict__ C, const float *__restrict__ A,
    const float *__restrict__ Bw, const float *__restrict__ D, int64_t d_in, int nbj, int nblocks,
    float *__restrict__ Gout, float *__restrict__ loss_part) {
    constexpr int B = SB;
    __shared__ SmemGrad sm;
    const int tid = threadIdx.x;
    const CS::Pos p(tid);
    const int ldw = (int)d_in;
    const uint32_t wboff = p.lane_boff(ldw);
    CS::Acc acc, accw;
    for (int blk = blockIdx.x; blk < nblocks; blk += gridDim.x) {
        const int i = blk / nbj, j = blk % nbj;
        const float *Cij = C + (int64_t)i * B * d_in + (int64_t)j * B;
        const float *Wij = Wbar + (int64_t)i * B * d_in + (int64_t)j * B;
        const float *Ai = A + (int64_t)i * B * B, *Bj = Bw + (int64_t)j * B * B;
        const float *Dj = D + (int64_t)j * B;
        mma_stream<Src::GK, Src::GX, true>(acc, Ai, B, Cij, ldw, p, [&]() { // S' = A C; Wbar requested behind it
            const uint32_t lb = opaque_u(wboff);
#pragma unroll
            for (int tm = 0; tm < 2; ++tm)
#pragma unroll
                for (int tn = 0; tn < 2; ++tn)
#pragma unroll
                    for (int r = 0; r < 16; ++r) accw.v[tm][tn][r] = gld(Wij, lb + CS::Pos::unif_boff(tm, tn, r, ldw));
        });
        CS::store_acc(sm.X, acc, p); // (the previous block is done with X: barriers at its end)
        __syncthreads();
        mma_stream<Src::LK, Src::GX, false, true>(accw, sm.X, 0, Bj, B, p); // R = Wbar - S' B
        float lsum = 0.f;
#pragma unroll
        for (int tn = 0; tn < 2; ++tn) {
            const float dj = Dj[p.col(tn)];
#pragma unroll
            for (int tm = 0; tm < 2; ++tm)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float res = accw.v[tm][tn][r];
                    lsum += res * res * dj;
                    accw.v[tm][tn][r] = res * dj;
                }
        }
        settle(lsum);
        __syncthreads();
        CS::store_acc(sm.X, accw, p); // R D
        __syncthreads();
        mma_stream<Src::LK, Src::GK, true>(acc, sm.X, 0, Bj, B, p); // U = (R D) B^T
        __syncthreads();
        CS::store_acc(sm.X, acc, p);
        __syncthreads();
        mma_stream<Src::GX, Src::LX, true>(acc, Ai, B, sm.X, 0, p); // G = A^T U
        {
            float *Gij = Gout + (int64_t)i * B * d_in + (int64_t)j * B;
            const uint32_t lb = opaque_u(wboff);
#pragma unroll
            for (int tm = 0; tm < 2; ++tm)
#pragma unroll
                for (int tn = 0; tn < 2; ++tn)
#pragma unroll
                    for (int r = 0; r < 16; ++r) gst(Gij, lb + CS::Pos::unif_boff(tm, tn, r, ldw), -2.f * acc.v[tm][tn][r]);
        }
        float unused = 0.f;
        block_sum2(lsum, unused, sm.red, tid); // (barriers: X is free again)
        if (tid == 0) loss_part[blk] = lsum;
    }
}

// ------------------------------------------------------------------------------------------------
// Forward/backward chain of the joint-Adam variant (see phase_FB_kernel in chain.hip).  Per block:
//   S = C B                      both operands streamed; resident
//   R D = (Wbar - A S) D         A^i streamed; Wbar is the accumulator's start; R D also to the scratch
//   grad_A += (R D) S^T          R D streamed back from the scratch, S resident
//   T = A^T (R D)                R D (still in registers) made resident; A^i streamed
//   C^T T -> grad_B partial      T resident, the core tile streamed (it is in L2 since the first product)
//   T B^T -> grad_W'             stays in the accumulator for the Adam update of the core, which runs
//                                one 32 x 32 tile at a time with the next tile's moments and core
//                                values already requested
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(CS::NT, 2) void phase_FB_stream_kernel(
    const float *__restrict__ Wbar, float *__restrict__ C, const float *__restrict__ A,
    const float *__restrict__ Bw, const float *__restrict__ D, const uint8_t *__restrict__ mask, int mask_group,
    float *__restrict__ mC, float *__restrict__ vC, AdamCoef k, int64_t d_in, int nbi, int nbj, int nsplit,
    float *__restrict__ gApart, float *__restrict__ gBpart, float *__restrict__ loss_part,
    float *__restrict__ scratch) {
    constexpr int B = SB;
    __shared__ SmemStream sm;
    const int tid = threadIdx.x;
    const CS::Pos p(tid);
    const int ldw = (int)d_in;
    const uint32_t wboff = p.lane_boff(ldw);
    const int i = blockIdx.x / nsplit, c = blockIdx.x % nsplit;
    const int chunk = (nbj + nsplit - 1) / nsplit;
    const int j0 = c * chunk, j1 = min(nbj, j0 + chunk);
    const int64_t mrow = d_in / mask_group;
    const int nb = B / mask_group; // mask bytes per block row: 16, 32 or 64
    const uint32_t mhalf = (uint32_t)((tid >> 1) * 64 + (tid & 1) * (nb >> 1));
    float *sc = scratch + (int64_t)blockIdx.x * B * B;
    const float *Ai = A + (int64_t)i * B * B;
    const uint32_t gb = p.lane_boff(B);
    CS::Acc gacc, acc, accw;
    gacc.zero();
    for (int j = j0; j < j1; ++j) {
        const int64_t boff = (int64_t)i * B * d_in + (int64_t)j * B;
        float *Cij = C + boff, *mij = mC + boff, *vij = vC + boff;
        const float *Wij = Wbar + boff;
        const float *Bj = Bw + (int64_t)j * B * B, *Dj = D + (int64_t)j * B;
        uint2 mreg[4];
        mma_stream<Src::GK, Src::GX, true>(acc, Cij, ldw, Bj, B, p, [&]() { // S = C B; Wbar and the mask bytes behind it
            const uint8_t *mb = mask + (int64_t)i * B * mrow + (int64_t)j * nb;
            const uint32_t mo = (uint32_t)((tid >> 1) * (int)mrow + (tid & 1) * (nb >> 1));
            const uint32_t lb = opaque_u(wboff);
#pragma unroll
            for (int it = 0; it < 4; ++it)
                if (it * 16 < nb) mreg[it] = gld(reinterpret_cast<const uint2 *>(mb), mo + 8u * it);
#pragma unroll
            for (int tm = 0; tm < 2; ++tm)
#pragma unroll
                for (int tn = 0; tn < 2; ++tn)
#pragma unroll
                    for (int r = 0; r < 16; ++r) accw.v[tm][tn][r] = gld(Wij, lb + CS::Pos::unif_boff(tm, tn, r, ldw));
        });
        CS::store_acc(sm.X, acc, p); // S   (the previous block is done with X and M: barriers at its end)
#pragma unroll
        for (int it = 0; it < 4; ++it)
            if (it * 16 < nb) *reinterpret_cast<uint2 *>(reinterpret_cast<char *>(sm.M) + mhalf + 8u * it) = mreg[it];
        __syncthreads();
        mma_stream<Src::GK, Src::LX, false, true>(accw, Ai, B, sm.X, 0, p); // R = Wbar - A S
        float lsum = 0.f;
#pragma unroll
        for (int tn = 0; tn < 2; ++tn) {
            const float dj = Dj[p.col(tn)];
#pragma unroll
            for (int tm = 0; tm < 2; ++tm)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float res = accw.v[tm][tn][r];
                    lsum += res * res * dj;
                    accw.v[tm][tn][r] = res * dj;
                }
        }
        settle(lsum);
        {
            const uint32_t lb = opaque_u(gb);
#pragma unroll
            for (int tm = 0; tm < 2; ++tm)
#pragma unroll
                for (int tn = 0; tn < 2; ++tn)
#pragma unroll
                    for (int r = 0; r < 16; ++r) gst(sc, lb + CS::Pos::unif_boff(tm, tn, r, B), accw.v[tm][tn][r]);
        }
        __syncthreads(); // scratch written by the whole workgroup (same CU, same L1: in order)
        mma_stream<Src::GK, Src::LK, false>(gacc, sc, B, sm.X, 0, p); // grad_A += (R D) S^T
        __syncthreads();
        CS::store_acc(sm.X, accw, p); // R D
        __syncthreads();
        mma_stream<Src::GX, Src::LX, true>(acc, Ai, B, sm.X, 0, p); // T = A^T (R D)
        __syncthreads();
        CS::store_acc(sm.X, acc, p); // T
        __syncthreads();
        mma_stream<Src::GX, Src::LX, true>(accw, Cij, ldw, sm.X, 0, p); // C^T T
        {
            float *gbp = gBpart + ((int64_t)j * nbi + i) * B * B;
            const uint32_t lb = opaque_u(gb);
#pragma unroll
            for (int tm = 0; tm < 2; ++tm)
#pragma unroll
                for (int tn = 0; tn < 2; ++tn)
#pragma unroll
                    for (int r = 0; r < 16; ++r) gst(gbp, lb + CS::Pos::unif_boff(tm, tn, r, B), -2.f * accw.v[tm][tn][r]);
        }
        // Adam on the core, g = -2 (T B^T) (.) M, one 32 x 32 tile (tm, tn) at a time; moments also decay on
        // pruned entries, whose core value is written back as it was.
        float cv[2][16], mo[2][16], vo[2][16];
        auto request_tile = [&](int slot, int tm, int tn) {
            const uint32_t lb = opaque_u(wboff);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const uint32_t off = lb + CS::Pos::unif_boff(tm, tn, r, ldw);
                cv[slot][r] = gld(Cij, off);
                mo[slot][r] = gld(mij, off);
                vo[slot][r] = gld(vij, off);
            }
        };
        mma_stream<Src::LK, Src::GK, true, false, STREAM_DEPTH>(acc, sm.X, 0, Bj, B, p, [&]() { request_tile(0, 0, 0); }); // T B^T
        {
            const uint8_t *ml = reinterpret_cast<const uint8_t *>(sm.M);
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int tm = t >> 1, tn = t & 1, slot = t & 1;
                if (t + 1 < 4) request_tile(slot ^ 1, (t + 1) >> 1, (t + 1) & 1);
                const uint32_t lb = opaque_u(wboff);
                const uint32_t mo_l = opaque_u((uint32_t)((p.wm0 + p.kh * 4) * 64 + p.col(tn) / mask_group));
                const int sh = p.col(tn) % mask_group;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const uint32_t off = lb + CS::Pos::unif_boff(tm, tn, r, ldw);
                    const uint32_t mbyte = ml[mo_l + (uint32_t)((tm * 32 + (r >> 2) * 8 + (r & 3)) * 64)];
                    const bool kp = (mbyte >> sh) & 1u;
                    const float g = kp ? -2.f * acc.v[tm][tn][r] : 0.f;
                    const float mn = k.b1 * mo[slot][r] + k.one_minus_b1 * g;
                    const float vn = k.b2 * vo[slot][r] + k.one_minus_b2 * g * g;
                    gst(mij, off, mn);
                    gst(vij, off, vn);
                    const float cn = cv[slot][r] - k.lr * (mn * k.inv_c1) / (sqrtf(vn * k.inv_c2) + k.eps);
                    gst(Cij, off, kp ? cn : cv[slot][r]);
                }
                __builtin_amdgcn_sched_barrier(0); // one tile at a time: bounds what is in flight
            }
        }
        float unused = 0.f;
        block_sum2(lsum, unused, sm.red, tid); // (barriers: X, M and the scratch are free again)
        if (tid == 0) loss_part[i * nbj + j] = lsum;
    }
    float *gp = gApart + (int64_t)blockIdx.x * B * B;
    const uint32_t lb = opaque_u(gb);
#pragma unroll
    for (int tm = 0; tm < 2; ++tm)
#pragma unroll
        for (int tn = 0; tn < 2; ++tn)
#pragma unroll
            for (int r = 0; r < 16; ++r) gst(gp, lb + CS::Pos::unif_boff(tm, tn, r, B), -2.f * gacc.v[tm][tn][r]);
}

} // namespace stream

using namespace stream;

void launch_phase_A_stream(const Dims &d, const float *Wbar, const float *C, const float *A, const float *B,
                           const float *D, int nsplit, float *gpart, float *beta_part, float *loss_part,
                           float *scratch, const WrapperPlanes *planes, hipStream_t s) {
    dim3 grid(d.nbi * nsplit), block(CS::NT);
    hipLaunchKernelGGL(phase_A_stream_kernel, grid, block, 0, s, Wbar, C, A, B, D, d.d_in, d.nbj, nsplit, gpart,
                       beta_part, loss_part, scratch, planes ? *planes : WrapperPlanes{});
}

bool stream_uses_planes() { return SPLIT_BF16; }
int stream_wgs_per_cu() { return SEQ_WGS; }

void launch_make_planes(const PlaneJob *job, int njobs, hipStream_t s) {
    PlaneJobs jobs = {};
    int total = 0;
    for (int j = 0; j < 3; ++j) {
        jobs.first[j] = total;
        if (j < njobs) {
            jobs.X[j] = job[j].X; jobs.P[j] = job[j].P; jobs.PT[j] = job[j].PT;
            total += job[j].nblk;
        }
    }
    jobs.first[3] = total;
    for (int j = njobs; j < 3; ++j) jobs.first[j] = total;
    if (total > 0) hipLaunchKernelGGL(make_planes_kernel, dim3(total, SB / 32), dim3(256), 0, s, jobs);
}

void launch_phase_B_stream(const Dims &d, const float *Wbar, const float *C, const float *A, const float *B,
                           const float *D, int nsplit, float *gpart, float *beta_part, float *Sp, float *scratch,
                           const WrapperPlanes *planes, hipStream_t s) {
    dim3 grid(d.nbj * nsplit), block(CS::NT);
    hipLaunchKernelGGL(phase_B_stream_kernel, grid, block, 0, s, Wbar, C, A, B, D, d.d_in, d.nbi, d.nbj, nsplit, gpart,
                       beta_part, Sp, scratch, planes ? *planes : WrapperPlanes{});
}

void launch_phase_WS_stream(const Dims &d, const float *Wbar, float *C, const float *A, const float *B,
                            const float *D, const float *AtA, const float *K, const uint8_t *mask, int mask_group,
                            const float *fro2A, const float *fro2K, float *Gout, float *loss_part, const float *Sp,
                            int grid_cap, const WrapperPlanes *planes, hipStream_t s) {
    dim3 grid(std::min(d.nblocks, grid_cap)), block(CS::NT);
    const WrapperPlanes pl = planes ? *planes : WrapperPlanes{};
    if (Gout != nullptr)
        hipLaunchKernelGGL(phase_WS_stream_kernel<true>, grid, block, 0, s, Wbar, C, A, B, D, AtA, K, mask, mask_group,
                           fro2A, d.nbi * gram_parts(d.b), fro2K, d.nbj * gram_parts(d.b), d.d_in, d.nbj, d.nblocks,
                           Gout, loss_part, Sp, pl);
    else // the W' step alone
        hipLaunchKernelGGL(phase_WS_stream_kernel<false>, grid, block, 0, s, Wbar, C, A, B, D, AtA, K, mask, mask_group,
                           fro2A, d.nbi * gram_parts(d.b), fro2K, d.nbj * gram_parts(d.b), d.d_in, d.nbj, d.nblocks,
                           Gout, loss_part, Sp, pl);
}

void launch_phase_GS_stream(const Dims &d, const float *Wbar, const float *C, const float *A, const float *B,
                            const float *D, float *Gout, float *loss_part, int grid_cap, hipStream_t s) {
    dim3 grid(std::min(d.nblocks, grid_cap)), block(CS::NT);
    hipLaunchKernelGGL(phase_GS_stream_kernel, grid, block, 0, s, Wbar, C, A, B, D, d.d_in, d.nbj, d.nblocks, Gout,
                       loss_part);
}

void launch_phase_FB_stream(const Dims &d, const float *Wbar, float *C, const float *A, const float *B,
                            const float *D, const uint8_t *mask, int mask_group, float *mC, float *vC,
                            double lr, double b1, double b2, double eps, int64_t t, int nsplit, float *gApart,
                            float *gBpart, float *loss_part, float *scratch, hipStream_t s) {
    const AdamCoef k = make_adam_coef(lr, b1, b2, eps, t);
    dim3 grid(d.nbi * nsplit), block(CS::NT);
    hipLaunchKernelGGL(phase_FB_stream_kernel, grid, block, 0, s, Wbar, C, A, B, D, mask, mask_group, mC, vC, k,
                       d.d_in, d.nbi, d.nbj, nsplit, gApart, gBpart, loss_part, scratch);
}

} // namespace armor
