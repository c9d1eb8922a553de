// Internal launch interface between the C ABI (armor_api.hip) and the kernel files.
// Everything here takes raw device pointers and a stream; nothing allocates.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace armor {

struct Dims {
    int64_t d_out, d_in;
    int b;        // block size of the wrappers (Sec. 3.1)
    int nbi, nbj; // number of row / column blocks
    int nblocks;  // nbi * nbj
};

// The wrapper-sized operands of the d_block 128 streamed chains cut into three bf16 pieces each
// (chain_stream.hip; all NULL when that path's fp32 matrix instruction is compiled in): A^i and B^j in both
// orientations, K^j = B^j D^j B^jT and A^iT A^i (symmetric).  Each array holds 3 * 128 * 128 16-bit values per block.
struct WrapperPlanes {
    uint16_t *A, *AT, *B, *BT, *K, *AtA;
};
bool stream_uses_planes();
int stream_wgs_per_cu(); // workgroups per CU the sequential-variant streamed kernels are built for
// pieces of the nblk blocks of X [nblk][128][128]: P = of X[x][k] (k = column), PT = of X[k][x] (may be NULL);
// up to three matrices per launch
struct PlaneJob {
    const float *X;
    int nblk;
    uint16_t *P, *PT;
};
void launch_make_planes(const PlaneJob *job, int njobs, hipStream_t s);

// ---- fused per-block chains (chain.hip) -------------------------------------------------------
// A-phase of Alg. 2: per block S = C B, R = Wbar - A S, partial grad_A, ||S D S^T||_F, block loss.
void launch_phase_A(const Dims &d, const float *Wbar, const float *C, const float *A, const float *B,
                    const float *D, int nsplit, float *gpart, float *beta_part, float *loss_part,
                    bool loss_only, float *stream_scratch, const WrapperPlanes *planes, hipStream_t s);
// B-phase: S' = A C, R = Wbar - S' B, partial grad_B, ||S'^T S'||_F ||D^j||_F.
void launch_phase_B(const Dims &d, const float *Wbar, const float *C, const float *A, const float *B,
                    const float *D, int nsplit, float *gpart, float *beta_part, float *Sp, float *stream_scratch,
                    const WrapperPlanes *planes, hipStream_t s);
// The same phases at d_block 128 with one operand streamed from global memory and two workgroups
// per CU (chain_stream.hip); launch_phase_A / _B / _WS go there when given the scratch (A, B: one
// b x b tile per workgroup) or S' (W' step).
void launch_phase_A_stream(const Dims &d, const float *Wbar, const float *C, const float *A, const float *B,
                           const float *D, int nsplit, float *gpart, float *beta_part, float *loss_part,
                           float *scratch, const WrapperPlanes *planes, hipStream_t s);
void launch_phase_FB_stream(const Dims &d, const float *Wbar, float *C, const float *A, const float *B,
                            const float *D, const uint8_t *mask, int mask_group, float *mC, float *vC,
                            double lr, double b1, double b2, double eps, int64_t t, int nsplit, float *gApart,
                            float *gBpart, float *loss_part, float *scratch, hipStream_t s);
void launch_phase_GS_stream(const Dims &d, const float *Wbar, const float *C, const float *A, const float *B,
                            const float *D, float *Gout, float *loss_part, int grid_cap, hipStream_t s);
void launch_phase_B_stream(const Dims &d, const float *Wbar, const float *C, const float *A, const float *B,
                           const float *D, int nsplit, float *gpart, float *beta_part, float *Sp, float *scratch,
                           const WrapperPlanes *planes, hipStream_t s);
// W' step of Alg. 2 alone (unstructured mode): C += (2/beta_W) (A^T ((Wbar - A C B) D) B^T) (.) M, beta_W
// read from scalars[2].  grid_cap workgroups at most, each walking blocks w, w + grid, ...
void launch_phase_W(const Dims &d, const float *Wbar, float *C, const float *A, const float *B, const float *D,
                    const uint8_t *mask, int mask_group, const float *fro2A, const float *fro2K, const float *Sp, int grid_cap,
                    const WrapperPlanes *planes, hipStream_t s);
// Per wrapper block: A^iT A^i, its diagonal ||A^i[:,p]||^2 and ||A^iT A^i||_F^2; K^j = B^j D^j B^jT, ||K^j||_F^2.
// PAtA / PK (d_block 128 only, else null): the two results also as bf16 plane sets.
void launch_wrapper_grams(const Dims &d, const float *A, const float *B, const float *D, float *colnorm2,
                          float *fro2A, float *AtA, float *K, float *fro2K, uint16_t *PAtA, uint16_t *PK,
                          hipStream_t s);
// W' step fused with the core gradient at the updated core (N:M mode): C += (2/beta_W) G (.) M,
// Gout = -2 (G - (2/beta_W) (A^T A)(G (.) M) K), block loss after the continuous step to loss_part.
void launch_phase_WS(const Dims &d, const float *Wbar, float *C, const float *A, const float *B, const float *D,
                     const float *AtA, const float *K, const uint8_t *mask, int mask_group, const float *fro2A,
                     const float *fro2K, float *Gout, float *loss_part, const float *Sp, int grid_cap,
                     const WrapperPlanes *planes, hipStream_t s);
void launch_phase_WS_stream(const Dims &d, const float *Wbar, float *C, const float *A, const float *B, const float *D,
                     const float *AtA, const float *K, const uint8_t *mask, int mask_group, const float *fro2A,
                     const float *fro2K, float *Gout, float *loss_part, const float *Sp, int grid_cap,
                     const WrapperPlanes *planes, hipStream_t s);
int chain_max_nsplit();
// Joint-Adam forward/backward pass: gradients of A (gApart, nsplit chunks per row block), B (gBpart,
// one partial per block, laid out [j][i]) and the Adam update of the core and its moments in place.
void launch_phase_FB(const Dims &d, const float *Wbar, float *C, const float *A, const float *B, const float *D,
                     const uint8_t *mask, int mask_group, float *mC, float *vC, double lr, double b1, double b2,
                     double eps, int64_t t, int nsplit, float *gApart, float *gBpart, float *loss_part,
                     float *stream_scratch, hipStream_t s);
// Core gradient at the current point: Gout = -2 A^T ((Wbar - A C B) D) B^T, block losses to loss_part.
void launch_phase_GS(const Dims &d, const float *Wbar, const float *C, const float *A, const float *B, const float *D,
                     float *Gout, float *loss_part, int grid_cap, hipStream_t s);

// ---- the same chains on 128 x 128 sub-tiles for d_block = 256 (chain_big.hip) ------------------
// scratch: big_scratch_floats(d, grid_cap) floats; grid_cap bounds the number of workgroups.
size_t big_scratch_floats(const Dims &d, int max_wgs);
void launch_big_phase_A(const Dims &d, const float *Wbar, const float *C, const float *A, const float *B,
                        const float *D, int nsplit, float *gpart, float *beta_part, float *loss_part, bool loss_only,
                        int grid_cap, float *scratch, hipStream_t s);
void launch_big_phase_B(const Dims &d, const float *Wbar, const float *C, const float *A, const float *B,
                        const float *D, int nsplit, float *gpart, float *beta_part, float *Sp, int grid_cap,
                        float *scratch, hipStream_t s);
void launch_big_phase_WS(const Dims &d, const float *Wbar, float *C, const float *A, const float *B, const float *D,
                         const float *AtA, const float *K, const uint8_t *mask, int mask_group, const float *fro2A,
                         const float *fro2K, float *Gout, float *loss_part, const float *Sp, bool fused, int grid_cap, float *scratch,
                         hipStream_t s);
void launch_big_phase_FB(const Dims &d, const float *Wbar, float *C, const float *A, const float *B, const float *D,
                         const uint8_t *mask, int mask_group, float *mC, float *vC, double lr, double b1, double b2,
                         double eps, int64_t t, int nsplit, float *gApart, float *gBpart, float *loss_part, int grid_cap,
                         float *scratch, hipStream_t s);
void launch_big_phase_GS(const Dims &d, const float *Wbar, const float *C, const float *A, const float *B,
                         const float *D, float *Gout, float *loss_part, int grid_cap, float *scratch, hipStream_t s);
void launch_big_wrapper_grams(const Dims &d, const float *A, const float *B, const float *D, float *colnorm2,
                              float *fro2A, float *AtA, float *K, float *fro2K, hipStream_t s);

// ---- small kernels (small.hip) ----------------------------------------------------------------
// partial: (nchunk + 1) * d_in floats; the last d_in receive 1 / r1, which launch_rownorm_scale takes
void launch_colnorm(const void *W, int bf16, int64_t d_out, int64_t d_in, float *partial, int nchunk, float *r1,
                    hipStream_t s);
void launch_rownorm_scale(const void *W, int bf16, int64_t d_out, int64_t d_in, const float *r1_inv, float *r2,
                          float *Wbar, hipStream_t s);
int diag_x_chunks(int64_t n);
void launch_diag_x(const void *X, int bf16, int64_t n, int64_t d_in, int64_t ldx, float *D, int accumulate,
                   float *partial, hipStream_t s);
void launch_init_identity(float *A, int nblk, int b, hipStream_t s);
void launch_init_nm(const float *Wbar, const float *D, int64_t d_out, int64_t d_in, int N, int M, float *C,
                    uint8_t *mask, hipStream_t s);
void launch_diag(const float *H, int64_t d_in, int64_t ldh, float *D, hipStream_t s);
// A -= (sum of partials)/beta, beta = 2 * sum(beta_part); optionally trace_out = sum(loss_part) and
// eta_out = 1/beta.
// P / PT (d_block 128 only, else null): the kernel also writes the updated wrapper's bf16 plane sets.
void launch_update_wrapper(float *A, int nblk, int b, const float *gpart, int nsplit, const float *beta_part,
                           int nblocks, const float *loss_part, double *trace_out, double *eta_out, uint16_t *P,
                           uint16_t *PT, hipStream_t s);
void launch_adam_wrapper(float *X, float *m, float *v, int nblk, int b, const float *gpart, int nsplit, double lr,
                         double b1, double b2, double eps, int64_t t, int nblocks, const float *loss_part,
                         double *trace_out, hipStream_t s);
void launch_zero(float *x, int64_t n, hipStream_t s);
void launch_fill(float *x, int64_t n, float v, hipStream_t s);

// Loss-only forward pass that can also leave the residual R sqrt(D) (R D at d_block 256) in Rout, a d_out x d_in
// matrix with leading dimension d_in (chain.hip: d_block <= 128; chain_big.hip: 256).  Rout may be null.
void launch_residual(const Dims &d, const float *Wbar, const float *C, const float *A, const float *B, const float *D,
                     int nsplit, float *Rout, float *loss_part, hipStream_t s);
void launch_big_residual(const Dims &d, const float *Wbar, const float *C, const float *A, const float *B,
                         const float *D, int nsplit, float *Rout, float *loss_part, int grid_cap, float *scratch,
                         hipStream_t s);

// ---- loss against the whole Gram matrix (full_h.hip) ---------------------------------------------
// tile edge used for d_out x d_in, number of per-tile partial sums, and the launch:  part[tile] = <R_tile, (R H)_tile>
int full_h_tile(int64_t d_out, int64_t d_in);
int64_t full_h_parts(int64_t d_out, int64_t d_in);
void launch_full_h_loss(const float *R, int64_t d_out, int64_t d_in, const float *H, int64_t ldh, float *part,
                        int grid_cap, hipStream_t s);
int gram_parts(int b);
void launch_sum_to_double(const float *part, int n, double *out, hipStream_t s);
void launch_broadcast_double(double *dst, int64_t n, const double *src, hipStream_t s); // dst[0..n) = *src
void launch_sparse_step(const Dims &d, const float *G, float *C, uint8_t *mask, const float *K,
                        const float *colnorm2, int N, int M, int selection, uint64_t seed, int64_t t,
                        const float *loss_part, double *loss_cont_out, int32_t *changes_out, hipStream_t s);
// eta_out = 1 / beta_W' (Eq. 11) from the same partial sums and in the same order as the W' kernels take it.
void launch_eta_W_trace(const Dims &d, const float *fro2A, const float *fro2K, double *eta_out, hipStream_t s);
// flag[0] = number of NaN/Inf entries of W (d_out x d_in, fp32 or bf16) plus NaN/Inf/negative entries of D.
void launch_count_nonfinite(const void *W, int bf16, int64_t n, const float *D, int64_t d_in, int32_t *flag,
                            hipStream_t s);
void launch_denormalize(float *A, float *B, const float *r1, const float *r2, int64_t d_out, int64_t d_in, int b,
                        hipStream_t s);
void launch_pack_nm(const float *S, const uint8_t *mask, int64_t d_out, int64_t d_in, int N, int M, void *values,
                    int bf16, uint8_t *meta, hipStream_t s);
void launch_unstructured_init(const float *Wbar, const float *D, int64_t d_out, int64_t d_in, int64_t keep,
                              float *C, uint8_t *mask, uint32_t *score_buf, void *ws, hipStream_t s);
size_t unstructured_init_ws_bytes(int64_t d_out, int64_t d_in);

// ---- Gram (gram.hip) --------------------------------------------------------------------------
// ws (optional): gram_workspace_bytes() bytes for split-K partial tiles; without it one slice is used.
size_t gram_workspace_bytes(int64_t n, int64_t d_in, int bf16);
void launch_gram(const void *X, int bf16, int64_t n, int64_t d_in, int64_t ldx, float *H, int64_t ldh,
                 int accumulate, void *ws, size_t ws_bytes, hipStream_t s);

// ---- factorized layer applied to activations (apply.hip) ----------------------------------------
void launch_to_bf16(const float *in, int64_t n, void *out, hipStream_t s);
int64_t apply_prepared_bytes(int64_t d_out, int64_t d_in);
int64_t apply_acts_bytes(int64_t n, int64_t d_in);
void launch_apply_prepare(const void *values, const uint8_t *meta, int64_t d_out, int64_t d_in, void *prepared,
                          hipStream_t s);
void launch_apply_pre(const void *X, int64_t n, int64_t d_in, int b, const void *Bw, void *U, hipStream_t s);
hipError_t launch_apply_main(const void *U, int64_t n, int64_t d_in, int64_t d_out, int b, const void *prepared,
                             const void *Aw, void *Y, hipStream_t s);

} // namespace armor
