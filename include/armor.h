/*
 * armor.h -- C ABI of the MI355X (gfx950) implementation of ARMOR's per-layer factorization:
 * fit  W-bar ~= A * S * B  with A, B block-diagonal wrappers and S = W' (.) M an N:M-sparse core
 * (Sec. 3.1, Eq. 1) by block coordinate descent on the layer-wise proxy loss (Sec. 3.2, Eq. 2;
 * Sec. 3.3, Alg. 1-3).
 *
 * General conventions
 *   - Every pointer is a DEVICE pointer unless a comment says "host".  The caller owns every
 *     buffer; the library never allocates or frees device memory: scratch comes from the `ws`
 *     argument, sized by the matching *_workspace_bytes() query.  All device buffers must be
 *     16-byte aligned.
 *   - Matrices are row-major.  W[i*d_in + j] couples output i with input j (Sec. 2).  The sparse
 *     axis is d_in: a group is M consecutive columns of one row (Sec. 2).  Block-diagonal wrappers
 *     are stored as [d/d_block][d_block][d_block], A[i][p][q] = (A^(i))_pq (Sec. 3.1).
 *   - mask_bits holds one byte per group, [d_out][d_in/M]; bit p set = column p of the group kept.
 *     In unstructured mode a byte covers 8 consecutive columns.
 *   - Calls are asynchronous on `hip_stream` (a hipStream_t passed as void*; NULL = default
 *     stream), return a status code, never throw and never print.  Argument errors are detected
 *     on the host before any launch.  Results are deterministic: no floating-point atomics.
 *     Two options of armor_factorize_layer make it wait for the stream: check_finite (once, before any
 *     work) and tol (once per iteration); armor_proxy_loss_noalloc takes its scratch from an array inside
 *     the library instead of a workspace argument.
 *   - d_block must divide d_out and d_in and be one of 32, 64, 128, 256; M must divide d_block,
 *     1 <= N < M <= 8; d_block * d_in <= 2^29 (a block row is addressed with 32-bit byte offsets).
 */
#ifndef ARMOR_H
#define ARMOR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Status and dtype codes travel as 32-bit integers (any value a caller passes is representable and is
 * validated; an out-of-range value of a C++ enumeration type would be undefined behaviour). */
typedef int32_t armor_status;
enum {
    ARMOR_OK = 0,
    ARMOR_ERR_NULL = 1,      /* a required pointer is NULL */
    ARMOR_ERR_SHAPE = 2,     /* d_block does not divide d_out/d_in, M does not divide d_block, bad N/M, ... */
    ARMOR_ERR_DTYPE = 3,     /* unknown armor_dtype */
    ARMOR_ERR_WORKSPACE = 4, /* ws is NULL or ws_bytes too small */
    ARMOR_ERR_ALIGN = 5,     /* a device buffer is not 16-byte aligned */
    ARMOR_ERR_DEVICE = 6,    /* a HIP call failed; see armor_last_hip_error() */
    ARMOR_ERR_UNSUPPORTED = 7, /* valid request that this build does not implement */
    ARMOR_ERR_NONFINITE = 8,   /* opts->check_finite: W has a NaN/Inf entry, or a loss weight H_jj is NaN/Inf/negative */
    ARMOR_ERR_TOO_LARGE = 9    /* armor_proxy_loss_noalloc: the problem needs more than the library's fixed scratch */
};

typedef int32_t armor_dtype;
enum { ARMOR_F32 = 0, ARMOR_BF16 = 1 };

/* Options of armor_factorize_layer.  Zero-initialise for the defaults. */
typedef struct {
    int32_t selection;          /* group selection heuristic (Sec. 3.3.2, App. E.1): 0 = L1-weighted random
                                   (default), 1 = L1 greedy, 2 = L2-weighted random, 3 = uniform random */
    int32_t sparsity;           /* 0 = N:M (both BCD steps); 1 = unstructured: continuous step only (Sec. 4.5) */
    int64_t unstructured_keep;  /* sparsity==1: number of kept entries (global top-k of the importance) */
    uint64_t seed;              /* seed of the counter-based selection hash */
    int32_t denormalize;        /* 1: fold r2 into the rows of A and r1 into the columns of B (Sec. 3.2) */
    int32_t variant;            /* continuous step (Sec. 3.3.1): 0 = sequential gradient steps with 1/beta step
                                   sizes (Alg. 2; monotone, default), 1 = joint Adam on A, B, W' (what the authors
                                   run in practice; one forward/backward pass per iteration) */
    double lr;                  /* Adam learning rate; 0 = 1e-4 (App. F) */
    double adam_beta1;          /* 0 = 0.9   (the optimiser's published default; the paper gives none) */
    double adam_beta2;          /* 0 = 0.999 */
    double adam_eps;            /* 0 = 1e-8  */
    int32_t init_from_outputs;  /* 1: theta_0 is not Eq. 3 but what the caller left in A, S, B and mask_bits (all
                                   required then; normalised space; S zero wherever its mask bit is clear).  Alg. 1
                                   takes theta_0 as an input: this is how a stopped run is continued.  The joint-Adam
                                   variant starts again with zero moments and step count 1. */
    int32_t check_finite;       /* 1: validate W and the loss weights first; the call then waits for the stream once
                                   and returns ARMOR_ERR_NONFINITE before anything else is enqueued */
    int64_t iter_offset;        /* iterations already done: iteration t of this call draws its groups (Alg. 3) with
                                   the counter of iteration iter_offset + t; >= 0 */
    double tol;                 /* the tolerance input of Alg. 1 (the listing declares it and never uses it): > 0 ends
                                   the loop after the first iteration t whose decrease is within it,
                                   L_{t-1} - L_t <= tol * L_0; 0 (default) runs all n_iters.  L_t is known one forward
                                   pass later, so with tol > 0 every iteration copies one double to the host and waits
                                   for the stream (the only synchronisation inside the loop); the forward pass that
                                   found the stop is discarded and the outputs are theta_t.  Trace entries of
                                   iterations that did not run repeat the final loss (loss_trace, loss_cont_trace) or
                                   are 0 (eta_trace, mask_changes); armor_last_iteration_count() tells how many ran.
                                   Sequential variant only (joint Adam updates the core inside its forward/backward
                                   kernel and cannot discard a pass): ARMOR_ERR_UNSUPPORTED with variant = 1. */
} armor_opts;

const char *armor_status_string(armor_status s);
/* Iterations the last armor_factorize_layer call of the calling thread ran (n_iters unless opts->tol ended it). host. */
int64_t armor_last_iteration_count(void);
/* hipError_t (as int) of the last failed HIP call made by this library on the calling thread. host. */
int armor_last_hip_error(void);

/*
 * Optional per-kernel timing (host-side; not thread-safe; off by default).  While enabled, the
 * library brackets each instrumented kernel launch with HIP events recorded on the caller's
 * stream (timing-only events, host resources created on first use and kept; no device memory).
 * Inside the iteration loop of armor_factorize_layer and inside armor_apply_packed, consecutive
 * launches share their boundary event: a launch is then timed from the end of its predecessor
 * to its own end.
 * armor_profile_read() waits for the recorded events, returns per kind the summed elapsed
 * milliseconds and the number of launches into two HOST arrays of ARMOR_PROF_KINDS entries, and
 * resets the record.  Kinds: the Gram kernel (Sec. 2), the A-step and B-step chains of Alg. 2,
 * the chain that fuses the W' step with the core gradient feeding Alg. 3, and the Alg. 3 kernel.
 */
#define ARMOR_PROF_GRAM 0
#define ARMOR_PROF_PHASE_A 1
#define ARMOR_PROF_PHASE_B 2
#define ARMOR_PROF_PHASE_WS 3
#define ARMOR_PROF_SPARSE 4
#define ARMOR_PROF_PHASE_FB 5 /* joint-Adam forward/backward chain */
#define ARMOR_PROF_PHASE_GS 6 /* core-gradient chain of the joint-Adam variant */
#define ARMOR_PROF_NORMALIZE 7 /* column norms + row norms and scaling (two kernels) */
#define ARMOR_PROF_INIT 8      /* initial mask and core (Eq. 3), N:M or unstructured */
#define ARMOR_PROF_PACK 9      /* armor_pack_nm */
#define ARMOR_PROF_SMALL 10    /* wrapper updates, wrapper Grams */
#define ARMOR_PROF_APPLY_PRE 11  /* armor_apply_packed: U = X B^T */
#define ARMOR_PROF_APPLY_MAIN 12 /* armor_apply_packed: Y = (U S^T) A^T */
#define ARMOR_PROF_DIAG_X 13     /* armor_gram_diag_x */
#define ARMOR_PROF_RESIDUAL 14   /* armor_proxy_loss_full_h: forward chain that leaves R */
#define ARMOR_PROF_FULL_H 15     /* armor_proxy_loss_full_h: <R, R H> */
#define ARMOR_PROF_KINDS 16
armor_status armor_profile_enable(int on);
armor_status armor_profile_read(double *ms_total /*host [ARMOR_PROF_KINDS]*/, int64_t *launches /*host*/);

/*
 * Gram matrix of the calibration activations (Sec. 2; the loss of Eq. 2 uses its diagonal).
 *   X   [n_tokens x d_in], leading dimension ldx (elements), fp32 or bf16; one token per row
 *       (this is the paper's X^T).
 *   H   [d_in x d_in] fp32, leading dimension ldh.  accumulate = 0: H = X^T X;  1: H += X^T X,
 *       so a caller can stream token chunks.  Both triangles are written.
 * d_in must be a multiple of 32; n_tokens >= 0 (0 leaves H unchanged / zeroes it).
 *   ws  optional scratch of armor_gram_workspace_bytes() bytes (may be NULL / 0): lets the bf16 kernel
 *       split the token axis into slices whose partial tiles are summed in a fixed order, which
 *       fills the GPU when d_in/256 gives few output tiles.  Results do not depend on timing, but the
 *       slice count (and so the rounding of the sums) depends on whether ws is given.
 */
size_t armor_gram_workspace_bytes(int64_t n_tokens, int64_t d_in, armor_dtype x_dtype);
armor_status armor_gram(const void *X, armor_dtype x_dtype, int64_t n_tokens, int64_t d_in, int64_t ldx,
                        float *H, int64_t ldh, int accumulate, void *ws, size_t ws_bytes, void *hip_stream);

/* D[j] = H[j][j]  (the weights ||X_j||^2 of Eq. 2). */
armor_status armor_gram_diag(const float *H, int64_t d_in, int64_t ldh, float *D, void *hip_stream);

/*
 * The same weights straight from the activations, without forming H (Eq. 2 only uses diag(X X^T)):
 *   D[j] (+)= sum_t X[t][j]^2        X [n_tokens][d_in] row-major with row pitch ldx, fp32 or bf16.
 * accumulate as in armor_gram.  d_in must be a multiple of 8 (bf16) / 4 (fp32), X 16-byte aligned and
 * ldx a multiple of the same count; ws of armor_gram_diag_x_workspace_bytes() bytes is required.
 * One pass over X: 2 (bf16) or 4 bytes per element, HBM-bound.
 */
size_t armor_gram_diag_x_workspace_bytes(int64_t n_tokens, int64_t d_in);
armor_status armor_gram_diag_x(const void *X, armor_dtype x_dtype, int64_t n_tokens, int64_t d_in, int64_t ldx,
                               float *D, int accumulate, void *ws, size_t ws_bytes, void *hip_stream);

/*
 * Row/column normalisation of Sec. 3.2:  r1[j] = ||W[:,j]||,  r2[i] = ||W[i,:]/r1||,
 * Wbar = W / r1 / r2.  A zero norm is replaced by 1.  W fp32 or bf16; outputs fp32.
 * ws: armor_normalize_workspace_bytes(d_out, d_in).
 */
size_t armor_normalize_workspace_bytes(int64_t d_out, int64_t d_in);
armor_status armor_normalize(const void *W, armor_dtype w_dtype, int64_t d_out, int64_t d_in, float *Wbar,
                             float *r1 /*[d_in]*/, float *r2 /*[d_out]*/, void *ws, size_t ws_bytes,
                             void *hip_stream);

/*
 * Proxy loss of Eq. 2:  L = sum_ij (Wbar - A S B)_ij^2 * H_jj.
 *   A [d_out/b][b][b] or NULL (= identity);  B [d_in/b][b][b] or NULL (= identity);
 *   S dense [d_out x d_in] (zeros at pruned positions);
 *   H: ldh > 0: the Gram matrix, only its diagonal is read;  ldh == 0: H is the vector D [d_in].
 *   loss_out: one double in DEVICE memory.
 */
size_t armor_proxy_loss_workspace_bytes(int64_t d_out, int64_t d_in, int64_t d_block);
armor_status armor_proxy_loss(const float *Wbar, const float *A, const float *S, const float *B, const float *H,
                              int64_t ldh, int64_t d_out, int64_t d_in, int64_t d_block, double *loss_out,
                              void *ws, size_t ws_bytes, void *hip_stream);

/*
 * armor_proxy_loss for callers that cannot allocate or supply a workspace: code under HIP graph capture,
 * tight serving/monitoring loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and the same
 * result as armor_proxy_loss, but the scratch (loss weights, identity wrappers for a NULL A / B, per-block
 * partial losses, chain scratch at d_block 256) is a fixed 32 MiB array inside the library's device image --
 * every GPU the library runs on holds one copy until the process ends -- whose device address is looked up on
 * the first call on each device.  No hipMalloc / hipFree or other allocating call is made.
 *   Limit: d_in*4 + (A ? 0 : d_out*d_block*4) + (B ? 0 : d_in*d_block*4) + 4*blocks (+ at d_block 256 at least
 *   one 512 KiB chain scratch; as many workgroups run as fit) must fit in 32 MiB, else ARMOR_ERR_TOO_LARGE and
 *   nothing is enqueued (e.g. 4096 x 4096 at d_block 128 needs 4.2 MiB; 28672 x 8192 at d_block 256 fits only
 *   with both wrappers given).
 *   All calls on one GPU share the array and it keeps the previous call's contents; every location is written
 *   before it is read, so nothing has to be cleared, but two calls that overlap on one GPU (different streams or
 *   threads) race: serialise them.  The first call on a device should be made outside a stream capture.
 */
armor_status armor_proxy_loss_noalloc(const float *Wbar, const float *A, const float *S, const float *B,
                                      const float *H, int64_t ldh, int64_t d_out, int64_t d_in, int64_t d_block,
                                      double *loss_out, void *hip_stream);

/*
 * The layer-wise objective against the WHOLE Gram matrix (Sec. 2 states the objective with the activations
 * themselves; Eq. 2, the proxy the method optimises, keeps only its diagonal):
 *     L_H = tr(R H R^T) = || R X^T ||_F^2  for H = X^T X,   R = Wbar - A S B.
 * Evaluation only -- the block decomposition of Eq. 5 needs a diagonal weight, so no step of Alg. 1-3 uses
 * this value; it tells how far the diagonal proxy is from the full second-order objective for a given
 * factorization.  For a diagonal H it equals armor_proxy_loss.
 *   Wbar, S: dense [d_out x d_in] fp32;  A [d_out/b][b][b] or NULL (= identity);  B [d_in/b][b][b] or NULL;
 *   H: [d_in x d_in] fp32, symmetric, leading dimension ldh >= d_in, ldh a multiple of 4 (all of it is read;
 *      express it in the same coordinates as Wbar: after the normalisation of Sec. 3.2, H_jk r1_j r1_k);
 *   loss_out: one double in DEVICE memory;  ws: armor_proxy_loss_full_h_workspace_bytes() bytes of device
 *   memory (holds R: 4*d_out*d_in bytes plus what armor_proxy_loss needs), 16-byte aligned like Wbar, S, H.
 * Cost: the forward chain of armor_proxy_loss plus one d_out x d_in x d_in product (fp32 operands as three
 * bf16 pieces each on the bf16 matrix instruction when d_out and d_in are multiples of 128, else the fp32
 * matrix instruction on 32 x 32 tiles); per-tile sums in fp32, their total in fp64.
 * Errors: ARMOR_ERR_NULL, ARMOR_ERR_SHAPE (shape rules of armor_proxy_loss; ldh), ARMOR_ERR_WORKSPACE,
 * ARMOR_ERR_ALIGN; nothing is enqueued on error.
 */
size_t armor_proxy_loss_full_h_workspace_bytes(int64_t d_out, int64_t d_in, int64_t d_block);
armor_status armor_proxy_loss_full_h(const float *Wbar, const float *A, const float *S, const float *B,
                                     const float *H, int64_t ldh, int64_t d_out, int64_t d_in, int64_t d_block,
                                     double *loss_out, void *ws, size_t ws_bytes, void *hip_stream);

/*
 * The whole BCD loop (Alg. 1): normalise W, initialise by Eq. 3 (A = B = I, top-N of every group by
 * Wbar^2 * H_jj), then n_iters times { continuous update (Alg. 2: sequential gradient steps on A, B,
 * W' with step 1/beta, App. D) ; sparse-core update (Alg. 3: one group per block, all C(M,N) masks,
 * closed-form least squares of Eq. 7/8) }.
 *   W          [d_out x d_in] fp32 or bf16 (not modified)
 *   H, ldh     as in armor_proxy_loss
 *   A, S, B    outputs; S is the core W' (.) M as a dense matrix with exact zeros at pruned positions
 *   mask_bits  output, [d_out][d_in/M] bytes (unstructured: [d_out][d_in/8]); may be NULL
 *   r1, r2     outputs [d_in], [d_out] (normalisation scales); may be NULL
 *   loss_trace output, n_iters+1 doubles in DEVICE memory, L(theta_0..theta_n) in the normalised
 *              space; loss_trace[0] is the loss of plain N:M pruning (Sec. 3.4).  May be NULL.
 *   loss_cont_trace  optional, n_iters doubles: loss after the continuous step of each iteration.
 *   eta_trace  optional, 3 * n_iters doubles in DEVICE memory: the step sizes eta_A, eta_B, eta_W' = 1/beta of
 *              Eq. 9-11 that iteration t applied, at [3(t-1) .. 3(t-1)+2] (0 where beta = 0).  Sequential
 *              variant only (the joint-Adam variant leaves it untouched).
 *   mask_changes  optional, n_iters int32 in DEVICE memory: number of groups whose kept set the sparse-core
 *              step of iteration t changed (0 in unstructured mode).
 * With opts->denormalize = 0 (default) A, S, B live in the normalised space:
 *   W ~= diag(r2) (A S B) diag(r1).
 * Errors: bad arguments as in the status codes above, found on the host before any launch; with
 * opts->check_finite the inputs are also scanned on the device (ARMOR_ERR_NONFINITE).  Without it a NaN/Inf
 * in W or H propagates into the outputs.
 */
size_t armor_factorize_workspace_bytes(int64_t d_out, int64_t d_in, int64_t d_block, int N, int M,
                                       const armor_opts *opts);
armor_status armor_factorize_layer(const void *W, armor_dtype w_dtype, const float *H, int64_t ldh, int64_t d_out,
                                   int64_t d_in, int64_t d_block, int N, int M, int n_iters,
                                   const armor_opts *opts, float *A, float *S, float *B, uint8_t *mask_bits,
                                   float *r1, float *r2, double *loss_trace, double *loss_cont_trace,
                                   double *eta_trace, int32_t *mask_changes, void *ws, size_t ws_bytes,
                                   void *hip_stream);

/*
 * Compressed N:M storage of the core (the form an N:M sparse matmul consumes; Sec. 3.1 stores the
 * core as an N:M matrix):
 *   values [d_out][d_in/M*N]  the kept entries of each group in increasing column order
 *          (fp32 or bf16 per v_dtype);
 *   meta   [d_out][meta_row]  per kept entry, in the same order, its column inside the group
 *          (0..M-1) in a field of 1, 2 or 4 bits for M = 2, 4, 8; fields fill each byte from bit 0
 *          upwards; meta_row = ceil(d_in/M*N*field_bits / 8) bytes, so every row starts on a byte
 *          boundary and unused bits of a row's last byte are zero.  For 2:4 one byte holds the
 *          four 2-bit indices of two groups.
 * S must be 16-byte aligned.  armor_pack_meta_row_bytes returns meta_row (0 on a bad shape).
 */
int64_t armor_pack_meta_row_bytes(int64_t d_in, int N, int M);
armor_status armor_pack_nm(const float *S, const uint8_t *mask_bits, int64_t d_out, int64_t d_in, int N, int M,
                           void *values, armor_dtype v_dtype, uint8_t *meta, void *hip_stream);

/*
 * The factorized layer applied to a batch of activations (Sec. 3.1: the wrappers are block
 * products around the N:M core; Sec. 4.4 times this product on a batch of tokens):
 *     Y[t] = A (S (B X[t]))      t = 0 .. n_tokens-1
 *
 * armor_apply_prepare (once per layer) re-tiles the compressed core into the order the product
 * streams it in:
 *   values   [d_out][d_in/2] bf16 and meta [d_out][d_in/8] bytes: armor_pack_nm with ARMOR_BF16
 *   prepared armor_apply_prepared_bytes(d_out, d_in) bytes, device, 16-byte aligned; opaque
 *            (per 64 input columns: the 64 B of values and the 8 B of index bits of every row,
 *            rows padded to a multiple of 256).
 * armor_apply_packed:
 *   X        [n_tokens][d_in]  bf16, row-major (one token per row)
 *   A_bf16   [d_out/d_block][d_block][d_block] bf16, B_bf16 [d_in/d_block][d_block][d_block] bf16:
 *            the wrappers of armor_factorize_layer (with opts->denormalize = 1 when the layer is
 *            to reproduce W rather than W-bar) converted by armor_to_bf16
 *   Y        [n_tokens][d_out] bf16, row-major
 *   ws       armor_apply_workspace_bytes(n_tokens, d_in) bytes (holds B X in bf16)
 * Arithmetic: bf16 operands, fp32 accumulation; the two intermediates B x and S (B x) are rounded
 * to bf16 (round to nearest even) before the next product, Y is rounded once at the end.
 * Supported: N:M = 2:4 (the pattern the structured-sparse matrix instruction takes), d_in a multiple
 * of 64; anything else returns ARMOR_ERR_UNSUPPORTED (d_block outside {32, 64, 128, 256}:
 * ARMOR_ERR_SHAPE, as everywhere).  All pointers
 * are device pointers, 16-byte aligned; asynchronous on the stream; n_tokens = 0 is a no-op.
 */
armor_status armor_to_bf16(const float *in, int64_t n, void *out_bf16, void *hip_stream);
size_t armor_apply_prepared_bytes(int64_t d_out, int64_t d_in);
armor_status armor_apply_prepare(const void *values, const uint8_t *meta, int64_t d_out, int64_t d_in, int N, int M,
                                 void *prepared, size_t prepared_bytes, void *hip_stream);
size_t armor_apply_workspace_bytes(int64_t n_tokens, int64_t d_in);
armor_status armor_apply_packed(const void *X, int64_t n_tokens, const void *A_bf16, const void *prepared,
                                const void *B_bf16, int64_t d_out, int64_t d_in, int64_t d_block, int N, int M,
                                void *Y, void *ws, size_t ws_bytes, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* ARMOR_H */
