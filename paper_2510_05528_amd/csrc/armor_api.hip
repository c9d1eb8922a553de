// C ABI of the library (see include/armor.h) and the host-side iteration driver (Alg. 1).
// The driver only validates, carves the caller's workspace and enqueues kernels on one stream:
// nothing is allocated, nothing synchronises, every scalar of the iteration (step sizes, losses)
// is produced and consumed on the device.
#include "../../include/armor.h"
#include "armor_internal.h"

#include <algorithm>
#include <cstring>
#include <mutex>
#include <vector>

using namespace armor;

namespace {

thread_local int g_last_hip_error = 0;

armor_status check_hip() {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        g_last_hip_error = (int)e;
        return ARMOR_ERR_DEVICE;
    }
    return ARMOR_OK;
}

// Optional per-kernel timing with HIP events recorded on the caller's stream around each
// instrumented launch (host-side bookkeeping only; off by default).  A scope that directly follows
// another scope on the same stream (nothing enqueued in between) may take that scope's closing
// event as its opening one: half as many event packets between the kernels of the iteration loop,
// and a launch's time then runs from the end of its predecessor to its own end.
struct Profiler {
    bool on = false;
    std::vector<hipEvent_t> pool;
    size_t used = 0;
    struct Rec { int kind; size_t e0, e1; };
    std::vector<Rec> recs;
    static constexpr size_t kMaxEvents = 1 << 15;
    long last_end = -1;            // closing event of the most recent scope
    hipStream_t last_stream = nullptr;
    long take(hipStream_t s) {
        if (used >= pool.size()) {
            if (pool.size() >= kMaxEvents) return -1;
            hipEvent_t a;
            // timing-only events: no system-scope fence (cache write-back + invalidate) when they
            // complete, which would otherwise sit between every two instrumented kernels
            if (hipEventCreateWithFlags(&a, hipEventDisableSystemFence) != hipSuccess) return -1;
            pool.push_back(a);
        }
        size_t e = used++;
        (void)hipEventRecord(pool[e], s);
        return (long)e;
    }
    long begin(hipStream_t s, bool follows) {
        if (!on) return -1;
        if (follows && last_end >= 0 && last_stream == s) return last_end;
        return take(s);
    }
    void end(int kind, long e0, hipStream_t s) {
        if (e0 < 0) return;
        long e1 = take(s);
        if (e1 < 0) return;
        recs.push_back({kind, (size_t)e0, (size_t)e1});
        last_end = e1;
        last_stream = s;
    }
    void reset() { recs.clear(); used = 0; last_end = -1; }
};
Profiler g_prof;

struct ProfScope {
    int kind;
    long e0;
    hipStream_t s;
    ProfScope(int k, hipStream_t st, bool follows = false) : kind(k), e0(g_prof.begin(st, follows)), s(st) {}
    ~ProfScope() { g_prof.end(kind, e0, s); }
};

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int device_cus() {
    static int cus = 0;
    if (cus == 0) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
            cus = n;
        else
            cus = 256;
    }
    return cus;
}

// Workgroups of a chain kernel that are resident at once (one per CU at b = 128: LDS-bound).
int chain_slots(int b) { return device_cus() * (b >= 128 ? 1 : 2); }

// How many chunks to split the accumulation axis of a gradient phase into: workgroup (k, c) walks
// `chunk` blocks and leaves one b x b partial.  Cost model in units of one block's chain time:
// rounds * (chunk + a small charge for writing the partial); finer splits balance the tail.
int choose_nsplit(int n_outer, int n_inner, int b, int slots = 0) {
    if (slots == 0) slots = chain_slots(b);
    int best = 1;
    double best_cost = 1e300;
    for (int ns = 1; ns <= n_inner && ns <= chain_max_nsplit(); ++ns) {
        int chunk = (n_inner + ns - 1) / ns;
        int eff = (n_inner + chunk - 1) / chunk; // splits that actually hold work
        if (eff != ns) continue;
        long wgs = (long)n_outer * ns;
        long rounds = (wgs + slots - 1) / slots;
        double cost = (double)rounds * (chunk + 0.08);
        if (cost < best_cost - 1e-12) { best_cost = cost; best = ns; }
    }
    return best;
}

struct Carver {
    char *base;
    size_t off;
    explicit Carver(void *p) : base(reinterpret_cast<char *>(p)), off(0) {}
    template <typename T> T *take(size_t count) {
        off = (off + 255) & ~size_t(255);
        T *r = base ? reinterpret_cast<T *>(base + off) : nullptr;
        off += count * sizeof(T);
        return r;
    }
};

struct FactorWs {
    float *Sp; // S' = A C handed from the B step to the W' step (sequential variant; at d_block < 128 in N:M mode only)
    float *Wbar, *G, *D, *gpart, *beta_part, *loss_part, *loss_part2, *K, *AtA, *colnorm2, *fro2A, *fro2K, *cn_partial,
        *r1, *r2;
    double *tol_loss; // the loss the tolerance test of Alg. 1 reads back
    uint8_t *mask;
    void *unstructured;
    float *big_scratch;
    float *stream_scratch; // one b x b tile per workgroup of a gradient phase (streamed-operand form, d_block 128)
    float *mA, *vA, *mB, *vB, *mC, *vC, *gBpart;
    WrapperPlanes planes; // bf16 pieces of the wrapper-sized operands (d_block 128, sequential variant)
    bool use_planes;
    int nsA, nsB, cn_chunks;
    size_t bytes;
};

int colnorm_chunks(int64_t d_out) { return (int)std::max<int64_t>(1, std::min<int64_t>(64, d_out / 64)); }

armor_status validate_shape(int64_t d_out, int64_t d_in, int64_t b) {
    if (d_out <= 0 || d_in <= 0 || b <= 0) return ARMOR_ERR_SHAPE;
    if (d_out % b != 0 || d_in % b != 0) return ARMOR_ERR_SHAPE;
    if (b != 32 && b != 64 && b != 128 && b != 256) return ARMOR_ERR_SHAPE;
    if (d_out / b > 1 << 20 || d_in / b > 1 << 20 || (d_out / b) * (d_in / b) > (int64_t)1 << 30) return ARMOR_ERR_SHAPE;
    // the chain kernels address inside a block row with 32-bit byte offsets: b rows of d_in fp32 values
    if (b * d_in > (int64_t)1 << 29) return ARMOR_ERR_SHAPE;
    return ARMOR_OK;
}

Dims make_dims(int64_t d_out, int64_t d_in, int64_t b) {
    Dims d;
    d.d_out = d_out; d.d_in = d_in; d.b = (int)b;
    d.nbi = (int)(d_out / b); d.nbj = (int)(d_in / b); d.nblocks = d.nbi * d.nbj;
    return d;
}

FactorWs carve_factor(void *ws, const Dims &d, int mask_group, const armor_opts *opts) {
    FactorWs f;
    Carver c(ws);
    const size_t P = (size_t)d.d_out * d.d_in, bb = (size_t)d.b * d.b;
    const bool adam = opts && opts->variant == 1, unstr = opts && opts->sparsity == 1;
    // at d_block 128 the gradient phases run with two workgroups per CU (streamed-operand form)
    const bool stream = d.b == 128;
    const int slots = chain_slots(d.b) * (stream ? (adam ? 2 : stream_wgs_per_cu()) : 1);
    f.nsA = choose_nsplit(d.nbi, d.nbj, d.b, slots);
    f.nsB = choose_nsplit(d.nbj, d.nbi, d.b, slots);
    f.cn_chunks = colnorm_chunks(d.d_out);
    f.Wbar = c.take<float>(P);
    f.G = c.take<float>(P);
    f.Sp = (!adam && (d.b >= 128 || !unstr)) ? c.take<float>(P) : nullptr;
    f.D = c.take<float>(d.d_in);
    f.gpart = c.take<float>(std::max((size_t)d.nbi * f.nsA, (size_t)d.nbj * f.nsB) * bb);
    f.stream_scratch = stream ? c.take<float>(std::max((size_t)d.nbi * f.nsA, (size_t)d.nbj * f.nsB) * bb) : nullptr;
    f.beta_part = c.take<float>(d.nblocks);
    f.loss_part = c.take<float>(d.nblocks);
    f.loss_part2 = c.take<float>(d.nblocks);
    f.tol_loss = c.take<double>(2);
    f.K = c.take<float>((size_t)d.nbj * bb);
    f.AtA = c.take<float>((size_t)d.nbi * bb);
    f.colnorm2 = c.take<float>(d.d_out);
    f.fro2A = c.take<float>((size_t)d.nbi * gram_parts(d.b));
    f.fro2K = c.take<float>((size_t)d.nbj * gram_parts(d.b));
    f.cn_partial = c.take<float>(((size_t)f.cn_chunks + 1) * d.d_in); // chunk sums, then 1/r1
    f.r1 = c.take<float>(d.d_in);
    f.r2 = c.take<float>(d.d_out);
    f.mask = c.take<uint8_t>((size_t)d.d_out * (d.d_in / mask_group));
    f.unstructured = (opts && opts->sparsity == 1)
                         ? c.take<char>(unstructured_init_ws_bytes(d.d_out, d.d_in)) : nullptr;
    f.big_scratch = d.b > 128 ? c.take<float>(big_scratch_floats(d, chain_slots(d.b))) : nullptr;
    f.planes = WrapperPlanes{};
    f.use_planes = stream && !adam && stream_uses_planes();
    if (f.use_planes) {
        const size_t per = (size_t)3 * bb;
        f.planes.A = c.take<uint16_t>(per * d.nbi);
        f.planes.AT = c.take<uint16_t>(per * d.nbi);
        f.planes.AtA = c.take<uint16_t>(per * d.nbi);
        f.planes.B = c.take<uint16_t>(per * d.nbj);
        f.planes.BT = c.take<uint16_t>(per * d.nbj);
        f.planes.K = c.take<uint16_t>(per * d.nbj);
    }
    f.mA = f.vA = f.mB = f.vB = f.mC = f.vC = f.gBpart = nullptr;
    if (opts && opts->variant == 1) { // Adam moments (one contiguous run, zeroed together) + per-block grad_B partials
        const size_t na = (size_t)d.nbi * bb, nb = (size_t)d.nbj * bb;
        f.mA = c.take<float>(2 * na + 2 * nb + 2 * P);
        f.vA = f.mA + na; f.mB = f.vA + na; f.vB = f.mB + nb; f.mC = f.vB + nb; f.vC = f.mC + P;
        f.gBpart = c.take<float>((size_t)d.nblocks * bb);
    }
    f.bytes = (c.off + 255) & ~size_t(255);
    return f;
}

armor_status validate_nm(int N, int M, int64_t b) {
    if (M != 2 && M != 4 && M != 8) return ARMOR_ERR_SHAPE;
    if (N < 1 || N >= M) return ARMOR_ERR_SHAPE;
    if (b % M != 0) return ARMOR_ERR_SHAPE;
    return ARMOR_OK;
}

} // namespace

extern "C" {

const char *armor_status_string(armor_status s) {
    switch (s) {
    case ARMOR_OK: return "ok";
    case ARMOR_ERR_NULL: return "null pointer";
    case ARMOR_ERR_SHAPE: return "bad shape";
    case ARMOR_ERR_DTYPE: return "bad dtype";
    case ARMOR_ERR_WORKSPACE: return "workspace missing or too small";
    case ARMOR_ERR_ALIGN: return "buffer not 16-byte aligned";
    case ARMOR_ERR_DEVICE: return "HIP error";
    case ARMOR_ERR_UNSUPPORTED: return "unsupported configuration";
    case ARMOR_ERR_NONFINITE: return "non-finite entry in W or non-finite/negative loss weight";
    case ARMOR_ERR_TOO_LARGE: return "problem needs more than the fixed scratch of the allocation-free entry point";
    }
    return "unknown status";
}

int armor_last_hip_error(void) { return g_last_hip_error; }

static thread_local int64_t g_last_iterations = 0;
int64_t armor_last_iteration_count(void) { return g_last_iterations; }

armor_status armor_profile_enable(int on) {
    g_prof.on = on != 0;
    g_prof.last_end = -1;
    return ARMOR_OK;
}

armor_status armor_profile_read(double *ms_total, int64_t *launches) {
    if (!ms_total || !launches) return ARMOR_ERR_NULL;
    for (int k = 0; k < ARMOR_PROF_KINDS; ++k) { ms_total[k] = 0.0; launches[k] = 0; }
    armor_status st = ARMOR_OK;
    for (const auto &r : g_prof.recs) {
        float ms = 0.f;
        if (hipEventSynchronize(g_prof.pool[r.e1]) != hipSuccess ||
            hipEventElapsedTime(&ms, g_prof.pool[r.e0], g_prof.pool[r.e1]) != hipSuccess) {
            st = check_hip();
            if (st == ARMOR_OK) st = ARMOR_ERR_DEVICE;
            break;
        }
        ms_total[r.kind] += (double)ms;
        launches[r.kind] += 1;
    }
    g_prof.reset();
    return st;
}

size_t armor_gram_workspace_bytes(int64_t n_tokens, int64_t d_in, armor_dtype x_dtype) {
    if (n_tokens <= 0 || d_in <= 0) return 0;
    return gram_workspace_bytes(n_tokens, d_in, x_dtype == ARMOR_BF16);
}

armor_status armor_gram(const void *X, armor_dtype x_dtype, int64_t n_tokens, int64_t d_in, int64_t ldx, float *H,
                        int64_t ldh, int accumulate, void *ws, size_t ws_bytes, void *hip_stream) {
    if (!H || (!X && n_tokens > 0)) return ARMOR_ERR_NULL;
    if (x_dtype != ARMOR_F32 && x_dtype != ARMOR_BF16) return ARMOR_ERR_DTYPE;
    if (d_in <= 0 || d_in % 32 != 0 || n_tokens < 0 || ldx < d_in || ldh < d_in) return ARMOR_ERR_SHAPE;
    if (!aligned16(X) || !aligned16(H) || (ws && !aligned16(ws))) return ARMOR_ERR_ALIGN;
    {
        ProfScope ps(ARMOR_PROF_GRAM, (hipStream_t)hip_stream);
        launch_gram(X, x_dtype == ARMOR_BF16, n_tokens, d_in, ldx, H, ldh, accumulate, ws, ws ? ws_bytes : 0,
                    (hipStream_t)hip_stream);
    }
    return check_hip();
}

armor_status armor_gram_diag(const float *H, int64_t d_in, int64_t ldh, float *D, void *hip_stream) {
    if (!H || !D) return ARMOR_ERR_NULL;
    if (d_in <= 0 || ldh < d_in) return ARMOR_ERR_SHAPE;
    launch_diag(H, d_in, ldh, D, (hipStream_t)hip_stream);
    return check_hip();
}

size_t armor_gram_diag_x_workspace_bytes(int64_t n_tokens, int64_t d_in) {
    if (n_tokens < 0 || d_in <= 0) return 0;
    return (size_t)diag_x_chunks(n_tokens) * (size_t)d_in * sizeof(float) + 256;
}

armor_status armor_gram_diag_x(const void *X, armor_dtype x_dtype, int64_t n_tokens, int64_t d_in, int64_t ldx,
                               float *D, int accumulate, void *ws, size_t ws_bytes, void *hip_stream) {
    if (!D || (!X && n_tokens != 0)) return ARMOR_ERR_NULL; // an empty batch may come with a null X
    if (x_dtype != ARMOR_F32 && x_dtype != ARMOR_BF16) return ARMOR_ERR_DTYPE;
    const int vec = x_dtype == ARMOR_BF16 ? 8 : 4;
    if (d_in <= 0 || n_tokens < 0 || ldx < d_in || d_in % vec != 0 || ldx % vec != 0) return ARMOR_ERR_SHAPE;
    if (!ws || ws_bytes < armor_gram_diag_x_workspace_bytes(n_tokens, d_in)) return ARMOR_ERR_WORKSPACE;
    if ((X && !aligned16(X)) || !aligned16(ws)) return ARMOR_ERR_ALIGN;
    hipStream_t s = (hipStream_t)hip_stream;
    {
        ProfScope ps(ARMOR_PROF_DIAG_X, s);
        launch_diag_x(X, x_dtype == ARMOR_BF16, n_tokens, d_in, ldx, D, accumulate, reinterpret_cast<float *>(ws), s);
    }
    return check_hip();
}

size_t armor_normalize_workspace_bytes(int64_t d_out, int64_t d_in) {
    if (d_out <= 0 || d_in <= 0) return 0;
    return ((size_t)colnorm_chunks(d_out) + 1) * (size_t)d_in * sizeof(float) + 256;
}

armor_status armor_normalize(const void *W, armor_dtype w_dtype, int64_t d_out, int64_t d_in, float *Wbar, float *r1,
                             float *r2, void *ws, size_t ws_bytes, void *hip_stream) {
    if (!W || !Wbar || !r1 || !r2) return ARMOR_ERR_NULL;
    if (w_dtype != ARMOR_F32 && w_dtype != ARMOR_BF16) return ARMOR_ERR_DTYPE;
    if (d_out <= 0 || d_in <= 0) return ARMOR_ERR_SHAPE;
    if (!ws || ws_bytes < armor_normalize_workspace_bytes(d_out, d_in)) return ARMOR_ERR_WORKSPACE;
    if (!aligned16(W) || !aligned16(Wbar) || !aligned16(ws)) return ARMOR_ERR_ALIGN;
    hipStream_t s = (hipStream_t)hip_stream;
    Carver c(ws);
    int chunks = colnorm_chunks(d_out);
    float *partial = c.take<float>(((size_t)chunks + 1) * d_in); // chunk sums, then 1/r1
    {
        ProfScope ps(ARMOR_PROF_NORMALIZE, s);
        launch_colnorm(W, w_dtype == ARMOR_BF16, d_out, d_in, partial, chunks, r1, s);
        launch_rownorm_scale(W, w_dtype == ARMOR_BF16, d_out, d_in, partial + (size_t)chunks * d_in, r2, Wbar, s);
    }
    return check_hip();
}

// Scratch layout of the proxy-loss evaluation: the loss weights D, identity wrappers standing in for a
// NULL A / B, one partial loss per block, and at d_block 256 the chain scratch of `big_wgs` workgroups.
struct LossWs {
    float *D, *Ai, *Bi, *loss_part, *big;
    size_t bytes;
};

static LossWs carve_loss(void *base, const Dims &d, bool need_Ai, bool need_Bi, int big_wgs) {
    LossWs w;
    Carver c(base);
    w.D = c.take<float>(d.d_in);
    w.Ai = need_Ai ? c.take<float>((size_t)d.nbi * d.b * d.b) : nullptr;
    w.Bi = need_Bi ? c.take<float>((size_t)d.nbj * d.b * d.b) : nullptr;
    w.loss_part = c.take<float>(d.nblocks);
    w.big = d.b > 128 ? c.take<float>(big_scratch_floats(d, big_wgs)) : nullptr;
    w.bytes = c.off + 256;
    return w;
}

// Enqueues Eq. 2 on scratch carved by carve_loss.  Every scratch location is written before it is read.
static armor_status enqueue_proxy_loss(const float *Wbar, const float *A, const float *S, const float *B, const float *H,
                                       int64_t ldh, const Dims &d, double *loss_out, const LossWs &w, int big_wgs,
                                       hipStream_t s) {
    if (ldh > 0) launch_diag(H, d.d_in, ldh, w.D, s);
    else if (hipMemcpyAsync(w.D, H, sizeof(float) * d.d_in, hipMemcpyDeviceToDevice, s) != hipSuccess) return check_hip();
    if (!A) { launch_init_identity(w.Ai, d.nbi, d.b, s); A = w.Ai; }
    if (!B) { launch_init_identity(w.Bi, d.nbj, d.b, s); B = w.Bi; }
    if (d.b > 128)
        launch_big_phase_A(d, Wbar, S, A, B, w.D, choose_nsplit(d.nbi, d.nbj, d.b), nullptr, nullptr, w.loss_part, true,
                           big_wgs, w.big, s);
    else
        launch_phase_A(d, Wbar, S, A, B, w.D, choose_nsplit(d.nbi, d.nbj, d.b), nullptr, nullptr, w.loss_part, true, nullptr,
                       nullptr, s);
    launch_sum_to_double(w.loss_part, d.nblocks, loss_out, s);
    return check_hip();
}

size_t armor_proxy_loss_workspace_bytes(int64_t d_out, int64_t d_in, int64_t d_block) {
    if (validate_shape(d_out, d_in, d_block) != ARMOR_OK) return 0;
    Dims d = make_dims(d_out, d_in, d_block);
    return carve_loss(nullptr, d, true, true, chain_slots(d.b)).bytes;
}

armor_status armor_proxy_loss(const float *Wbar, const float *A, const float *S, const float *B, const float *H,
                              int64_t ldh, int64_t d_out, int64_t d_in, int64_t d_block, double *loss_out, void *ws,
                              size_t ws_bytes, void *hip_stream) {
    if (!Wbar || !S || !H || !loss_out) return ARMOR_ERR_NULL;
    armor_status st = validate_shape(d_out, d_in, d_block);
    if (st != ARMOR_OK) return st;
    if (ldh != 0 && ldh < d_in) return ARMOR_ERR_SHAPE;
    if (!ws || ws_bytes < armor_proxy_loss_workspace_bytes(d_out, d_in, d_block)) return ARMOR_ERR_WORKSPACE;
    if (!aligned16(Wbar) || !aligned16(S) || !aligned16(ws) || (A && !aligned16(A)) || (B && !aligned16(B)))
        return ARMOR_ERR_ALIGN;
    Dims d = make_dims(d_out, d_in, d_block);
    const int big_wgs = chain_slots(d.b);
    return enqueue_proxy_loss(Wbar, A, S, B, H, ldh, d, loss_out, carve_loss(ws, d, true, true, big_wgs), big_wgs,
                              (hipStream_t)hip_stream);
}

// ---- loss against the whole Gram matrix: tr(R H R^T) ------------------------------------------------
// Scratch: all-ones loss weights (the residual pass then leaves R itself), identity wrappers for a NULL A / B,
// the per-block losses of that pass (unused), chain scratch at d_block 256, R, one partial per output tile.
struct FullHWs {
    LossWs l;
    float *R, *part;
    size_t bytes;
};

static FullHWs carve_full_h(void *base, const Dims &d, int big_wgs) {
    FullHWs w;
    w.l = carve_loss(base, d, true, true, big_wgs);
    Carver c(base);
    c.off = w.l.bytes;
    w.R = c.take<float>((size_t)d.d_out * d.d_in);
    w.part = c.take<float>((size_t)full_h_parts(d.d_out, d.d_in));
    w.bytes = c.off + 256;
    return w;
}

size_t armor_proxy_loss_full_h_workspace_bytes(int64_t d_out, int64_t d_in, int64_t d_block) {
    if (validate_shape(d_out, d_in, d_block) != ARMOR_OK) return 0;
    Dims d = make_dims(d_out, d_in, d_block);
    return carve_full_h(nullptr, d, chain_slots(d.b)).bytes;
}

armor_status armor_proxy_loss_full_h(const float *Wbar, const float *A, const float *S, const float *B, const float *H,
                                     int64_t ldh, int64_t d_out, int64_t d_in, int64_t d_block, double *loss_out,
                                     void *ws, size_t ws_bytes, void *hip_stream) {
    if (!Wbar || !S || !H || !loss_out) return ARMOR_ERR_NULL;
    armor_status st = validate_shape(d_out, d_in, d_block);
    if (st != ARMOR_OK) return st;
    if (ldh < d_in || ldh % 4 != 0 || ldh > INT32_MAX) return ARMOR_ERR_SHAPE; // 16-byte row loads of H
    if (!ws || ws_bytes < armor_proxy_loss_full_h_workspace_bytes(d_out, d_in, d_block)) return ARMOR_ERR_WORKSPACE;
    if (!aligned16(Wbar) || !aligned16(S) || !aligned16(H) || !aligned16(ws) || (A && !aligned16(A)) ||
        (B && !aligned16(B)))
        return ARMOR_ERR_ALIGN;
    Dims d = make_dims(d_out, d_in, d_block);
    hipStream_t s = (hipStream_t)hip_stream;
    const int big_wgs = chain_slots(d.b);
    const FullHWs w = carve_full_h(ws, d, big_wgs);
    launch_fill(w.l.D, d.d_in, 1.f, s);
    if (!A) { launch_init_identity(w.l.Ai, d.nbi, d.b, s); A = w.l.Ai; }
    if (!B) { launch_init_identity(w.l.Bi, d.nbj, d.b, s); B = w.l.Bi; }
    // the loss-only forward pass with unit weights leaves R = Wbar - A S B in its gradient argument
    {
        ProfScope ps(ARMOR_PROF_RESIDUAL, s);
        if (d.b > 128)
            launch_big_residual(d, Wbar, S, A, B, w.l.D, choose_nsplit(d.nbi, d.nbj, d.b), w.R, w.l.loss_part, big_wgs,
                                w.l.big, s);
        else
            launch_residual(d, Wbar, S, A, B, w.l.D, choose_nsplit(d.nbi, d.nbj, d.b), w.R, w.l.loss_part, s);
    }
    {
        ProfScope ps(ARMOR_PROF_FULL_H, s);
        launch_full_h_loss(w.R, d.d_out, d.d_in, H, ldh, w.part, chain_slots(128), s);
    }
    launch_sum_to_double(w.part, (int)full_h_parts(d.d_out, d.d_in), loss_out, s);
    return check_hip();
}

// ---- allocation-free evaluation of Eq. 2 ---------------------------------------------------------
// The scratch of armor_proxy_loss_noalloc lives in the library's own device image, one copy per GPU,
// held until the process ends.  Host code must not use the array's name as an address: the device
// address is looked up once per device and only that pointer is handed to kernels and copies.
#define ARMOR_NOALLOC_SCRATCH_BYTES ((size_t)32 << 20)
static __device__ __align__(256) unsigned char scratch[ARMOR_NOALLOC_SCRATCH_BYTES];

static armor_status noalloc_scratch(void **out) {
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static void *ptr[kMaxDevices] = {};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        armor_status st = check_hip();
        return st != ARMOR_OK ? st : ARMOR_ERR_DEVICE;
    }
    std::lock_guard<std::mutex> lock(mu);
    if (ptr[dev] == nullptr) { // first call on this device (the current one): resolve its copy of the array
        void *p = nullptr;
        hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || p == nullptr) {
            g_last_hip_error = (int)e;
            (void)hipGetLastError();
            return ARMOR_ERR_DEVICE;
        }
        ptr[dev] = p;
    }
    *out = ptr[dev];
    return ARMOR_OK;
}

armor_status armor_proxy_loss_noalloc(const float *Wbar, const float *A, const float *S, const float *B,
                                      const float *H, int64_t ldh, int64_t d_out, int64_t d_in, int64_t d_block,
                                      double *loss_out, void *hip_stream) {
    if (!Wbar || !S || !H || !loss_out) return ARMOR_ERR_NULL;
    armor_status st = validate_shape(d_out, d_in, d_block);
    if (st != ARMOR_OK) return st;
    if (ldh != 0 && ldh < d_in) return ARMOR_ERR_SHAPE;
    if (!aligned16(Wbar) || !aligned16(S) || (A && !aligned16(A)) || (B && !aligned16(B))) return ARMOR_ERR_ALIGN;
    Dims d = make_dims(d_out, d_in, d_block);
    // at d_block 256 as many workgroups as the fixed scratch has room for (each needs 2 b^2 floats)
    int big_wgs = chain_slots(d.b);
    if (d.b > 128) {
        const size_t fixed = carve_loss(nullptr, d, !A, !B, 0).bytes, per_wg = big_scratch_floats(d, 1) * sizeof(float);
        if (fixed + per_wg > ARMOR_NOALLOC_SCRATCH_BYTES) return ARMOR_ERR_TOO_LARGE;
        big_wgs = (int)std::min<size_t>((size_t)big_wgs, (ARMOR_NOALLOC_SCRATCH_BYTES - fixed) / per_wg);
    }
    if (carve_loss(nullptr, d, !A, !B, big_wgs).bytes > ARMOR_NOALLOC_SCRATCH_BYTES) return ARMOR_ERR_TOO_LARGE;
    void *base = nullptr;
    st = noalloc_scratch(&base);
    if (st != ARMOR_OK) return st;
    return enqueue_proxy_loss(Wbar, A, S, B, H, ldh, d, loss_out, carve_loss(base, d, !A, !B, big_wgs), big_wgs,
                              (hipStream_t)hip_stream);
}

size_t armor_factorize_workspace_bytes(int64_t d_out, int64_t d_in, int64_t d_block, int N, int M,
                                       const armor_opts *opts) {
    if (validate_shape(d_out, d_in, d_block) != ARMOR_OK) return 0;
    const bool unstructured = opts && opts->sparsity == 1;
    if (!unstructured && validate_nm(N, M, d_block) != ARMOR_OK) return 0;
    Dims d = make_dims(d_out, d_in, d_block);
    FactorWs f = carve_factor(nullptr, d, unstructured ? 8 : M, opts);
    return f.bytes;
}

armor_status armor_factorize_layer(const void *W, armor_dtype w_dtype, const float *H, int64_t ldh, int64_t d_out,
                                   int64_t d_in, int64_t d_block, int N, int M, int n_iters, const armor_opts *opts,
                                   float *A, float *S, float *B, uint8_t *mask_bits, float *r1, float *r2,
                                   double *loss_trace, double *loss_cont_trace, double *eta_trace,
                                   int32_t *mask_changes, void *ws, size_t ws_bytes, void *hip_stream) {
    if (!W || !H || !A || !S || !B) return ARMOR_ERR_NULL;
    if (w_dtype != ARMOR_F32 && w_dtype != ARMOR_BF16) return ARMOR_ERR_DTYPE;
    armor_status st = validate_shape(d_out, d_in, d_block);
    if (st != ARMOR_OK) return st;
    armor_opts o;
    std::memset(&o, 0, sizeof(o));
    if (opts) o = *opts;
    const bool unstructured = o.sparsity == 1;
    if (o.sparsity != 0 && o.sparsity != 1) return ARMOR_ERR_SHAPE;
    if (o.selection < 0 || o.selection > 3 || o.variant < 0 || o.variant > 1) return ARMOR_ERR_SHAPE;
    if (o.lr < 0 || o.adam_beta1 < 0 || o.adam_beta1 >= 1 || o.adam_beta2 < 0 || o.adam_beta2 >= 1 || o.adam_eps < 0)
        return ARMOR_ERR_SHAPE;
    if (!unstructured) {
        st = validate_nm(N, M, d_block);
        if (st != ARMOR_OK) return st;
    } else if (o.unstructured_keep < 0 || o.unstructured_keep > d_out * d_in) {
        return ARMOR_ERR_SHAPE;
    }
    if (n_iters < 0 || (ldh != 0 && ldh < d_in)) return ARMOR_ERR_SHAPE;
    if (unstructured && d_in % 8 != 0) return ARMOR_ERR_SHAPE;
    if (o.init_from_outputs < 0 || o.init_from_outputs > 1 || o.check_finite < 0 || o.check_finite > 1 ||
        o.iter_offset < 0 || o.iter_offset + n_iters >= ((int64_t)1 << 31))
        return ARMOR_ERR_SHAPE;
    // the selection counter (iteration, block, group) must fit in 63 bits
    if (!unstructured && (double)(o.iter_offset + n_iters + 1) * ((double)d_out * (double)d_in / M) >= 4.0e18)
        return ARMOR_ERR_SHAPE;
    if (o.init_from_outputs && !mask_bits) return ARMOR_ERR_NULL;
    if (!(o.tol >= 0.0) || o.tol > 1.0) return ARMOR_ERR_SHAPE; // (a NaN fails the first test)
    if (o.tol > 0.0 && o.variant == 1) return ARMOR_ERR_UNSUPPORTED;
    const int mask_group = unstructured ? 8 : M;
    Dims d = make_dims(d_out, d_in, d_block);
    if (!ws) return ARMOR_ERR_WORKSPACE;
    FactorWs f = carve_factor(ws, d, mask_group, &o);
    if (ws_bytes < f.bytes) return ARMOR_ERR_WORKSPACE;
    if (!aligned16(W) || !aligned16(A) || !aligned16(S) || !aligned16(B) || !aligned16(ws) || (ldh > 0 && !aligned16(H)))
        return ARMOR_ERR_ALIGN;
    hipStream_t s = (hipStream_t)hip_stream;
    uint8_t *mask = mask_bits ? mask_bits : f.mask;
    float *r1p = r1 ? r1 : f.r1, *r2p = r2 ? r2 : f.r2;

    // weights of Eq. 2
    if (ldh > 0) launch_diag(H, d_in, ldh, f.D, s);
    else if (hipMemcpyAsync(f.D, H, sizeof(float) * d_in, hipMemcpyDeviceToDevice, s) != hipSuccess) return check_hip();
    if (o.check_finite) { // optional validation: the only place the call waits for the device
        int32_t *flag = reinterpret_cast<int32_t *>(f.beta_part), bad = 0;
        launch_zero(f.beta_part, 1, s);
        launch_count_nonfinite(W, w_dtype == ARMOR_BF16, d_out * d_in, f.D, d_in, flag, s);
        if (hipMemcpyAsync(&bad, flag, sizeof(bad), hipMemcpyDeviceToHost, s) != hipSuccess ||
            hipStreamSynchronize(s) != hipSuccess) {
            st = check_hip();
            return st != ARMOR_OK ? st : ARMOR_ERR_DEVICE;
        }
        if (bad != 0) return ARMOR_ERR_NONFINITE;
    }
    if (mask_changes && n_iters > 0) launch_zero(reinterpret_cast<float *>(mask_changes), n_iters, s);
    // Alg. 1: normalise, initialise
    {
        ProfScope ps(ARMOR_PROF_NORMALIZE, s);
        launch_colnorm(W, w_dtype == ARMOR_BF16, d_out, d_in, f.cn_partial, f.cn_chunks, r1p, s);
        launch_rownorm_scale(W, w_dtype == ARMOR_BF16, d_out, d_in, f.cn_partial + (size_t)f.cn_chunks * d_in, r2p, f.Wbar, s);
    }
    if (!o.init_from_outputs) {
        launch_init_identity(A, d.nbi, d.b, s);
        launch_init_identity(B, d.nbj, d.b, s);
        ProfScope ps(ARMOR_PROF_INIT, s);
        if (unstructured)
            launch_unstructured_init(f.Wbar, f.D, d_out, d_in, o.unstructured_keep, S, mask,
                                     reinterpret_cast<uint32_t *>(f.G), f.unstructured, s);
        else
            launch_init_nm(f.Wbar, f.D, d_out, d_in, N, M, S, mask, s);
    }
    st = check_hip();
    if (st != ARMOR_OK) return st;

    const bool big = d.b > 128;
    const int slots = chain_slots(d.b);
    const WrapperPlanes *pl = f.use_planes ? &f.planes : nullptr;
    auto run_phase_A = [&](bool loss_only) {
        if (big) launch_big_phase_A(d, f.Wbar, S, A, B, f.D, f.nsA, f.gpart, f.beta_part, f.loss_part, loss_only, slots,
                                    f.big_scratch, s);
        else launch_phase_A(d, f.Wbar, S, A, B, f.D, f.nsA, f.gpart, f.beta_part, f.loss_part, loss_only, f.stream_scratch,
                            pl, s);
    };
    if (pl) { // pieces of theta_0's wrappers
        const PlaneJob jobs[2] = {{A, d.nbi, f.planes.A, f.planes.AT}, {B, d.nbj, f.planes.B, f.planes.BT}};
        launch_make_planes(jobs, 2, s);
    }
    if (o.variant == 1) {
        const double lr = o.lr > 0 ? o.lr : 1e-4, b1 = o.adam_beta1 > 0 ? o.adam_beta1 : 0.9,
                     b2 = o.adam_beta2 > 0 ? o.adam_beta2 : 0.999, eps = o.adam_eps > 0 ? o.adam_eps : 1e-8;
        launch_zero(f.mA, 2 * ((int64_t)d.nbi + d.nbj) * d.b * d.b + 2 * d_out * d_in, s);
        for (int t = 1; t <= n_iters; ++t) {
            const int64_t t_draw = o.iter_offset + t;
            // joint Adam continuous step (Sec. 3.3.1): all three gradients at theta_{t-1}
            {
                ProfScope ps(ARMOR_PROF_PHASE_FB, s, t > 1);
                if (big) launch_big_phase_FB(d, f.Wbar, S, A, B, f.D, mask, mask_group, f.mC, f.vC, lr, b1, b2, eps, t, f.nsA,
                                             f.gpart, f.gBpart, f.loss_part, slots, f.big_scratch, s);
                else launch_phase_FB(d, f.Wbar, S, A, B, f.D, mask, mask_group, f.mC, f.vC, lr, b1, b2, eps, t, f.nsA,
                                     f.gpart, f.gBpart, f.loss_part, f.stream_scratch, s);
            }
            {
                ProfScope ps(ARMOR_PROF_SMALL, s, true);
                launch_adam_wrapper(A, f.mA, f.vA, d.nbi, d.b, f.gpart, f.nsA, lr, b1, b2, eps, t, d.nblocks, f.loss_part,
                                    loss_trace ? loss_trace + (t - 1) : nullptr, s);
                launch_adam_wrapper(B, f.mB, f.vB, d.nbj, d.b, f.gBpart, d.nbi, lr, b1, b2, eps, t, d.nblocks, nullptr,
                                    nullptr, s);
                if (!unstructured) {
                    if (big) launch_big_wrapper_grams(d, A, B, f.D, f.colnorm2, f.fro2A, f.AtA, f.K, f.fro2K, s);
                    else launch_wrapper_grams(d, A, B, f.D, f.colnorm2, f.fro2A, f.AtA, f.K, f.fro2K, nullptr, nullptr, s);
                }
            }
            if (!unstructured) {
                // sparse-core step (Alg. 3) at the updated point
                {
                    ProfScope ps(ARMOR_PROF_PHASE_GS, s, true);
                    if (big) launch_big_phase_GS(d, f.Wbar, S, A, B, f.D, f.G, f.loss_part2, slots, f.big_scratch, s);
                    else launch_phase_GS(d, f.Wbar, S, A, B, f.D, f.G, f.loss_part2, slots, s);
                }
                {
                    ProfScope ps(ARMOR_PROF_SPARSE, s, true);
                    launch_sparse_step(d, f.G, S, mask, f.K, f.colnorm2, N, M, o.selection, o.seed, t_draw, f.loss_part2,
                                       loss_cont_trace ? loss_cont_trace + (t - 1) : nullptr,
                                       mask_changes ? mask_changes + (t - 1) : nullptr, s);
                }
            }
            if ((t & 15) == 0) {
                st = check_hip();
                if (st != ARMOR_OK) return st;
            }
        }
    }
    int iters_done = n_iters;
    double L0 = 0.0, Lprev = 0.0; // host copies of L_0 and L_{t-2} (tolerance test only)
    for (int t = 1; o.variant == 0 && t <= n_iters; ++t) {
        const int64_t t_draw = o.iter_offset + t;
        double *eta_t = eta_trace ? eta_trace + 3 * (size_t)(t - 1) : nullptr;
        // continuous step (Alg. 2), each gradient at the already-updated parameters (Lemma 1)
        {
            ProfScope ps(ARMOR_PROF_PHASE_A, s, t > 1);
            run_phase_A(false);
        }
        if (o.tol > 0.0) {
            // The A phase has just left the block losses of theta_{t-1}: L_{t-1} is known now, one forward pass
            // after the iteration that produced it.  The tolerance test of Alg. 1 is the one place where the
            // loop waits for the device.
            double Lcur = 0.0;
            launch_sum_to_double(f.loss_part, d.nblocks, f.tol_loss, s);
            if (hipMemcpyAsync(&Lcur, f.tol_loss, sizeof(double), hipMemcpyDeviceToHost, s) != hipSuccess ||
                hipStreamSynchronize(s) != hipSuccess) {
                st = check_hip();
                return st != ARMOR_OK ? st : ARMOR_ERR_DEVICE;
            }
            if (t == 1) L0 = Lcur;
            else if (Lprev - Lcur <= o.tol * L0) { // iteration t - 1 moved the loss by no more than the tolerance
                iters_done = t - 1;
                break;
            }
            Lprev = Lcur;
        }
        {
            ProfScope ps(ARMOR_PROF_SMALL, s, true);
            launch_update_wrapper(A, d.nbi, d.b, f.gpart, f.nsA, f.beta_part, d.nblocks, f.loss_part,
                                  loss_trace ? loss_trace + (t - 1) : nullptr, eta_t, pl ? f.planes.A : nullptr,
                                  pl ? f.planes.AT : nullptr, s);
        }
        {
            ProfScope ps(ARMOR_PROF_PHASE_B, s, true);
            if (big) launch_big_phase_B(d, f.Wbar, S, A, B, f.D, f.nsB, f.gpart, f.beta_part, f.Sp, slots, f.big_scratch, s);
            else launch_phase_B(d, f.Wbar, S, A, B, f.D, f.nsB, f.gpart, f.beta_part, f.Sp, f.stream_scratch, pl, s);
        }
        {
            ProfScope ps(ARMOR_PROF_SMALL, s, true);
            launch_update_wrapper(B, d.nbj, d.b, f.gpart, f.nsB, f.beta_part, d.nblocks, nullptr, nullptr,
                                  eta_t ? eta_t + 1 : nullptr, pl ? f.planes.B : nullptr, pl ? f.planes.BT : nullptr, s);
            if (big) launch_big_wrapper_grams(d, A, B, f.D, f.colnorm2, f.fro2A, f.AtA, f.K, f.fro2K, s);
            else launch_wrapper_grams(d, A, B, f.D, f.colnorm2, f.fro2A, f.AtA, f.K, f.fro2K, pl ? f.planes.AtA : nullptr,
                                      pl ? f.planes.K : nullptr, s);
            if (eta_t) launch_eta_W_trace(d, f.fro2A, f.fro2K, eta_t + 2, s);
        }
        if (unstructured) {
            // Sec. 4.5: continuous step only.  W' step on the kept entries, no core-gradient follow-up.
            ProfScope ps(ARMOR_PROF_PHASE_WS, s, true);
            if (big) launch_big_phase_WS(d, f.Wbar, S, A, B, f.D, f.AtA, f.K, mask, mask_group, f.fro2A, f.fro2K, nullptr,
                                         nullptr, f.Sp, false, slots, f.big_scratch, s);
            else launch_phase_W(d, f.Wbar, S, A, B, f.D, mask, mask_group, f.fro2A, f.fro2K, f.Sp, slots, pl, s);
        } else {
            // W' step fused with the core gradient at the updated core; then the sparse-core step (Alg. 3)
            {
                ProfScope ps(ARMOR_PROF_PHASE_WS, s, true);
                if (big) launch_big_phase_WS(d, f.Wbar, S, A, B, f.D, f.AtA, f.K, mask, mask_group, f.fro2A, f.fro2K, f.G,
                                             f.loss_part2, f.Sp, true, slots, f.big_scratch, s);
                else launch_phase_WS(d, f.Wbar, S, A, B, f.D, f.AtA, f.K, mask, mask_group, f.fro2A, f.fro2K, f.G,
                                     f.loss_part2, f.Sp, slots, pl, s);
            }
            {
                ProfScope ps(ARMOR_PROF_SPARSE, s, true);
                launch_sparse_step(d, f.G, S, mask, f.K, f.colnorm2, N, M, o.selection, o.seed, t_draw, f.loss_part2,
                                   loss_cont_trace ? loss_cont_trace + (t - 1) : nullptr,
                                   mask_changes ? mask_changes + (t - 1) : nullptr, s);
            }
        }
        if ((t & 15) == 0) {
            st = check_hip();
            if (st != ARMOR_OK) return st;
        }
    }
    g_last_iterations = iters_done;
    if (iters_done < n_iters) {
        // ended by the tolerance: the outputs are theta_{iters_done}, whose loss the discarded forward pass left
        // in tol_loss; entries of iterations that did not run repeat it (step sizes: 0; mask changes are 0 already)
        if (loss_trace) launch_broadcast_double(loss_trace + iters_done, n_iters + 1 - iters_done, f.tol_loss, s);
        if (loss_cont_trace) launch_broadcast_double(loss_cont_trace + iters_done, n_iters - iters_done, f.tol_loss, s);
        if (eta_trace) launch_zero(reinterpret_cast<float *>(eta_trace + 3 * (size_t)iters_done), 6 * (int64_t)(n_iters - iters_done), s);
    } else if (loss_trace) {
        run_phase_A(true);
        launch_sum_to_double(f.loss_part, d.nblocks, loss_trace + n_iters, s);
    }
    if (unstructured && loss_trace && loss_cont_trace && n_iters > 0 &&
        hipMemcpyAsync(loss_cont_trace, loss_trace + 1, sizeof(double) * n_iters, hipMemcpyDeviceToDevice, s) != hipSuccess)
        return check_hip(); // no sparse step: the loss after the continuous step is the loss of the iterate
    if (o.denormalize) launch_denormalize(A, B, r1p, r2p, d_out, d_in, d.b, s);
    return check_hip();
}

int64_t armor_pack_meta_row_bytes(int64_t d_in, int N, int M) {
    if (d_in <= 0 || (M != 2 && M != 4 && M != 8) || N < 1 || N >= M || d_in % M != 0) return 0;
    const int field_bits = M == 2 ? 1 : (M == 4 ? 2 : 4);
    return (d_in / M * N * field_bits + 7) / 8;
}

armor_status armor_pack_nm(const float *S, const uint8_t *mask_bits, int64_t d_out, int64_t d_in, int N, int M,
                           void *values, armor_dtype v_dtype, uint8_t *meta, void *hip_stream) {
    if (!S || !mask_bits || !values || !meta) return ARMOR_ERR_NULL;
    if (v_dtype != ARMOR_F32 && v_dtype != ARMOR_BF16) return ARMOR_ERR_DTYPE;
    if (d_out <= 0 || d_in <= 0 || (M != 2 && M != 4 && M != 8) || N < 1 || N >= M || d_in % M != 0) return ARMOR_ERR_SHAPE;
    if (!aligned16(S)) return ARMOR_ERR_ALIGN;
    {
        ProfScope ps(ARMOR_PROF_PACK, (hipStream_t)hip_stream);
        launch_pack_nm(S, mask_bits, d_out, d_in, N, M, values, v_dtype == ARMOR_BF16, meta, (hipStream_t)hip_stream);
    }
    return check_hip();
}

armor_status armor_to_bf16(const float *in, int64_t n, void *out_bf16, void *hip_stream) {
    if (!in || !out_bf16) return ARMOR_ERR_NULL;
    if (n < 0) return ARMOR_ERR_SHAPE;
    if (n > 0) launch_to_bf16(in, n, out_bf16, (hipStream_t)hip_stream);
    return check_hip();
}

static armor_status validate_apply(int64_t d_out, int64_t d_in, int64_t d_block, int N, int M) {
    if (d_out <= 0 || d_in <= 0) return ARMOR_ERR_SHAPE;
    if (d_block > 0 && (d_out % d_block != 0 || d_in % d_block != 0)) return ARMOR_ERR_SHAPE;
    if (N != 2 || M != 4) return ARMOR_ERR_UNSUPPORTED;
    if (d_block > 0 && d_block != 32 && d_block != 64 && d_block != 128 && d_block != 256) return ARMOR_ERR_SHAPE;
    if (d_in % 64 != 0) return ARMOR_ERR_UNSUPPORTED;
    if (d_out >= (int64_t)1 << 31 || d_in >= (int64_t)1 << 31) return ARMOR_ERR_SHAPE;
    return ARMOR_OK;
}

size_t armor_apply_prepared_bytes(int64_t d_out, int64_t d_in) {
    if (d_out <= 0 || d_in <= 0 || d_in % 64 != 0) return 0;
    return (size_t)apply_prepared_bytes(d_out, d_in);
}

armor_status armor_apply_prepare(const void *values, const uint8_t *meta, int64_t d_out, int64_t d_in, int N, int M,
                                 void *prepared, size_t prepared_bytes, void *hip_stream) {
    if (!values || !meta || !prepared) return ARMOR_ERR_NULL;
    armor_status st = validate_apply(d_out, d_in, 0, N, M);
    if (st != ARMOR_OK) return st;
    if (prepared_bytes < armor_apply_prepared_bytes(d_out, d_in)) return ARMOR_ERR_WORKSPACE;
    if (!aligned16(values) || !aligned16(meta) || !aligned16(prepared)) return ARMOR_ERR_ALIGN;
    launch_apply_prepare(values, meta, d_out, d_in, prepared, (hipStream_t)hip_stream);
    return check_hip();
}

size_t armor_apply_workspace_bytes(int64_t n_tokens, int64_t d_in) {
    if (n_tokens < 0 || d_in <= 0 || d_in % 64 != 0) return 0;
    return (size_t)apply_acts_bytes(n_tokens, d_in) + 256;
}

armor_status armor_apply_packed(const void *X, int64_t n_tokens, const void *A_bf16, const void *prepared,
                                const void *B_bf16, int64_t d_out, int64_t d_in, int64_t d_block, int N, int M,
                                void *Y, void *ws, size_t ws_bytes, void *hip_stream) {
    if (!A_bf16 || !prepared || !B_bf16) return ARMOR_ERR_NULL;
    if ((!X || !Y) && n_tokens != 0) return ARMOR_ERR_NULL; // an empty batch may come with null X, Y
    if (n_tokens < 0 || d_block <= 0) return ARMOR_ERR_SHAPE;
    armor_status st = validate_apply(d_out, d_in, d_block, N, M);
    if (st != ARMOR_OK) return st;
    if (n_tokens >= (int64_t)1 << 30) return ARMOR_ERR_SHAPE;
    if (n_tokens == 0) return ARMOR_OK;
    if (!ws || ws_bytes < armor_apply_workspace_bytes(n_tokens, d_in)) return ARMOR_ERR_WORKSPACE;
    if (!aligned16(X) || !aligned16(A_bf16) || !aligned16(prepared) || !aligned16(B_bf16) || !aligned16(Y) ||
        !aligned16(ws))
        return ARMOR_ERR_ALIGN;
    hipStream_t s = (hipStream_t)hip_stream;
    {
        ProfScope ps(ARMOR_PROF_APPLY_PRE, s);
        launch_apply_pre(X, n_tokens, d_in, (int)d_block, B_bf16, ws, s);
    }
    {
        ProfScope ps(ARMOR_PROF_APPLY_MAIN, s, true);
        if (launch_apply_main(ws, n_tokens, d_in, d_out, (int)d_block, prepared, A_bf16, Y, s) != hipSuccess)
            return ARMOR_ERR_DEVICE;
    }
    return check_hip();
}

} // extern "C"
