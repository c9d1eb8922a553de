"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element, on the
same seeded inputs.  Bars (stated by the benchmark spec): N:M structure bit-exact, mask agreement >= 99.9 %,
A / S / B relative Frobenius error <= 1e-3, losses within 0.5 % relative -- applied to the UPDATES
(theta_t - theta_0) and to the loss DECREASES, see parity_util, so that a step of the wrong size or a
kernel that does nothing fails."""
import numpy as np
import pytest

from paper_2510_05528_amd import synth
from parity_util import (assert_diagnostics_parity, assert_trace_parity, assert_update_parity, identity_blocks,
                         relfro, say)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def armor():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2510_05528_amd as armor
    armor.load_library()      # raises if the HIP library is not built: no fallback
    return armor


@pytest.fixture(scope="module")
def torch():
    import torch
    return torch


def dev(torch, a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def make_layer(d_out, d_in, n_tokens, seed, act_outliers=(0.0, 1.0)):
    W = synth.make_weight(d_out, d_in, seed=seed)
    X = synth.make_calibration(n_tokens, d_in, seed=seed, outlier_frac=act_outliers[0], outlier_scale=act_outliers[1])
    return W, X


# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("n,d_in,bf16", [(512, 256, False), (70, 96, False), (333, 384, True), (16, 32, False), (1, 64, True),
                                         (333, 512, True), (64, 256, True), (1000, 768, True), (129, 256, True),
                                         (8192, 256, True), (9000, 512, True)])
def test_gram(armor, torch, orc, n, d_in, bf16):
    say("gram", n, d_in, bf16)
    X = synth.make_calibration(n, d_in, seed=4, outlier_frac=0.02, outlier_scale=20.0)
    if bf16:
        bits = synth.to_bf16_bits(X)
        Xd = dev(torch, bits.view(np.int16)).view(torch.bfloat16)
        Xh = synth.bf16_bits_to_f32(bits)
    else:
        Xd, Xh = dev(torch, X), X
    H = armor.gram(Xd)
    ref = orc.gram(Xh)
    got = H.cpu().numpy()
    scale = np.sqrt(np.outer(np.diag(ref), np.diag(ref)))     # |H_ab| <= sqrt(H_aa H_bb)
    assert np.max(np.abs(got - ref) / scale) < 2e-5
    np.testing.assert_array_equal(got, got.T)
    # streaming: two chunks accumulate to the same matrix
    if n >= 16:
        h = n // 2
        H2 = armor.gram(Xd[:h])
        armor.gram(Xd[h:], H=H2, accumulate=True)
        assert np.max(np.abs(H2.cpu().numpy() - ref) / scale) < 2e-5
    D = armor.gram_diag(H).cpu().numpy()
    np.testing.assert_array_equal(D, np.diag(got))


@pytest.mark.parametrize("n,d_in,bf16", [(512, 256, False), (70, 96, False), (333, 384, True), (1, 64, True), (9000, 512, True),
                                         (0, 64, True)])
def test_gram_diag_x(armor, torch, orc, n, d_in, bf16):
    """The weights of Eq. 2 straight from X: against the oracle's Gram diagonal, and accumulation."""
    say("gram_diag_x", n, d_in, bf16)
    X = synth.make_calibration(max(n, 1), d_in, seed=4)[:n]
    if bf16:
        bits = synth.to_bf16_bits(X)
        Xd = dev(torch, bits.view(np.int16)).view(torch.bfloat16)
        Xh = synth.bf16_bits_to_f32(bits)
    else:
        Xd, Xh = dev(torch, X), X
    D = armor.gram_diag_x(Xd)
    idx = np.arange(d_in, dtype=np.int64)
    ref = orc.gram_entries(Xh, idx, idx) if n > 0 else np.zeros(d_in)
    np.testing.assert_allclose(D.cpu().numpy(), ref, rtol=3e-6, atol=1e-30)
    D2 = armor.gram_diag_x(Xd, D=D.clone(), accumulate=True)
    np.testing.assert_allclose(D2.cpu().numpy(), 2 * ref, rtol=3e-6, atol=1e-30)


@pytest.mark.parametrize("d_out,d_in,bf16", [(256, 256, False), (96, 160, False), (384, 640, True)])
def test_normalize(armor, torch, orc, d_out, d_in, bf16):
    say("normalize", d_out, d_in, bf16)
    W = synth.make_weight(d_out, d_in, seed=2)
    W[:, 5] = 0
    if bf16:
        bits = synth.to_bf16_bits(W)
        Wd = dev(torch, bits.view(np.int16)).view(torch.bfloat16)
        Wh = synth.bf16_bits_to_f32(bits)
    else:
        Wd, Wh = dev(torch, W), W
    Wbar, r1, r2 = armor.normalize(Wd)
    eb, e1, e2 = orc.normalize(Wh)
    np.testing.assert_allclose(r1.cpu().numpy(), e1, rtol=2e-6)
    np.testing.assert_allclose(r2.cpu().numpy(), e2, rtol=2e-6)
    np.testing.assert_allclose(Wbar.cpu().numpy(), eb, rtol=3e-6, atol=1e-12)


@pytest.mark.parametrize("d_out,d_in,b", [(64, 96, 32), (128, 192, 64), (256, 384, 128), (512, 768, 256)])
def test_proxy_loss(armor, torch, orc, d_out, d_in, b):
    say("proxy_loss", d_out, d_in, b)
    rng = np.random.default_rng(1)
    Wbar = rng.standard_normal((d_out, d_in)).astype(np.float32)
    D = (rng.random(d_in) * 5 + 0.1).astype(np.float32)
    A = (np.eye(b)[None] + 0.1 * rng.standard_normal((d_out // b, b, b))).astype(np.float32)
    B = (np.eye(b)[None] + 0.1 * rng.standard_normal((d_in // b, b, b))).astype(np.float32)
    C, _ = orc.init_nm(Wbar, D, 2, 4)
    got = armor.proxy_loss(dev(torch, Wbar), dev(torch, A), dev(torch, C), dev(torch, B), dev(torch, D)).item()
    assert got == pytest.approx(orc.proxy_loss(Wbar, A, C, B, D), rel=2e-5)
    # identity wrappers (NULL) = plain masked loss; H given as a full matrix uses only its diagonal
    H = np.diag(D) + 0.01
    np.fill_diagonal(H, D)
    got = armor.proxy_loss(dev(torch, Wbar), None, dev(torch, C), None, dev(torch, H.astype(np.float32)), d_block=b).item()
    expect = ((Wbar.astype(np.float64) - C) ** 2 * D[None, :]).sum()
    assert got == pytest.approx(expect, rel=2e-5)


@pytest.mark.parametrize("d_out,d_in,b", [(64, 96, 32), (192, 160, 32), (128, 192, 64), (256, 384, 128), (384, 256, 64),
                                          (512, 768, 256), (1024, 1536, 128)])
def test_full_gram_loss(armor, torch, orc, d_out, d_in, b):
    """tr(R H R^T) against the oracle: correlated activations (the off-diagonal part of H carries a good share of
    the value), H handed over with a padded row pitch; shapes on the 32-wide tile path and on the 128-wide one."""
    say("full_gram_loss", d_out, d_in, b)
    rng = np.random.default_rng(5)
    v = np.sign(rng.standard_normal(d_in)).astype(np.float32)
    # a factor all channels share, in the activations and (weaker) in the rows of the weight: the residual
    # then correlates with it and the off-diagonal part of H carries most of the value
    Wbar = (rng.standard_normal((d_out, d_in)) + 0.5 * rng.standard_normal((d_out, 1)) * v[None, :]).astype(np.float32)
    X = rng.standard_normal((2 * d_in, d_in)).astype(np.float32)
    X[:, ::5] *= 4.0
    X += rng.standard_normal((2 * d_in, 1)).astype(np.float32) * v[None, :]
    H = (X.astype(np.float64).T @ X.astype(np.float64)).astype(np.float32)
    D = np.diag(H).copy()
    A = (np.eye(b)[None] + 0.1 * rng.standard_normal((d_out // b, b, b))).astype(np.float32)
    B = (np.eye(b)[None] + 0.1 * rng.standard_normal((d_in // b, b, b))).astype(np.float32)
    C, _ = orc.init_nm(Wbar, D, 2, 4)
    ref = orc.proxy_loss_full_h(Wbar, A, C, B, H)
    assert abs(ref - orc.proxy_loss(Wbar, A, C, B, D)) > 0.5 * ref  # not the diagonal loss in disguise
    Hd = torch.zeros((d_in, d_in + 4), device="cuda", dtype=torch.float32)  # row pitch d_in + 4
    Hd[:, :d_in] = dev(torch, H)
    got = armor.proxy_loss_full_h(dev(torch, Wbar), dev(torch, A), dev(torch, C), dev(torch, B), Hd[:, :d_in]).item()
    assert got == pytest.approx(ref, rel=2e-5)
    # identity wrappers (NULL): R = Wbar - C
    got = armor.proxy_loss_full_h(dev(torch, Wbar), None, dev(torch, C), None, dev(torch, H), d_block=b).item()
    R = Wbar.astype(np.float64) - C
    assert got == pytest.approx(float(np.sum((R @ H.astype(np.float64)) * R)), rel=2e-5)
    # a diagonal H gives Eq. 2, and an exact factorization gives zero
    got = armor.proxy_loss_full_h(dev(torch, Wbar), dev(torch, A), dev(torch, C), dev(torch, B), dev(torch, np.diag(D).astype(np.float32))).item()
    assert got == pytest.approx(orc.proxy_loss(Wbar, A, C, B, D), rel=2e-5)
    assert armor.proxy_loss_full_h(dev(torch, Wbar), None, dev(torch, Wbar), None, dev(torch, H), d_block=b).item() == 0.0


def check_factorization(armor, torch, orc, W, D, b, N, M, n_iters, seed, selection=0, tag="", init=None, iter_offset=0):
    """One run on both sides from the same start (Eq. 3, or `init` = (A, B, C, mask) numpy arrays)."""
    d_out, d_in = W.shape
    say("factorize", tag, d_out, d_in, "b", b, N, M, "iters", n_iters, "seed", seed, "sel", selection,
        "from a given point" if init is not None else "")
    ginit = rinit = None
    if init is not None:
        A0, B0, C0, m0 = init
        ginit = dict(A=dev(torch, A0), B=dev(torch, B0), S=dev(torch, C0), mask_bits=dev(torch, armor.pack_mask(m0, M)))
        rinit = dict(A=A0, B=B0, C=C0, mask=m0)
    out = armor.factorize_layer(dev(torch, W), dev(torch, D), b, N, M, n_iters, seed=seed, selection=selection,
                                want_cont_trace=True, want_diagnostics=True, init=ginit, iter_offset=iter_offset)
    torch.cuda.synchronize()
    ref = orc.factorize_layer(W, D, b, N, M, n_iters, seed=seed, selection=selection, init=rinit, iter_offset=iter_offset)
    tr = out["loss_trace"].cpu().numpy()
    ct = out["loss_cont_trace"].cpu().numpy()
    mask = armor.unpack_mask(out["mask_bits"].cpu().numpy(), M)
    S = out["S"].cpu().numpy()
    # bit-exact structure
    assert np.all(mask.reshape(d_out, d_in // M, M).sum(-1) == N)
    assert np.all(S[mask == 0] == 0)
    agree = float((mask == ref["mask"]).mean())
    eA, eB, eS = relfro(out["A"].cpu().numpy(), ref["A"]), relfro(out["B"].cpu().numpy(), ref["B"]), relfro(S, ref["C"])
    say("   mask agreement %.6f  relF A %.2e B %.2e S %.2e  loss %.9g->%.9g (oracle %.9g)" %
        (agree, eA, eB, eS, tr[0], tr[-1], ref["loss_trace"][-1]))
    assert agree >= 0.999
    assert eA <= 1e-3 and eB <= 1e-3 and eS <= 1e-3
    # the updates: what the iterations changed, against what the oracle's iterations changed
    C0_gpu = None
    if init is None:
        A0, B0 = identity_blocks(d_out // b, b), identity_blocks(d_in // b, b)
        C0, m0 = orc.init_nm(ref["Wbar"], D, N, M)
        if n_iters > 0:     # the kernels' own theta_0 (their normalised weight differs from the oracle's by rounding)
            C0_gpu = armor.factorize_layer(dev(torch, W), dev(torch, D), b, N, M, 0)["S"].cpu().numpy()
    for name, got, want, start, sg in (("A", out["A"].cpu().numpy(), ref["A"], A0, None),
                                       ("B", out["B"].cpu().numpy(), ref["B"], B0, None), ("S", S, ref["C"], C0, C0_gpu)):
        say("   " + assert_update_parity(name, got, want, start, n_iters, start_got=sg))
    worst = assert_trace_parity(tr, ref["loss_trace"])
    if n_iters > 0:
        assert_trace_parity(np.concatenate([tr[:1], ct]), np.concatenate([ref["loss_trace"][:1], ref["loss_cont_trace"]]),
                            "loss after the continuous step")
        say("   loss decrease %.4f %% of L0; worst relative error of a decrease %.2e; groups changed per iteration %s" %
            (100 * (tr[0] - tr[-1]) / tr[0], worst, out["mask_changes"].cpu().numpy().tolist()))
        tol = 1e-6 * tr[0]
        assert np.all(np.diff(tr) <= tol)                       # Thm. 1 on the device trace
        assert np.all(ct <= tr[:-1] + tol) and np.all(tr[1:] <= ct + tol)
    assert_diagnostics_parity(out, ref, n_iters, (d_out // b) * (d_in // b))
    np.testing.assert_allclose(out["r1"].cpu().numpy(), ref["r1"], rtol=2e-6)
    np.testing.assert_allclose(out["r2"].cpu().numpy(), ref["r2"], rtol=2e-6)
    # the reported final loss is the loss of the returned factors (oracle evaluates them)
    Wbar = ref["Wbar"]
    assert tr[-1] == pytest.approx(orc.proxy_loss(Wbar, out["A"].cpu().numpy(), S, out["B"].cpu().numpy(), D), rel=1e-4)
    return out, ref


def test_factorize_config1(armor, torch, orc):
    """BASELINE config 1: 256x256 fp32, 512 calibration tokens, 2:4, d_block 32, 20 iterations, seed 0."""
    W, X = make_layer(256, 256, 512, seed=0)
    H = armor.gram(dev(torch, X))
    D = armor.gram_diag(H).cpu().numpy()
    np.testing.assert_allclose(D, np.diag(orc.gram(X)), rtol=1e-5)
    check_factorization(armor, torch, orc, W, D, 32, 2, 4, 20, seed=0, tag="cfg1")


@pytest.mark.parametrize("d_out,d_in,b,iters", [(128, 192, 64, 6), (384, 640, 128, 5), (640, 256, 128, 4), (96, 160, 32, 8)])
def test_factorize_shapes(armor, torch, orc, d_out, d_in, b, iters):
    """Several blocks in both directions, non-square block grids, every chain instantiation."""
    W, X = make_layer(d_out, d_in, 300, seed=3, act_outliers=(0.01, 20.0))
    D = np.diag(orc.gram(X)).astype(np.float32)
    check_factorization(armor, torch, orc, W, D, b, 2, 4, iters, seed=11)


@pytest.mark.parametrize("sel", [1, 2, 3])
def test_factorize_selection_modes(armor, torch, orc, sel):
    W, X = make_layer(128, 128, 200, seed=5)
    D = np.diag(orc.gram(X)).astype(np.float32)
    check_factorization(armor, torch, orc, W, D, 32, 2, 4, 6, seed=2, selection=sel)


@pytest.mark.parametrize("N,M", [(4, 8), (1, 4), (3, 4), (5, 8), (6, 8), (1, 2), (2, 8), (3, 8), (7, 8), (1, 8)])
def test_factorize_general_nm(armor, torch, orc, N, M):
    W, X = make_layer(128, 192, 200, seed=6)
    D = np.diag(orc.gram(X)).astype(np.float32)
    check_factorization(armor, torch, orc, W, D, 64, N, M, 5, seed=4)


@pytest.mark.parametrize("d_out,d_in,N,M", [(256, 384, 4, 8), (256, 384, 1, 2), (384, 256, 3, 4), (256, 256, 2, 8), (128, 128, 2, 4)])
def test_factorize_block128_patterns(armor, torch, orc, d_out, d_in, N, M):
    """d_block = 128 runs the streamed-operand chains, whose W' step takes the mask from an LDS copy with
    16, 32 or 64 bytes per block row (M = 8, 4, 2); the last case is a single block (a grid of one)."""
    W, X = make_layer(d_out, d_in, 300, seed=21, act_outliers=(0.01, 20.0))
    D = np.diag(orc.gram(X)).astype(np.float32)
    check_factorization(armor, torch, orc, W, D, 128, N, M, 4, seed=9)


@pytest.mark.parametrize("d_out,d_in,N,M,iters", [(512, 768, 2, 4, 3), (768, 256, 4, 8, 3)])
def test_factorize_block256(armor, torch, orc, d_out, d_in, N, M, iters):
    """d_block = 256 (the 70B-shaped stress config): sub-tiled chains with L2-resident scratch."""
    W, X = make_layer(d_out, d_in, 300, seed=12, act_outliers=(0.01, 20.0))
    D = np.diag(orc.gram(X)).astype(np.float32)
    check_factorization(armor, torch, orc, W, D, 256, N, M, iters, seed=5)


@pytest.mark.parametrize("d_out,d_in,b,N,M,iters", [(96, 160, 32, 2, 4, 3), (128, 192, 64, 4, 8, 3), (384, 256, 128, 2, 4, 3),
                                                    (256, 384, 128, 4, 8, 2), (512, 768, 256, 2, 4, 2), (768, 256, 256, 6, 8, 2)])
def test_step_from_a_generic_point(armor, torch, orc, d_out, d_in, b, N, M, iters):
    """Alg. 2 + Alg. 3 started from a generic feasible point (wrappers well away from the identity, random
    mask and core) instead of Eq. 3: every sub-step moves its parameter by 0.1 .. 20 % per iteration and
    masks do change, so step sizes, gradients and the refit are all visible at the 1e-3 bar."""
    W, X = make_layer(d_out, d_in, 300, seed=3, act_outliers=(0.01, 20.0))
    D = np.diag(orc.gram(X)).astype(np.float32)
    A0, B0, C0, m0 = synth.make_state(d_out, d_in, b, N, M, seed=7)
    out, ref = check_factorization(armor, torch, orc, W, D, b, N, M, iters, seed=5, init=(A0, B0, C0, m0), iter_offset=3)
    assert ref["mask_changes"].sum() > 0
    for k, start in (("A", A0), ("B", B0), ("C", C0)):
        assert relfro(ref[k], start) > 1e-3, k          # the oracle did move every parameter well beyond the bar


def rank_deficient_state(d_out, d_in, b, N, M, seed):
    """A feasible point whose every group has fewer than N distinct rows of B: the first N-1 rows of a group are
    identical (their core columns too, all kept), the N-th is on its own, the pruned M-N rows are identical.
    Identical kept columns receive identical gradients and pruned rows none, so the continuous step keeps the
    duplicates exact and EVERY pattern of the sparse-core step has a singular B' D B'^T (Eq. 7/8 with a true
    pseudo-inverse; the minimum-norm weights are unique)."""
    A, B, _, _ = synth.make_state(d_out, d_in, b, N, M, seed=seed)
    rng = np.random.default_rng(seed)
    B = B.reshape(d_in // b, b // M, M, b).copy()
    B[:, :, 1:N - 1, :] = B[:, :, 0:1, :]
    B[:, :, N + 1:, :] = B[:, :, N:N + 1, :]
    mask = np.zeros((d_out, d_in // M, M), np.uint8)
    mask[:, :, :N] = 1
    C = (rng.standard_normal((d_out, d_in // M, M)) / np.sqrt(d_in)).astype(np.float32)
    C[:, :, 1:N - 1] = C[:, :, 0:1]
    return A, B.reshape(d_in // b, b, b), (C * mask).reshape(d_out, d_in), mask.reshape(d_out, d_in)


@pytest.mark.parametrize("d_out,d_in,b,N,M", [(128, 192, 64, 4, 8), (256, 128, 128, 6, 8), (96, 160, 32, 3, 4), (128, 128, 64, 3, 8)])
def test_sparse_step_with_singular_patterns(armor, torch, orc, d_out, d_in, b, N, M):
    """The pseudo-inverse branch of Eq. 7/8 on the device: a group has three distinct rows of B, so for N >= 4
    every pattern's B' D B'^T is singular and the written weights come from the pseudo-inverse; for N = 3 the
    singular patterns only compete with the regular ones, and must lose."""
    W, X = make_layer(d_out, d_in, 300, seed=3, act_outliers=(0.01, 20.0))
    D = np.diag(orc.gram(X)).astype(np.float32)
    init = rank_deficient_state(d_out, d_in, b, N, M, seed=5)
    out, ref = check_factorization(armor, torch, orc, W, D, b, N, M, 1, seed=2, init=init)
    assert ref["mask_changes"][0] > 0
    np.testing.assert_array_equal(armor.unpack_mask(out["mask_bits"].cpu().numpy(), M), ref["mask"])
    if N >= 4:                    # three distinct rows, fewer than N: the refit groups carry equal weights on duplicates
        S, m0 = out["S"].cpu().numpy().reshape(d_out, d_in // M, M), init[3].reshape(d_out, d_in // M, M)
        changed = (ref["mask"].reshape(d_out, d_in // M, M) != m0).any(-1)
        assert np.all(S[changed][:, 0] == S[changed][:, 1])


@pytest.mark.parametrize("d_out,d_in,b,N,M", [(3072, 3072, 128, 2, 4), (4352, 4096, 256, 2, 4)])
def test_step_from_a_generic_point_many_blocks(armor, torch, orc, d_out, d_in, b, N, M):
    """The same with more blocks than resident workgroups (576 blocks of 128 on 512 slots; 272 blocks of
    256 on 256): every workgroup of a gradient phase walks a chunk of two blocks and keeps the partial
    gradient across them, the W' chain walks blocks w, w + grid.  Two iterations: the second consumes
    everything the first wrote."""
    rng = np.random.default_rng(17)
    W = synth.make_weight(d_out, d_in, seed=23)
    D = (rng.random(d_in) * 3 + 0.2).astype(np.float32)
    D[rng.choice(d_in, d_in // 200, replace=False)] *= 400.0           # outlier channels (x20 activations)
    A0, B0, C0, m0 = synth.make_state(d_out, d_in, b, N, M, seed=11)
    check_factorization(armor, torch, orc, W, D, b, N, M, 2, seed=2, init=(A0, B0, C0, m0))


def test_block128_fifty_iterations(armor, torch, orc):
    """d_block 128 over the iteration count the benchmark runs (50), element by element against the oracle."""
    W, X = make_layer(1024, 1024, 600, seed=41, act_outliers=(0.005, 20.0))
    D = np.diag(orc.gram(X)).astype(np.float32)
    check_factorization(armor, torch, orc, W, D, 128, 2, 4, 50, seed=0)


@pytest.mark.parametrize("d_out,d_in,b", [(128, 192, 64), (256, 384, 128), (512, 512, 256)])
def test_a_stopped_run_continues_bit_for_bit(armor, torch, d_out, d_in, b):
    """theta_0 is an input of Alg. 1 (opts.init_from_outputs): two iterations, then three more from the
    returned state with the iteration counter carried over, are the five-iteration run, bit for bit."""
    W, X = make_layer(d_out, d_in, 200, seed=8)
    Wd = dev(torch, W)
    Dd = dev(torch, (X.astype(np.float64) ** 2).sum(0).astype(np.float32))
    whole = armor.factorize_layer(Wd, Dd, b, 2, 4, 5, seed=1, want_diagnostics=True)
    first = armor.factorize_layer(Wd, Dd, b, 2, 4, 2, seed=1, want_diagnostics=True)
    second = armor.factorize_layer(Wd, Dd, b, 2, 4, 3, seed=1, want_diagnostics=True, init=first, iter_offset=2)
    for k in ("A", "S", "B", "mask_bits"):
        assert torch.equal(second[k], whole[k]), k
    assert torch.equal(second["loss_trace"], whole["loss_trace"][2:])
    assert torch.equal(torch.cat([first["eta_trace"], second["eta_trace"]]), whole["eta_trace"])
    assert torch.equal(torch.cat([first["mask_changes"], second["mask_changes"]]), whole["mask_changes"])
    # the caller's tensors were not touched (the binding works on copies)
    again = armor.factorize_layer(Wd, Dd, b, 2, 4, 2, seed=1)
    for k in ("A", "S", "B", "mask_bits"):
        assert torch.equal(first[k], again[k]), k


@pytest.mark.parametrize("d_out,d_in,b,unstructured", [(128, 192, 64, False), (256, 256, 32, False), (384, 256, 128, False),
                                                       (512, 512, 256, False), (128, 192, 64, True)])
def test_tolerance_stop_matches_the_oracle(armor, torch, orc, d_out, d_in, b, unstructured):
    """opts.tol, the tolerance input of Alg. 1: the run ends after the first iteration t with
    L_{t-1} - L_t <= tol * L_0, at the same t as the oracle, and what it returns is bit for bit the run of
    exactly t iterations; trace entries are cut to t."""
    W, X = make_layer(d_out, d_in, 200, seed=12)
    D = (X.astype(np.float64) ** 2).sum(0).astype(np.float32)
    n = 10
    kw = dict(sparsity=1, keep=d_out * d_in // 2) if unstructured else {}
    gkw = dict(sparsity=1, unstructured_keep=d_out * d_in // 2) if unstructured else {}
    full = orc.factorize_layer(W, D, b, 2, 4, n, seed=2, **kw)
    L = full["loss_trace"]
    dec = (L[:-1] - L[1:]) / L[0]
    # a tolerance between two consecutive decreases of the oracle's run (they shrink by 3 .. 10 % per iteration
    # here), 1.5 % or more away from both: the two sides' decreases agree to 1e-3 or better, so rounding cannot
    # move the stop
    k = 5
    assert np.all(np.diff(dec) < 0) and dec[k] < 0.98 * dec[k - 1]
    tol = float(np.sqrt(dec[k - 1] * dec[k]))
    stop = k + 1                                             # iteration k + 1 is the first within the tolerance
    say("tolerance stop", d_out, d_in, b, "tol %.3e" % tol, "expected stop after iteration", stop, "decreases", dec[:stop + 1])
    ref = orc.factorize_layer(W, D, b, 2, 4, n, seed=2, tol=tol, **kw)
    assert ref["iters_done"] == stop
    Wd, Dd = dev(torch, W), dev(torch, D)
    out = armor.factorize_layer(Wd, Dd, b, 2, 4, n, seed=2, tol=tol, want_cont_trace=True, want_diagnostics=True, **gkw)
    assert out["iters_done"] == stop
    assert out["loss_trace"].numel() == stop + 1 and out["eta_trace"].shape[0] == stop and out["mask_changes"].numel() == stop
    exact = armor.factorize_layer(Wd, Dd, b, 2, 4, stop, seed=2, want_cont_trace=True, want_diagnostics=True, **gkw)
    for key in ("A", "S", "B", "mask_bits", "loss_cont_trace", "eta_trace", "mask_changes"):
        assert torch.equal(out[key], exact[key]), key
    # (the last loss comes from the forward pass of the discarded iteration here and from the loss-only pass
    # there: the same value from two kernels at d_block 128 and 256)
    assert torch.equal(out["loss_trace"][:-1], exact["loss_trace"][:-1])
    np.testing.assert_allclose(out["loss_trace"][-1].item(), exact["loss_trace"][-1].item(), rtol=2e-6)
    assert_trace_parity(out["loss_trace"].cpu().numpy(), ref["loss_trace"])
    eye_a, eye_b = identity_blocks(d_out // b, b), identity_blocks(d_in // b, b)
    say("  ", assert_update_parity("A", out["A"].cpu().numpy(), ref["A"], eye_a, stop))
    say("  ", assert_update_parity("B", out["B"].cpu().numpy(), ref["B"], eye_b, stop))
    # tol = 0 runs everything; the joint-Adam variant cannot discard a pass and refuses a tolerance
    assert armor.factorize_layer(Wd, Dd, b, 2, 4, 3, seed=2, **gkw)["iters_done"] == 3
    with pytest.raises(armor.ArmorError, match="status 7"):
        armor.factorize_layer(Wd, Dd, b, 2, 4, 3, seed=2, tol=1e-3, variant=1, **gkw)


@pytest.mark.parametrize("b,variant", [(32, 0), (128, 0), (256, 0), (128, 1)])
def test_all_zero_weight_stays_put(armor, torch, orc, b, variant):
    """W = 0: every norm of Sec. 3.2 is replaced by 1, the core is zero, the betas of Eq. 9-10 are zero and the
    wrapper updates are skipped (sequential variant), every selection score is zero and Alg. 3 takes group 0 of each
    block.  Nothing may become NaN; the result is A = B = I, S = 0, loss 0 on both sides."""
    d_out, d_in = 2 * b, 3 * b
    W = np.zeros((d_out, d_in), dtype=np.float32)
    D = (np.random.default_rng(0).random(d_in) + 0.5).astype(np.float32)
    out = armor.factorize_layer(dev(torch, W), dev(torch, D), b, 2, 4, 3, seed=1, variant=variant, want_cont_trace=True,
                                want_diagnostics=variant == 0)
    torch.cuda.synchronize()
    f = orc.factorize_layer_adam if variant == 1 else orc.factorize_layer
    ref = f(W, D, b, 2, 4, 3, seed=1)
    for k, rk in (("A", "A"), ("B", "B"), ("S", "C")):
        got = out[k].cpu().numpy()
        assert np.all(np.isfinite(got)), k
        np.testing.assert_array_equal(got, ref[rk])
    np.testing.assert_array_equal(out["A"].cpu().numpy(), identity_blocks(d_out // b, b))
    assert float(out["loss_trace"].abs().max()) == 0.0 and float(out["loss_cont_trace"].abs().max()) == 0.0
    mask = armor.unpack_mask(out["mask_bits"].cpu().numpy(), 4)
    assert np.all(mask.reshape(d_out, d_in // 4, 4).sum(-1) == 2)
    if variant == 0:
        eta = out["eta_trace"].cpu().numpy()
        assert np.all(eta[:, :2] == 0.0)                      # beta_A = beta_B = 0: steps skipped, reported as 0
        np.testing.assert_allclose(eta, ref["etas"], rtol=1e-5)   # beta_W' = 2 ||I|| ||D|| is not zero
        assert np.array_equal(out["mask_changes"].cpu().numpy(), ref["mask_changes"])
    np.testing.assert_array_equal(out["r1"].cpu().numpy(), np.ones(d_in, dtype=np.float32))


def test_check_finite_rejects_bad_inputs(armor, torch):
    """opts.check_finite: NaN/Inf in W, NaN/Inf/negative loss weights -> ARMOR_ERR_NONFINITE (status 8),
    outputs untouched; clean inputs pass and give the same result as without the check."""
    W, X = make_layer(128, 128, 100, seed=9)
    D = (X.astype(np.float64) ** 2).sum(0).astype(np.float32)
    good = armor.factorize_layer(dev(torch, W), dev(torch, D), 32, 2, 4, 2, seed=1)
    checked = armor.factorize_layer(dev(torch, W), dev(torch, D), 32, 2, 4, 2, seed=1, check_finite=True)
    for k in ("A", "S", "B", "mask_bits", "loss_trace"):
        assert torch.equal(good[k], checked[k]), k
    for what, idx, val in (("W", (5, 7), np.nan), ("W", (127, 127), np.inf), ("D", 3, np.nan), ("D", 127, -1.0),
                           ("D", 0, np.inf)):
        Wb, Db = W.copy(), D.copy()
        (Wb if what == "W" else Db)[idx] = val
        with pytest.raises(armor.ArmorError, match="status 8"):
            armor.factorize_layer(dev(torch, Wb), dev(torch, Db), 32, 2, 4, 2, seed=1, check_finite=True)
    # bf16 weights take the same path
    Wb = torch.from_numpy(W).to("cuda:0").to(torch.bfloat16)
    Wb[3, 3] = float("nan")
    with pytest.raises(armor.ArmorError, match="status 8"):
        armor.factorize_layer(Wb, dev(torch, D), 32, 2, 4, 1, check_finite=True)


@pytest.mark.parametrize("d_out,d_in,b,keep_frac", [(128, 192, 64, 0.5), (256, 256, 128, 0.5), (512, 512, 256, 0.5), (96, 160, 32, 0.3)])
def test_factorize_unstructured(armor, torch, orc, d_out, d_in, b, keep_frac):
    """50 % unstructured: global top-k initial mask, continuous step only (Sec. 4.5)."""
    W, X = make_layer(d_out, d_in, 200, seed=13, act_outliers=(0.01, 20.0))
    D = np.diag(orc.gram(X)).astype(np.float32)
    keep = int(d_out * d_in * keep_frac)
    n_iters = 4
    say("unstructured", d_out, d_in, b, keep)
    out = armor.factorize_layer(dev(torch, W), dev(torch, D), b, 2, 4, n_iters, sparsity=1, unstructured_keep=keep,
                                want_cont_trace=True, want_diagnostics=True)
    torch.cuda.synchronize()
    ref = orc.factorize_layer(W, D, b, 2, 4, n_iters, sparsity=1, keep=keep)
    mask = armor.unpack_mask(out["mask_bits"].cpu().numpy(), 8)
    S = out["S"].cpu().numpy()
    assert mask.sum() == keep                                   # exact count
    assert np.all(S[mask == 0] == 0)
    assert float((mask == ref["mask"]).mean()) >= 0.999
    tr = out["loss_trace"].cpu().numpy()
    assert_trace_parity(tr, ref["loss_trace"])
    np.testing.assert_allclose(out["loss_cont_trace"].cpu().numpy(), tr[1:], rtol=0, atol=0)
    assert np.all(np.diff(tr) <= 1e-6 * tr[0])
    for k, rk in (("A", "A"), ("B", "B"), ("S", "C")):
        assert relfro(out[k].cpu().numpy(), ref[rk]) <= 1e-3, k
    C0, _ = orc.init_unstructured(ref["Wbar"], D, keep)
    C0_gpu = armor.factorize_layer(dev(torch, W), dev(torch, D), b, 2, 4, 0, sparsity=1, unstructured_keep=keep)["S"].cpu().numpy()
    for name, got, want, start, sg in (("A", out["A"], ref["A"], identity_blocks(d_out // b, b), None),
                                       ("B", out["B"], ref["B"], identity_blocks(d_in // b, b), None),
                                       ("S", out["S"], ref["C"], C0, C0_gpu)):
        say("   " + assert_update_parity(name, got.cpu().numpy(), want, start, n_iters, start_got=sg))
    assert_diagnostics_parity(out, ref, n_iters, (d_out // b) * (d_in // b))
    assert int(out["mask_changes"].sum()) == 0


def test_unstructured_ties_go_to_lower_index(armor, torch, orc):
    """All-equal importances: the kept set must be exactly the first `keep` entries in row-major order."""
    d_out, d_in, b = 64, 64, 32
    W = np.ones((d_out, d_in), dtype=np.float32)
    D = np.ones(d_in, dtype=np.float32)
    for keep in (0, 1, 2049, 4095, 4096):
        out = armor.factorize_layer(dev(torch, W), dev(torch, D), b, 2, 4, 0, sparsity=1, unstructured_keep=keep)
        mask = armor.unpack_mask(out["mask_bits"].cpu().numpy(), 8).ravel()
        expect = np.zeros(d_out * d_in, dtype=np.uint8)
        expect[:keep] = 1
        np.testing.assert_array_equal(mask, expect)


@pytest.mark.parametrize("d_out,d_in,b,N,M,sparsity", [(128, 192, 64, 2, 4, 0), (256, 384, 128, 2, 4, 0), (96, 160, 32, 4, 8, 0),
                                                        (128, 128, 64, 2, 4, 1), (512, 768, 256, 2, 4, 0),
                                                        (512, 512, 256, 2, 4, 1)])
def test_factorize_joint_adam(armor, torch, orc, d_out, d_in, b, N, M, sparsity):
    """The joint-Adam continuous step (what the authors run in practice) against the oracle's.

    A group refit by Eq. 8 sits at a least-squares optimum, so its gradient at the next evaluation
    is zero up to rounding, and the sign of Adam's next step on it (size ~0.74 lr, independent of the
    gradient's magnitude) is decided by rounding noise in any implementation, the oracle included.
    Parity is therefore: exact-to-rounding for one iteration; to 1e-5 outside the refit groups for
    two; for longer runs loss trace, mask agreement, structure, and the bound 2 lr t on every entry."""
    W, X = make_layer(d_out, d_in, 300, seed=21, act_outliers=(0.01, 20.0))
    D = np.diag(orc.gram(X)).astype(np.float32)
    lr = 1e-3
    keep = (d_out * d_in) // 2 if sparsity else 0
    mg = 8 if sparsity else M
    nblk = (d_out // b) * (d_in // b)

    def run(n_iters):
        out = armor.factorize_layer(dev(torch, W), dev(torch, D), b, N, M, n_iters, seed=9, variant=1, lr=lr,
                                    sparsity=sparsity, unstructured_keep=keep, want_cont_trace=True)
        torch.cuda.synchronize()
        ref = orc.factorize_layer_adam(W, D, b, N, M, n_iters, seed=9, lr=lr, sparsity=sparsity, keep=keep)
        return out, ref

    say("adam", d_out, d_in, b, N, M, sparsity)
    # one iteration from theta_0: every quantity is determined
    out, ref = run(1)
    for k, rk in (("A", "A"), ("B", "B"), ("S", "C")):
        assert relfro(out[k].cpu().numpy(), ref[rk]) <= 1e-6, k
    np.testing.assert_array_equal(armor.unpack_mask(out["mask_bits"].cpu().numpy(), mg), ref["mask"])
    # two iterations: the moment recursion; only the groups refit at t = 1 may differ, by < 2 lr
    out, ref = run(2)
    assert relfro(out["A"].cpu().numpy(), ref["A"]) <= 1e-5 and relfro(out["B"].cpu().numpy(), ref["B"]) <= 1e-5
    dS = np.abs(out["S"].cpu().numpy() - ref["C"])
    assert int((dS > 1e-5).sum()) <= 2 * nblk * M and dS.max() <= 2 * lr
    # longer run
    n_iters = 8
    out, ref = run(n_iters)
    mask = armor.unpack_mask(out["mask_bits"].cpu().numpy(), mg)
    S = out["S"].cpu().numpy()
    if sparsity == 0:
        assert np.all(mask.reshape(d_out, d_in // M, M).sum(-1) == N)
    else:
        assert int(mask.sum()) == keep
    assert np.all(S[mask == 0] == 0)
    agree = float((mask == ref["mask"]).mean())
    tr = out["loss_trace"].cpu().numpy()
    dmax = max(np.abs(out["A"].cpu().numpy() - ref["A"]).max(), np.abs(out["B"].cpu().numpy() - ref["B"]).max(),
               np.abs(S - ref["C"])[(mask == 1) & (ref["mask"] == 1)].max())
    say("   mask agreement %.6f  max entry diff %.2e (2 lr t = %.1e)  loss %.6g -> %.6g (oracle %.6g)" %
        (agree, dmax, 2 * lr * n_iters, tr[0], tr[-1], ref["loss_trace"][-1]))
    assert agree >= 0.999
    assert dmax <= 2 * lr * n_iters
    np.testing.assert_allclose(tr, ref["loss_trace"], rtol=5e-3)
    np.testing.assert_allclose(out["loss_cont_trace"].cpu().numpy(), ref["loss_cont_trace"], rtol=5e-3)
    assert tr[-1] < tr[0]
    # the reported loss is the loss of the returned factors
    assert tr[-1] == pytest.approx(orc.proxy_loss(ref["Wbar"], out["A"].cpu().numpy(), S, out["B"].cpu().numpy(), D), rel=1e-4)


def test_factorize_zero_iterations_is_plain_nm_pruning(armor, torch, orc):
    W, X = make_layer(64, 128, 100, seed=7)
    D = np.diag(orc.gram(X)).astype(np.float32)
    out, ref = check_factorization(armor, torch, orc, W, D, 32, 2, 4, 0, seed=0)
    np.testing.assert_array_equal(armor.unpack_mask(out["mask_bits"].cpu().numpy(), 4), ref["mask"])
    np.testing.assert_array_equal(out["A"].cpu().numpy(), ref["A"])


def test_factorize_is_deterministic(armor, torch):
    W, X = make_layer(128, 128, 100, seed=8)
    D = (X.astype(np.float64) ** 2).sum(0).astype(np.float32)
    a = armor.factorize_layer(dev(torch, W), dev(torch, D), 64, 2, 4, 5, seed=1)
    b = armor.factorize_layer(dev(torch, W), dev(torch, D), 64, 2, 4, 5, seed=1)
    for k in ("A", "S", "B", "mask_bits", "loss_trace"):
        assert torch.equal(a[k], b[k]), k


def test_factorize_block128_deterministic_and_dead_channels(armor, torch, orc):
    """d_block 128 (streamed chains, two workgroups per CU, global scratch): two runs agree bit for bit,
    and input channels that never fire (D = 0: zero-weight columns of the loss) match the oracle."""
    W, X = make_layer(256, 384, 300, seed=31, act_outliers=(0.01, 20.0))
    D = np.diag(orc.gram(X)).astype(np.float32)
    D[np.random.default_rng(5).choice(384, 24, replace=False)] = 0.0
    a = armor.factorize_layer(dev(torch, W), dev(torch, D), 128, 2, 4, 4, seed=1)
    b = armor.factorize_layer(dev(torch, W), dev(torch, D), 128, 2, 4, 4, seed=1)
    for k in ("A", "S", "B", "mask_bits", "loss_trace"):
        assert torch.equal(a[k], b[k]), k
    check_factorization(armor, torch, orc, W, D, 128, 2, 4, 4, seed=1)


def test_denormalize_and_pack(armor, torch, orc):
    W, X = make_layer(128, 128, 100, seed=9)
    D = (X.astype(np.float64) ** 2).sum(0).astype(np.float32)
    plain = armor.factorize_layer(dev(torch, W), dev(torch, D), 32, 2, 4, 3, seed=1)
    folded = armor.factorize_layer(dev(torch, W), dev(torch, D), 32, 2, 4, 3, seed=1, denormalize=True)
    A2, B2 = orc.denormalize(plain["A"].cpu().numpy(), plain["B"].cpu().numpy(), plain["r1"].cpu().numpy(),
                             plain["r2"].cpu().numpy())
    np.testing.assert_allclose(folded["A"].cpu().numpy(), A2, rtol=1e-6)
    np.testing.assert_allclose(folded["B"].cpu().numpy(), B2, rtol=1e-6)
    vals, meta = armor.pack_nm(plain["S"], plain["mask_bits"], 2, 4)
    mask = armor.unpack_mask(plain["mask_bits"].cpu().numpy(), 4)
    ev, ei = orc.pack_nm(plain["S"].cpu().numpy(), mask, 2, 4)
    np.testing.assert_array_equal(vals.cpu().numpy(), ev)
    np.testing.assert_array_equal(meta.cpu().numpy(), orc.pack_index_bits(ei, 4))
    vb, _ = armor.pack_nm(plain["S"], plain["mask_bits"], 2, 4, bf16=True)
    np.testing.assert_array_equal(vb.view(torch.int16).cpu().numpy().view(np.uint16), synth.to_bf16_bits(ev))


@pytest.mark.parametrize("N,M,d_in", [(1, 2, 70), (2, 4, 136), (3, 4, 100), (1, 4, 36), (4, 8, 200), (5, 8, 72), (7, 8, 40),
                                      (2, 8, 24), (6, 8, 1024)])
def test_pack_nm_formats(armor, torch, orc, N, M, d_in):
    """Every N:M the library packs, with ragged rows (groups per row not a multiple of the groups a
    thread packs, index bits of a row not a whole number of bytes): values and bit-packed indices
    are bit-exact against the oracle's."""
    rng = np.random.default_rng(100 * N + M)
    d_out = 37
    S = rng.standard_normal((d_out, d_in)).astype(np.float32)
    scores = rng.random((d_out, d_in // M, M))
    keep = np.argsort(-scores, axis=-1)[..., :N]
    mask = np.zeros((d_out, d_in // M, M), dtype=np.uint8)
    np.put_along_axis(mask, keep, 1, axis=-1)
    S = S * mask.reshape(d_out, d_in)
    bits = (mask.astype(np.uint32) << np.arange(M, dtype=np.uint32)).sum(-1).astype(np.uint8)
    say("pack", N, M, d_in)
    vals, meta = armor.pack_nm(dev(torch, S), dev(torch, bits), N, M)
    ev, ei = orc.pack_nm(S, mask.reshape(d_out, d_in), N, M)
    np.testing.assert_array_equal(vals.cpu().numpy(), ev)
    np.testing.assert_array_equal(meta.cpu().numpy(), orc.pack_index_bits(ei, M))
    np.testing.assert_array_equal(armor.unpack_meta(meta.cpu().numpy(), d_in, N, M), ei)


def test_kernel_timing_counts_every_launch(armor, torch):
    """The library's own HIP-event timing: one record per instrumented launch, positive times that add up
    to no more than the wall time, nothing recorded when switched off."""
    import time
    W, X = make_layer(256, 256, 100, seed=3)
    D = (X.astype(np.float64) ** 2).sum(0).astype(np.float32)
    Wd, Dd = dev(torch, W), dev(torch, D)
    armor.factorize_layer(Wd, Dd, 64, 2, 4, 1, seed=1)
    torch.cuda.synchronize()
    armor.profile_enable(True)
    armor.profile_read()
    try:
        t0 = time.perf_counter()
        armor.factorize_layer(Wd, Dd, 64, 2, 4, 3, seed=1)
        armor.factorize_layer(Wd, Dd, 64, 2, 4, 2, seed=1, variant=1)
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3
        prof = armor.profile_read()
    finally:
        armor.profile_enable(False)
    expect = {"phase_A": 3, "phase_B": 3, "phase_WS": 3, "sparse_step": 5, "phase_FB": 2, "phase_GS": 2,
              "small_kernels": 2 * 3 + 2, "normalize": 2, "init": 2, "gram": 0, "pack_nm": 0}
    for k, n in expect.items():
        assert prof[k][1] == n, (k, prof[k])
        assert (prof[k][0] > 0) == (n > 0), (k, prof[k])
    assert sum(ms for ms, _ in prof.values()) <= wall_ms
    armor.factorize_layer(Wd, Dd, 64, 2, 4, 1, seed=1)
    torch.cuda.synchronize()
    assert all(n == 0 for _, n in armor.profile_read().values())
