"""Pins of the CPU oracle against things other than itself: closed forms, numpy dense algebra,
finite differences, brute-force least squares and the invariants the paper proves.  No GPU."""
import itertools

import numpy as np
import pytest
from scipy.linalg import block_diag

from paper_2510_05528_amd import synth


# ---------------------------------------------------------------------------------------------
# independent numpy helpers (dense algebra; none of this is oracle code)
# ---------------------------------------------------------------------------------------------
def dense(blocks):
    return block_diag(*[np.asarray(x, dtype=np.float64) for x in blocks])


def dense_loss(Wbar, A, C, B, D):
    R = Wbar.astype(np.float64) - dense(A) @ C.astype(np.float64) @ dense(B)
    return float((R * R * D.astype(np.float64)[None, :]).sum())


def rand_state(rng, d_out, d_in, b, N=2, M=4, perturb=0.1):
    """A generic point: wrappers near identity, random N:M core."""
    Wbar = rng.standard_normal((d_out, d_in)).astype(np.float32)
    D = (rng.random(d_in) * 3 + 0.2).astype(np.float32)
    A = np.stack([np.eye(b) + perturb * rng.standard_normal((b, b)) for _ in range(d_out // b)]).astype(np.float32)
    B = np.stack([np.eye(b) + perturb * rng.standard_normal((b, b)) for _ in range(d_in // b)]).astype(np.float32)
    mask = np.zeros((d_out, d_in), dtype=np.uint8)
    for i in range(d_out):
        for g in range(d_in // M):
            keep = rng.choice(M, size=N, replace=False)
            mask[i, g * M + keep] = 1
    C = (rng.standard_normal((d_out, d_in)) * mask).astype(np.float32)
    return Wbar, D, A, B, C, mask


# ---------------------------------------------------------------------------------------------
# normalisation (Sec. 3.2)
# ---------------------------------------------------------------------------------------------
def test_normalize_invariants(orc):
    W = synth.make_weight(24, 40, seed=3)
    Wbar, r1, r2 = orc.normalize(W)
    np.testing.assert_allclose(np.linalg.norm(Wbar.astype(np.float64), axis=1), 1.0, rtol=2e-6)
    np.testing.assert_allclose(Wbar.astype(np.float64) * r2[:, None] * r1[None, :], W, rtol=3e-6, atol=1e-12)
    W1 = W.astype(np.float64) / r1[None, :]
    np.testing.assert_allclose(np.linalg.norm(W1, axis=0), 1.0, rtol=2e-6)
    np.testing.assert_allclose(r1, np.linalg.norm(W.astype(np.float64), axis=0), rtol=1e-6)
    np.testing.assert_allclose(r2, np.linalg.norm(W1, axis=1), rtol=1e-6)


def test_normalize_zero_column_and_row(orc):
    W = synth.make_weight(8, 12, seed=1)
    W[:, 3] = 0
    W[5, :] = 0
    Wbar, r1, r2 = orc.normalize(W)
    assert r1[3] == 1.0 and r2[5] == 1.0
    assert np.all(Wbar[:, 3] == 0) and np.all(Wbar[5, :] == 0) and np.all(np.isfinite(Wbar))


# ---------------------------------------------------------------------------------------------
# initialisation + loss (Eq. 2, Eq. 3): L0 equals plain N:M pruning by W^2 D
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("N,M", [(2, 4), (4, 8), (1, 4), (5, 8)])
def test_init_loss_closed_form(orc, N, M):
    rng = np.random.default_rng(5)
    d_out, d_in, b = 16, 32, 8
    Wbar = rng.standard_normal((d_out, d_in)).astype(np.float32)
    D = (rng.random(d_in) + 0.1).astype(np.float32)
    C, mask = orc.init_nm(Wbar, D, N, M)
    # structure: exactly N per group, C = Wbar on the mask
    assert np.all(mask.reshape(d_out, d_in // M, M).sum(-1) == N)
    np.testing.assert_array_equal(C, Wbar * mask)
    # closed form: the M-N smallest importances of every group are lost
    imp = (Wbar.astype(np.float64) ** 2) * D.astype(np.float64)[None, :]
    expect = np.sort(imp.reshape(d_out, d_in // M, M), axis=-1)[..., : M - N].sum()
    I_A, I_B = orc.identity_blocks(d_out // b, b), orc.identity_blocks(d_in // b, b)
    got = orc.proxy_loss(Wbar, I_A, C, I_B, D)
    assert got == pytest.approx(expect, rel=1e-12)


def test_init_is_bruteforce_optimal_per_group(orc):
    rng = np.random.default_rng(11)
    Wbar = rng.standard_normal((4, 8)).astype(np.float32)
    D = (rng.random(8) + 0.1).astype(np.float32)
    _, mask = orc.init_nm(Wbar, D, 2, 4)
    for i in range(4):
        for g in range(2):
            w = Wbar[i, 4 * g:4 * g + 4].astype(np.float64)
            d = D[4 * g:4 * g + 4].astype(np.float64)
            losses = {}
            for keep in itertools.combinations(range(4), 2):
                m = np.zeros(4)
                m[list(keep)] = 1
                losses[keep] = float((((1 - m) * w) ** 2 * d).sum())
            best = min(losses, key=losses.get)
            assert tuple(np.nonzero(mask[i, 4 * g:4 * g + 4])[0]) == best


def test_init_ties_go_to_lower_index(orc):
    Wbar = np.array([[1, -1, 1, 1, 0, 0, 0, 0, 2, 1, 1, 2]], dtype=np.float32)
    D = np.ones(12, dtype=np.float32)
    _, mask = orc.init_nm(Wbar, D, 2, 4)
    np.testing.assert_array_equal(mask[0], [1, 1, 0, 0, 1, 1, 0, 0, 1, 0, 0, 1])
    D0 = np.zeros(12, dtype=np.float32)  # all scores zero -> first two of every group
    _, mask = orc.init_nm(Wbar, D0, 2, 4)
    np.testing.assert_array_equal(mask[0], [1, 1, 0, 0] * 3)


def test_init_unstructured_is_global_topk(orc):
    rng = np.random.default_rng(2)
    Wbar = rng.standard_normal((6, 8)).astype(np.float32)
    D = (rng.random(8) + 0.1).astype(np.float32)
    keep = 24
    C, mask = orc.init_unstructured(Wbar, D, keep)
    imp = ((Wbar * Wbar) * D[None, :]).ravel()
    order = np.lexsort((np.arange(imp.size), -imp))
    expect = np.zeros(imp.size, dtype=np.uint8)
    expect[order[:keep]] = 1
    np.testing.assert_array_equal(mask.ravel(), expect)
    assert mask.sum() == keep
    # optimal under a count budget: lost importance = sum of the smallest P-keep
    I_A, I_B = orc.identity_blocks(3, 2), orc.identity_blocks(4, 2)
    lost = orc.proxy_loss(Wbar, I_A, C, I_B, D)
    assert lost == pytest.approx(np.sort((Wbar.astype(np.float64) ** 2 * D[None, :]).ravel())[: imp.size - keep].sum(), rel=1e-12)
    # ties: equal scores -> lower linear index
    C, mask = orc.init_unstructured(np.ones((2, 4), np.float32), np.ones(4, np.float32), 3)
    np.testing.assert_array_equal(mask.ravel(), [1, 1, 1, 0, 0, 0, 0, 0])


def test_loss_matches_dense_algebra_and_is_nonnegative(orc):
    rng = np.random.default_rng(7)
    for (d_out, d_in, b) in [(8, 16, 4), (12, 8, 4), (16, 16, 8)]:
        Wbar, D, A, B, C, _ = rand_state(rng, d_out, d_in, b)
        got = orc.proxy_loss(Wbar, A, C, B, D)
        assert got >= 0
        assert got == pytest.approx(dense_loss(Wbar, A, C, B, D), rel=1e-12)
    np.testing.assert_allclose(orc.reconstruct(A, C, B), dense(A) @ C.astype(np.float64) @ dense(B), rtol=1e-12, atol=1e-14)


def test_wrapper_overheads_printed_in_the_paper(orc):
    """tests/golden/wrapper_overhead.txt: the relative parameter overhead of the wrappers over all linear layers of
    a decoder block (caption of the perplexity table), and the flop overhead and theoretical speedup of one 2:4
    layer (Sec. 4.4), all at d_block 128, reproduced from the entry counts of the factorized format and from the
    shapes the factorization itself returns."""
    import os
    rows = [l.split() for l in open(os.path.join(os.path.dirname(__file__), "golden", "wrapper_overhead.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 5
    for kind, name, *nums in rows:
        if kind == "params":
            hidden, inter, kv, printed = int(nums[0]), int(nums[1]), int(nums[2]), float(nums[3])
            layers = [(hidden, hidden), (kv, hidden), (kv, hidden), (hidden, hidden),    # q, k, v, o
                      (inter, hidden), (inter, hidden), (hidden, inter)]                 # gate, up, down
            sizes = [orc.factor_sizes(do, di, 128) for do, di in layers]
            o = 100.0 * sum(s["wrappers"] for s in sizes) / sum(s["dense"] for s in sizes)
            assert round(o, 2) == printed, (name, o)
        else:
            d_out, d_in, printed = int(nums[0]), int(nums[1]), float(nums[2])
            s = orc.factor_sizes(d_out, d_in, 128, 2, 4)
            if kind == "flops":
                assert round(100.0 * s["wrappers"] / s["dense"], 1) == printed
            else:
                assert round(s["dense"] / (s["core"] + s["wrappers"]), 2) == printed
    # the counts are those of the tensors the factorization returns
    W = synth.make_weight(64, 96, seed=0)
    D = np.ones(96, dtype=np.float32)
    out = orc.factorize_layer(W, D, 16, 2, 4, 0)
    s = orc.factor_sizes(64, 96, 16)
    assert out["A"].size + out["B"].size == s["wrappers"] and int(out["mask"].sum()) == s["core"] and out["C"].size == s["dense"]


def test_full_gram_loss_is_the_activation_error_and_reduces_to_eq2(orc):
    """tr(R H R^T) (Sec. 2, the objective before Eq. 2 drops the off-diagonal of H): equals the squared output
    error ||R X^T||_F^2 on the activations that made H, the plain triple sum on a tiny case whose residual is
    built entry by entry, and the proxy loss of Eq. 2 when H is diagonal."""
    d_out, d_in, b, N, M = 64, 96, 16, 2, 4
    rng = np.random.default_rng(2)
    Wbar, D, A, B, C, mask = rand_state(rng, d_out, d_in, b, N, M)
    X = rng.standard_normal((40, d_in))
    X[:, ::7] *= 5.0  # correlated, badly scaled channels: off-diagonal terms matter
    X += 0.5 * X[:, [0]]
    H = X.T @ X
    R = Wbar.astype(np.float64) - dense(A) @ C.astype(np.float64) @ dense(B)
    got = orc.proxy_loss_full_h(Wbar, A, C, B, H)
    assert np.isclose(got, np.linalg.norm(R @ X.T) ** 2, rtol=1e-12)
    assert abs(got - orc.proxy_loss(Wbar, A, C, B, np.diag(H))) > 0.05 * got  # the off-diagonal part is not negligible here
    # diagonal H: Eq. 2
    assert np.isclose(orc.proxy_loss_full_h(Wbar, A, C, B, np.diag(D.astype(np.float64))), orc.proxy_loss(Wbar, A, C, B, D), rtol=1e-12)
    # tiny case, entry by entry: R_ij = W_ij - sum_{p,q in the blocks} A^i[r,p] C[p,q] B^j[q,c]
    d_out, d_in, b = 4, 8, 2
    Wt, Dt, At, Bt, Ct, _ = rand_state(rng, d_out, d_in, b, 1, 2)
    Ht = rng.standard_normal((d_in, 5)); Ht = Ht @ Ht.T
    Rt = np.zeros((d_out, d_in))
    for i in range(d_out):
        for j in range(d_in):
            bi, bj = i // b, j // b
            s = 0.0
            for pp in range(b):
                for q in range(b):
                    s += float(At[bi, i % b, pp]) * float(Ct[bi * b + pp, bj * b + q]) * float(Bt[bj, q, j % b])
            Rt[i, j] = float(Wt[i, j]) - s
    brute = sum(Rt[i, j] * Ht[j, k] * Rt[i, k] for i in range(d_out) for j in range(d_in) for k in range(d_in))
    assert np.isclose(orc.proxy_loss_full_h(Wt, At, Ct, Bt, Ht), brute, rtol=1e-12)
    # exact factorization: zero
    I_A = np.tile(np.eye(b, dtype=np.float32), (d_out // b, 1, 1)); I_B = np.tile(np.eye(b, dtype=np.float32), (d_in // b, 1, 1))
    assert orc.proxy_loss_full_h(Wt, I_A, Wt, I_B, Ht) == 0.0


def test_diagonal_wrappers_commute_with_mask(orc):
    """App. A, Eq. 4: diag(a) (W' . M) diag(b) = (diag(a) W' diag(b)) . M, as an identity of the loss."""
    rng = np.random.default_rng(9)
    d_out, d_in, b = 8, 16, 4
    Wbar, D, _, _, C, _ = rand_state(rng, d_out, d_in, b)
    a = rng.standard_normal(d_out).astype(np.float32)
    bb = rng.standard_normal(d_in).astype(np.float32)
    A = np.stack([np.diag(a[i * b:(i + 1) * b]) for i in range(d_out // b)])
    B = np.stack([np.diag(bb[j * b:(j + 1) * b]) for j in range(d_in // b)])
    C2 = (a[:, None].astype(np.float64) * C * bb[None, :]).astype(np.float32)
    l1 = orc.proxy_loss(Wbar, A, C, B, D)
    l2 = orc.proxy_loss(Wbar, orc.identity_blocks(d_out // b, b), C2, orc.identity_blocks(d_in // b, b), D)
    assert l1 == pytest.approx(l2, rel=1e-5)


# ---------------------------------------------------------------------------------------------
# gradients (App. D) against central finite differences of the DENSE numpy loss
# ---------------------------------------------------------------------------------------------
def _fd(f, x, idxs, h=1e-4):
    out = []
    for idx in idxs:
        xp, xm = x.copy(), x.copy()
        xp[idx] += h
        xm[idx] -= h
        out.append((f(xp) - f(xm)) / (2 * h))
    return np.array(out)


def test_gradients_match_finite_differences(orc):
    rng = np.random.default_rng(13)
    d_out, d_in, b = 8, 12, 4
    Wbar, D, A, B, C, mask = rand_state(rng, d_out, d_in, b)
    A64, B64, C64 = A.astype(np.float64), B.astype(np.float64), C.astype(np.float64)
    gA, _ = orc.grad_A(Wbar, A, C, B, D)
    gB, _ = orc.grad_B(Wbar, A, C, B, D)
    gC, _ = orc.grad_core(Wbar, A, C, B, D)
    idxA = [tuple(rng.integers(0, s) for s in A.shape) for _ in range(25)]
    idxB = [tuple(rng.integers(0, s) for s in B.shape) for _ in range(25)]
    idxC = [tuple(rng.integers(0, s) for s in C.shape) for _ in range(25)]
    fdA = _fd(lambda a: dense_loss(Wbar, a, C64, B64, D), A64, idxA)
    fdB = _fd(lambda x: dense_loss(Wbar, A64, C64, x, D), B64, idxB)
    fdC = _fd(lambda c: dense_loss(Wbar, A64, c, B64, D), C64, idxC)  # w.r.t. the core entries, masked or not
    np.testing.assert_allclose([gA[i] for i in idxA], fdA, rtol=1e-5, atol=1e-6)
    np.testing.assert_allclose([gB[i] for i in idxB], fdB, rtol=1e-5, atol=1e-6)
    np.testing.assert_allclose([gC[i] for i in idxC], fdC, rtol=1e-5, atol=1e-6)


def test_gradients_at_initial_point(orc):
    """At theta_0 the residual and the core have disjoint support: grad_W' . M = 0, diag(grad_A^i) = 0."""
    rng = np.random.default_rng(3)
    d_out, d_in, b = 8, 16, 4
    Wbar = rng.standard_normal((d_out, d_in)).astype(np.float32)
    D = (rng.random(d_in) + 0.1).astype(np.float32)
    C, mask = orc.init_nm(Wbar, D, 2, 4)
    I_A, I_B = orc.identity_blocks(d_out // b, b), orc.identity_blocks(d_in // b, b)
    gC, _ = orc.grad_core(Wbar, I_A, C, I_B, D)
    assert np.all(gC[mask == 1] == 0)
    np.testing.assert_allclose(gC[mask == 0], (-2 * Wbar.astype(np.float64) * D[None, :])[mask == 0], rtol=1e-12)
    gA, _ = orc.grad_A(Wbar, I_A, C, I_B, D)
    for i in range(d_out // b):
        np.testing.assert_allclose(np.diag(gA[i]), 0, atol=1e-12)


# ---------------------------------------------------------------------------------------------
# smoothness constants (Eq. 9-11): formulas, the Lipschitz inequality, and monotone sub-steps
# ---------------------------------------------------------------------------------------------
def _np_betas(Wbar, A, C, B, D, b):
    d_out, d_in = Wbar.shape
    A64, B64, C64, D64 = dense(A), dense(B), C.astype(np.float64), D.astype(np.float64)
    S, Sp = C64 @ B64, A64 @ C64
    bA = bB = 0.0
    for i in range(d_out // b):
        for j in range(d_in // b):
            s = S[i * b:(i + 1) * b, j * b:(j + 1) * b]
            sp = Sp[i * b:(i + 1) * b, j * b:(j + 1) * b]
            dj = D64[j * b:(j + 1) * b]
            bA += 2 * np.linalg.norm(s @ np.diag(dj) @ s.T)
            bB += 2 * np.linalg.norm(sp.T @ sp) * np.linalg.norm(dj)
    bW = 2 * np.linalg.norm(A64.T @ A64) * np.linalg.norm(B64 @ np.diag(D64) @ B64.T)
    return bA, bB, bW


def test_beta_formulas_and_lipschitz(orc):
    rng = np.random.default_rng(17)
    d_out, d_in, b = 8, 12, 4
    Wbar, D, A, B, C, mask = rand_state(rng, d_out, d_in, b, perturb=0.3)
    gA, bA = orc.grad_A(Wbar, A, C, B, D)
    gB, bB = orc.grad_B(Wbar, A, C, B, D)
    gC, bW = orc.grad_core(Wbar, A, C, B, D)
    eA, eB, eW = _np_betas(Wbar, A, C, B, D, b)
    assert bA == pytest.approx(eA, rel=1e-10) and bB == pytest.approx(eB, rel=1e-10) and bW == pytest.approx(eW, rel=1e-10)
    for _ in range(5):
        A2 = (A + rng.standard_normal(A.shape)).astype(np.float32)
        B2 = (B + rng.standard_normal(B.shape)).astype(np.float32)
        C2 = (C + rng.standard_normal(C.shape) * mask).astype(np.float32)
        gA2, _ = orc.grad_A(Wbar, A2, C, B, D)
        gB2, _ = orc.grad_B(Wbar, A, C, B2, D)
        gC2, _ = orc.grad_core(Wbar, A, C2, B, D)
        assert np.linalg.norm(gA2 - gA) <= bA * np.linalg.norm(A2.astype(np.float64) - A) * (1 + 1e-9)
        assert np.linalg.norm(gB2 - gB) <= bB * np.linalg.norm(B2.astype(np.float64) - B) * (1 + 1e-9)
        assert np.linalg.norm((gC2 - gC) * mask) <= bW * np.linalg.norm(C2.astype(np.float64) - C) * (1 + 1e-9)


def test_continuous_update_is_three_steps_at_updated_points_and_monotone(orc):
    """Lemma 1: A step at (A,B,C), B step at (A_new,B,C), W' step at (A_new,B_new,C); each lowers L."""
    rng = np.random.default_rng(19)
    d_out, d_in, b = 8, 16, 4
    Wbar, D, A, B, C, mask = rand_state(rng, d_out, d_in, b, perturb=0.2)
    L0 = dense_loss(Wbar, A, C, B, D)
    gA, bA = orc.grad_A(Wbar, A, C, B, D)
    A1 = (A.astype(np.float64) - gA / bA).astype(np.float32)
    L1 = dense_loss(Wbar, A1, C, B, D)
    gB, bB = orc.grad_B(Wbar, A1, C, B, D)
    B1 = (B.astype(np.float64) - gB / bB).astype(np.float32)
    L2 = dense_loss(Wbar, A1, C, B1, D)
    gC, bW = orc.grad_core(Wbar, A1, C, B1, D)
    C1 = (C.astype(np.float64) - gC * mask / bW).astype(np.float32)
    L3 = dense_loss(Wbar, A1, C1, B1, D)
    assert L3 <= L2 <= L1 <= L0 and L3 < L0
    A_o, C_o, B_o, etas = orc.continuous_update(Wbar, D, mask, A, C, B)
    np.testing.assert_array_equal(A_o, A1)
    np.testing.assert_array_equal(B_o, B1)
    np.testing.assert_array_equal(C_o, C1)
    np.testing.assert_allclose(etas, [1 / bA, 1 / bB, 1 / bW], rtol=1e-12)
    assert np.all(C_o[mask == 0] == 0)


# ---------------------------------------------------------------------------------------------
# sparse-core step (App. B.1, Eq. 6-8, Alg. 3) against brute-force least squares
# ---------------------------------------------------------------------------------------------
def _block_bruteforce(Wbar, A, B, D, C, i, j, ip, k0, b, N, M):
    """Enumerate every N-of-M mask of group (ip, k0) in block (i,j); solve each with lstsq on the
    vectorised problem  min_w || DeltaW - a (w^T B') ||_{F,D}."""
    A_i, B_j = A[i].astype(np.float64), B[j].astype(np.float64)
    Dj = D[j * b:(j + 1) * b].astype(np.float64)
    Cb = C[i * b:(i + 1) * b, j * b:(j + 1) * b].astype(np.float64).copy()
    Wb = Wbar[i * b:(i + 1) * b, j * b:(j + 1) * b].astype(np.float64)
    Cb[ip, k0:k0 + M] = 0
    dW = Wb - A_i @ Cb @ B_j
    a = A_i[:, ip]
    sq = np.sqrt(Dj)[None, :]
    res = []
    for s in itertools.combinations(range(M), N):
        cols = [np.outer(a, B_j[k0 + p, :]) * sq for p in s]
        X = np.stack([c.ravel() for c in cols], axis=1)
        y = (dW * sq).ravel()
        w, *_ = np.linalg.lstsq(X, y, rcond=None)
        loss = float(((y - X @ w) ** 2).sum())
        res.append((s, w, loss))
    base = float(((dW * sq) ** 2).sum())
    return res, base


@pytest.mark.parametrize("N,M,b", [(2, 4, 8), (4, 8, 8), (1, 4, 4), (6, 8, 8)])
def test_sparse_step_matches_bruteforce(orc, N, M, b):
    rng = np.random.default_rng(23 + N)
    d_out, d_in = 2 * b, 3 * b
    Wbar, D, A, B, C, mask = rand_state(rng, d_out, d_in, b, N=N, M=M, perturb=0.3)
    before = dense_loss(Wbar, A, C, B, D)
    C2, mask2, kap, pat = orc.sparse_core_update(Wbar, A, B, D, C, mask, N, M, seed=5, t=1, selection=0)
    assert np.all(mask2.reshape(d_out, d_in // M, M).sum(-1) == N)
    assert np.all(C2[mask2 == 0] == 0)
    gpr = b // M
    nbj = d_in // b
    changed = np.argwhere((C2 != C) | (mask2 != mask))
    total_gain = 0.0
    for blk in range((d_out // b) * nbj):
        i, j = divmod(blk, nbj)
        ip, k0 = kap[blk] // gpr, (kap[blk] % gpr) * M
        res, base = _block_bruteforce(Wbar, A, B, D, C, i, j, ip, k0, b, N, M)
        best = min(res, key=lambda r: r[2])
        got_pat = tuple(p for p in range(M) if (pat[blk] >> p) & 1)
        got_loss = dict((r[0], r[2]) for r in res)[got_pat]
        assert got_loss <= best[2] * (1 + 1e-6) + 1e-12          # the winner is a brute-force optimum
        w_ref = dict((r[0], r[1]) for r in res)[got_pat]
        row = C2[i * b + ip, j * b + k0:j * b + k0 + M]
        np.testing.assert_allclose(row[list(got_pat)], w_ref, rtol=2e-5, atol=1e-6)
        assert np.all(np.delete(row, list(got_pat)) == 0)
        # block loss after the write = ||DeltaW||_D^2 - gain  (Eq. 7)
        blk_after = dense_loss(Wbar[i * b:(i + 1) * b, j * b:(j + 1) * b], A[i:i + 1],
                               C2[i * b:(i + 1) * b, j * b:(j + 1) * b], B[j:j + 1], D[j * b:(j + 1) * b])
        assert blk_after == pytest.approx(got_loss, rel=1e-4, abs=1e-9)
        total_gain += base - got_loss
    # only the drawn group of each block was touched
    for (r, c) in changed:
        blk = (r // b) * nbj + c // b
        assert r % b == kap[blk] // gpr and (c % b) // M == kap[blk] % gpr
    after = dense_loss(Wbar, A, C2, B, D)
    assert after <= before * (1 + 1e-9)     # Lemma 2


def test_sparse_step_identity_wrappers_reselects_topn(orc):
    """A = B = I: gain_s = sum of importances in s, so the sweep re-selects the Eq. 3 mask and
    w* = W-bar there; from theta_0 the step is a no-op (reduces to plain N:M pruning)."""
    rng = np.random.default_rng(29)
    d_out, d_in, b = 8, 16, 8
    Wbar = rng.standard_normal((d_out, d_in)).astype(np.float32)
    D = (rng.random(d_in) + 0.1).astype(np.float32)
    C, mask = orc.init_nm(Wbar, D, 2, 4)
    I_A, I_B = orc.identity_blocks(d_out // b, b), orc.identity_blocks(d_in // b, b)
    for sel in (0, 1, 2, 3):
        C2, mask2, kap, pat = orc.sparse_core_update(Wbar, I_A, I_B, D, C, mask, 2, 4, seed=1, t=1, selection=sel)
        np.testing.assert_array_equal(mask2, mask)
        np.testing.assert_allclose(C2, C, rtol=1e-6)
    # and from a scrambled mask, the drawn groups move to the top-2 pattern with w* = Wbar
    bad = np.roll(mask, 1, axis=1)
    Cb = Wbar * bad
    C2, mask2, kap, pat = orc.sparse_core_update(Wbar, I_A, I_B, D, Cb, bad, 2, 4, seed=1, t=1, selection=1)
    for blk in range(2):
        i, j = divmod(blk, 2)
        ip, k0 = kap[blk] // 2, (kap[blk] % 2) * 4
        np.testing.assert_array_equal(mask2[i * b + ip, j * b + k0:j * b + k0 + 4], mask[i * b + ip, j * b + k0:j * b + k0 + 4])
        np.testing.assert_allclose(C2[i * b + ip, j * b + k0:j * b + k0 + 4], C[i * b + ip, j * b + k0:j * b + k0 + 4], rtol=1e-6)


def test_sparse_step_rank_deficient_uses_pseudo_inverse(orc):
    """Two identical rows of B inside the group: B' D B'^T is singular for the pair; the
    Moore-Penrose solution splits the weight evenly and the loss still equals the lstsq optimum."""
    rng = np.random.default_rng(31)
    b = 4
    Wbar, D, A, B, C, mask = rand_state(rng, 4, 4, b, perturb=0.3)
    B[0, 1, :] = B[0, 0, :]
    C2, mask2, kap, pat = orc.sparse_core_update(Wbar, A, B, D, C, mask, 2, 4, seed=0, t=1, selection=1)
    ip = kap[0]
    res, base = _block_bruteforce(Wbar, A, B, D, C, 0, 0, ip, 0, b, 2, 4)
    best = min(r[2] for r in res)
    after = dense_loss(Wbar, A, C2, B, D)
    assert after == pytest.approx(best, rel=1e-5, abs=1e-9)
    assert np.all(np.isfinite(C2))
    if pat[0] == 0b0011:
        assert C2[ip, 0] == pytest.approx(C2[ip, 1], rel=1e-5)


def test_sparse_step_zero_column_of_A_skips_block(orc):
    rng = np.random.default_rng(37)
    b = 4
    Wbar, D, A, B, C, mask = rand_state(rng, 4, 4, b)
    A[0] = 0
    C2, mask2, kap, pat = orc.sparse_core_update(Wbar, A, B, D, C, mask, 2, 4, seed=0, t=1, selection=3)
    assert kap[0] == -1
    np.testing.assert_array_equal(C2, C)
    np.testing.assert_array_equal(mask2, mask)


# ---------------------------------------------------------------------------------------------
# selection rule (Sec. 3.3.2, App. E.1)
# ---------------------------------------------------------------------------------------------
def _py_uniform(seed, t, n_blocks, blk, gpb, kappa):
    """Independent restatement of the counter hash (splitmix64 finaliser, top 24 bits)."""
    mask64 = (1 << 64) - 1
    ctr = ((t * n_blocks + blk) * gpb + kappa) + 1
    z = (seed + 0x9E3779B97F4A7C15 * ctr) & mask64
    z ^= z >> 30
    z = (z * 0xBF58476D1CE4E5B9) & mask64
    z ^= z >> 27
    z = (z * 0x94D049BB133111EB) & mask64
    z ^= z >> 31
    return np.float32(((z >> 40) + 1)) * np.float32(2.0 ** -24)


def test_uniform_hash_spec(orc):
    vals = []
    for (seed, t, nb, blk, gpb, kap) in [(0, 1, 1, 0, 16, 0), (0, 1, 64, 63, 256, 255), (12345, 50, 1024, 1000, 4096, 4095),
                                         (2 ** 63 + 5, 20000, 3584, 3583, 16384, 16383)]:
        u = orc.uniform(seed, t, nb, blk, gpb, kap)
        assert u == float(_py_uniform(seed, t, nb, blk, gpb, kap))
        assert 0.0 < u <= 1.0
        vals.append(u)
    us = np.array([orc.uniform(7, 1, 1, 0, 100000, k) for k in range(20000)])
    assert abs(us.mean() - 0.5) < 0.01 and abs(us.var() - 1 / 12) < 0.005
    assert us.min() > 0 and us.max() <= 1.0


def test_selection_frequencies_follow_l1_of_gradient(orc):
    rng = np.random.default_rng(41)
    b, N, M = 8, 2, 4
    Wbar, D, A, B, C, mask = rand_state(rng, b, b, b, perturb=0.2)
    G, _ = orc.grad_core(Wbar, A, C, B, D)
    g = np.abs(G).reshape(b, b // M, M).sum(-1).ravel()          # kappa = i' * (b/M) + k
    p = g / g.sum()
    n_draw = 6000
    counts = np.zeros(g.size)
    for seed in range(n_draw):
        _, _, kap, _ = orc.sparse_core_update(Wbar, A, B, D, C, mask, N, M, seed=seed, t=1, selection=0)
        counts[kap[0]] += 1
    chi2 = ((counts - n_draw * p) ** 2 / (n_draw * p)).sum()
    assert chi2 < 45.0   # 15 dof, p ~ 1e-4 false alarm
    # greedy = argmax of the L1 score; L2-weighted uses sqrt(sum g^2)
    _, _, kap, _ = orc.sparse_core_update(Wbar, A, B, D, C, mask, N, M, seed=0, t=1, selection=1)
    assert kap[0] == int(np.argmax(g))
    g2 = np.sqrt((G ** 2).reshape(b, b // M, M).sum(-1)).ravel()
    p2 = g2 / g2.sum()
    counts2 = np.zeros(g.size)
    for seed in range(n_draw):
        _, _, kap, _ = orc.sparse_core_update(Wbar, A, B, D, C, mask, N, M, seed=seed, t=1, selection=2)
        counts2[kap[0]] += 1
    assert ((counts2 - n_draw * p2) ** 2 / (n_draw * p2)).sum() < 45.0
    counts3 = np.zeros(g.size)
    for seed in range(n_draw):
        _, _, kap, _ = orc.sparse_core_update(Wbar, A, B, D, C, mask, N, M, seed=seed, t=1, selection=3)
        counts3[kap[0]] += 1
    assert ((counts3 - n_draw / g.size) ** 2 / (n_draw / g.size)).sum() < 45.0


def test_selection_key_is_exponential_race_with_lower_index_ties(orc):
    """Replay the draw in numpy from the hash and the gradient: argmin of -ln(u)/g."""
    rng = np.random.default_rng(43)
    b, N, M = 8, 2, 4
    d_out, d_in = 16, 24
    Wbar, D, A, B, C, mask = rand_state(rng, d_out, d_in, b, perturb=0.2)
    G, _ = orc.grad_core(Wbar, A, C, B, D)
    nbj, gpr = d_in // b, b // M
    gpb = b * gpr
    nblk = (d_out // b) * nbj
    seed, t = 99, 7
    _, _, kap, _ = orc.sparse_core_update(Wbar, A, B, D, C, mask, N, M, seed=seed, t=t, selection=0)
    for blk in range(nblk):
        i, j = divmod(blk, nbj)
        g = np.abs(G[i * b:(i + 1) * b, j * b:(j + 1) * b]).reshape(b, gpr, M).sum(-1).ravel().astype(np.float32)
        keys = np.array([np.float32(-np.log(np.float64(_py_uniform(seed, t, nblk, blk, gpb, k)))) / g[k] for k in range(gpb)],
                        dtype=np.float32)
        assert kap[blk] == int(np.argmin(keys))


# ---------------------------------------------------------------------------------------------
# whole loop (Alg. 1, Thm. 1, Lemma 1, Lemma 2)
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("N,M,sel", [(2, 4, 0), (4, 8, 0), (2, 4, 1)])
def test_factorize_trace_monotone_and_mask_valid(orc, N, M, sel):
    d_out, d_in, b = 32, 48, 16
    W = synth.make_weight(d_out, d_in, seed=1, outlier_frac=0.05)
    X = synth.make_calibration(96, d_in, seed=1)
    D = np.diag(orc.gram(X)).astype(np.float32)
    out = orc.factorize_layer(W, D, b, N, M, n_iters=12, seed=3, selection=sel)
    tr, ct = out["loss_trace"], out["loss_cont_trace"]
    assert np.all(tr >= 0)
    tol = 1e-6 * tr[0]
    assert np.all(ct <= tr[:-1] + tol)          # Lemma 1
    assert np.all(tr[1:] <= ct + tol)           # Lemma 2
    assert np.all(np.diff(tr) <= tol) and tr[-1] < 0.999 * tr[0]     # Thm. 1, and it actually moves
    mask, C = out["mask"], out["C"]
    assert np.all(mask.reshape(d_out, d_in // M, M).sum(-1) == N)
    assert np.all(C[mask == 0] == 0)
    # L0 is the plain N:M pruning loss of the normalised weight
    imp = (out["Wbar"].astype(np.float64) ** 2) * D.astype(np.float64)[None, :]
    assert tr[0] == pytest.approx(np.sort(imp.reshape(d_out, d_in // M, M), axis=-1)[..., : M - N].sum(), rel=1e-9)
    # the trace is the dense loss of the returned factors
    assert tr[-1] == pytest.approx(dense_loss(out["Wbar"], out["A"], C, out["B"], D), rel=1e-9)


def _normalized_inverse(Wbar, r1, r2):
    """A weight whose normalisation is (close to) the given W-bar: W = diag(r2) Wbar diag(r1)."""
    return (r2[:, None].astype(np.float64) * Wbar.astype(np.float64) * r1[None, :]).astype(np.float32)


@pytest.mark.parametrize("N,M", [(2, 4), (4, 8)])
def test_factorize_from_a_given_point_is_a_replay_of_the_two_steps(orc, N, M):
    """Alg. 1 from a caller-supplied theta_0 (generic point, so every step moves and masks change):
    the loop is exactly continuous_update then sparse_core_update, iteration after iteration; the step
    sizes it reports are 1/beta of Eq. 9-11 evaluated by dense numpy algebra at the points of Lemma 1;
    mask_changes counts the groups whose kept set moved; the iteration counter of the draw is offset."""
    rng = np.random.default_rng(101 + N)
    d_out, d_in, b, iters, off = 16, 24, 8, 4, 7
    W = synth.make_weight(d_out, d_in, seed=5, outlier_frac=0.05)
    _, D, A, B, C, mask = rand_state(rng, d_out, d_in, b, N=N, M=M, perturb=0.3)
    C = (0.1 * C).astype(np.float32)
    out = orc.factorize_layer(W, D, b, N, M, iters, seed=4, init=dict(A=A, B=B, C=C, mask=mask), iter_offset=off)
    Wbar, _, _ = orc.normalize(W)
    np.testing.assert_array_equal(out["Wbar"], Wbar)
    a, c, bb, m = A, C, B, mask
    assert out["loss_trace"][0] == pytest.approx(dense_loss(Wbar, a, c, bb, D), rel=1e-10)
    total_changes = 0
    for t in range(1, iters + 1):
        bA, _, _ = _np_betas(Wbar, a, c, bb, D, b)
        a1, c1, b1, etas = orc.continuous_update(Wbar, D, m, a, c, bb)
        _, bB, _ = _np_betas(Wbar, a1, c, bb, D, b)          # B step sees the new A
        _, _, bW = _np_betas(Wbar, a1, c, b1, D, b)          # W' step sees the new A and B
        np.testing.assert_allclose(out["etas"][t - 1], [1 / bA, 1 / bB, 1 / bW], rtol=1e-9)
        np.testing.assert_array_equal(out["etas"][t - 1], etas)
        assert out["loss_cont_trace"][t - 1] == pytest.approx(dense_loss(Wbar, a1, c1, b1, D), rel=1e-10)
        c2, m2, _, _ = orc.sparse_core_update(Wbar, a1, b1, D, c1, m, N, M, seed=4, t=off + t)
        changed = int((m2.reshape(-1, M) != m.reshape(-1, M)).any(axis=1).sum())
        assert out["mask_changes"][t - 1] == changed
        total_changes += changed
        a, c, bb, m = a1, c2, b1, m2
        assert out["loss_trace"][t] == pytest.approx(dense_loss(Wbar, a, c, bb, D), rel=1e-10)
    assert total_changes > 0                                   # the case does exercise mask moves
    for k, v in (("A", a), ("C", c), ("B", bb), ("mask", m)):
        np.testing.assert_array_equal(out[k], v)
    # a different offset draws different groups
    other = orc.factorize_layer(W, D, b, N, M, iters, seed=4, init=dict(A=A, B=B, C=C, mask=mask), iter_offset=0)
    assert not np.array_equal(other["C"], out["C"])


def test_tolerance_stop_is_the_full_run_cut_at_the_first_small_decrease(orc):
    """The tolerance input of Alg. 1 (declared in the listing, never used in it), read as: the loop ends after
    the first iteration whose decrease is within it, L_{t-1} - L_t <= tol * L_0.  The stopped run must be the
    full run cut at that iteration, found here from the full run's own loss trace."""
    d_out, d_in, b = 32, 48, 16
    W = synth.make_weight(d_out, d_in, seed=1, outlier_frac=0.05)
    D = (np.random.default_rng(0).random(d_in) + 0.5).astype(np.float32)
    n = 12
    full = orc.factorize_layer(W, D, b, 2, 4, n, seed=3)
    L = full["loss_trace"]
    assert full["iters_done"] == n and len(L) == n + 1
    dec = (L[:-1] - L[1:]) / L[0]
    # a tolerance that at least one iteration in the middle of the run meets and the first ones do not
    tol = float(np.sort(dec[2:])[len(dec[2:]) // 2])
    tol = max(tol, float(np.nextafter(dec[:2].min(), 0)) * 0.5) if dec[:2].min() > tol else tol
    stop = 1 + int(np.argmax(dec <= tol))
    assert 1 <= stop < n
    cut = orc.factorize_layer(W, D, b, 2, 4, n, seed=3, tol=tol)
    assert cut["iters_done"] == stop
    np.testing.assert_array_equal(cut["loss_trace"], L[:stop + 1])
    prefix = orc.factorize_layer(W, D, b, 2, 4, stop, seed=3)
    for k in ("A", "C", "B", "mask"):
        np.testing.assert_array_equal(cut[k], prefix[k])
    assert len(cut["etas"]) == stop and len(cut["mask_changes"]) == stop
    # a tolerance nothing meets changes nothing; one that everything meets stops after the first iteration
    none = orc.factorize_layer(W, D, b, 2, 4, n, seed=3, tol=float(dec.min()) * 0.5 if dec.min() > 0 else 1e-300)
    assert none["iters_done"] == n or dec.min() <= 0
    first = orc.factorize_layer(W, D, b, 2, 4, n, seed=3, tol=1.0)
    assert first["iters_done"] == 1
    np.testing.assert_array_equal(first["loss_trace"], L[:2])


@pytest.mark.parametrize("adam", [False, True])
def test_a_run_cut_in_two_is_the_same_run(orc, adam):
    """theta_0 is an input of Alg. 1: stopping after k iterations and starting again from the result,
    with the iteration counter carried over, gives the uninterrupted run (sequential variant: exactly;
    the joint-Adam variant restarts its moments, so only its first leg and the structure agree)."""
    d_out, d_in, b = 32, 48, 16
    W = synth.make_weight(d_out, d_in, seed=1, outlier_frac=0.05)
    D = (np.random.default_rng(0).random(d_in) + 0.5).astype(np.float32)
    f = orc.factorize_layer_adam if adam else orc.factorize_layer
    kw = dict(lr=1e-3) if adam else {}
    whole = f(W, D, b, 2, 4, 5, seed=3, **kw)
    first = f(W, D, b, 2, 4, 2, seed=3, **kw)
    second = f(W, D, b, 2, 4, 3, seed=3, init=first, iter_offset=2, **kw)
    np.testing.assert_array_equal(first["loss_trace"], whole["loss_trace"][:3])
    assert second["loss_trace"][0] == first["loss_trace"][-1]
    assert np.all(second["mask"].reshape(d_out, d_in // 4, 4).sum(-1) == 2)
    if not adam:
        for k in ("A", "C", "B", "mask"):
            np.testing.assert_array_equal(second[k], whole[k])
        np.testing.assert_array_equal(second["loss_trace"], whole["loss_trace"][2:])
        np.testing.assert_array_equal(np.concatenate([first["etas"], second["etas"]]), whole["etas"])
        np.testing.assert_array_equal(np.concatenate([first["mask_changes"], second["mask_changes"]]),
                                      whole["mask_changes"])


def test_factorize_unstructured_runs_continuous_step_only(orc):
    d_out, d_in, b = 16, 32, 8
    W = synth.make_weight(d_out, d_in, seed=2)
    D = (np.random.default_rng(0).random(d_in) + 0.5).astype(np.float32)
    keep = d_out * d_in // 2
    out = orc.factorize_layer(W, D, b, 2, 4, n_iters=6, sparsity=1, keep=keep)
    C0, mask0 = orc.init_unstructured(out["Wbar"], D, keep)
    np.testing.assert_array_equal(out["mask"], mask0)        # the mask never moves
    assert out["mask"].sum() == keep
    assert np.all(np.diff(out["loss_trace"]) <= 0)
    np.testing.assert_allclose(out["loss_trace"][1:], out["loss_cont_trace"], rtol=1e-12)


def test_denormalize_identity(orc):
    rng = np.random.default_rng(47)
    d_out, d_in, b = 8, 12, 4
    _, _, A, B, C, _ = rand_state(rng, d_out, d_in, b)
    r1 = (rng.random(d_in) + 0.5).astype(np.float32)
    r2 = (rng.random(d_out) + 0.5).astype(np.float32)
    A2, B2 = orc.denormalize(A, B, r1, r2)
    lhs = dense(A2) @ C.astype(np.float64) @ dense(B2)
    rhs = r2[:, None] * (dense(A) @ C.astype(np.float64) @ dense(B)) * r1[None, :]
    np.testing.assert_allclose(lhs, rhs, rtol=1e-5, atol=1e-6)


def test_denormalized_factors_approximate_original_weight(orc):
    """End to end: diag(r2) (A S B) diag(r1) is closer to W (in the D-weighted norm of the
    normalised space) than plain N:M pruning of W-bar."""
    d_out, d_in, b = 32, 32, 16
    W = synth.make_weight(d_out, d_in, seed=4)
    D = np.ones(d_in, dtype=np.float32)
    out = orc.factorize_layer(W, D, b, 2, 4, n_iters=10, seed=0)
    A2, B2 = orc.denormalize(out["A"], out["B"], out["r1"], out["r2"])
    What = dense(A2) @ out["C"].astype(np.float64) @ dense(B2)
    err = (((W - What) / out["r2"][:, None] / out["r1"][None, :]) ** 2).sum()
    assert err == pytest.approx(out["loss_trace"][-1], rel=1e-4)
    assert err < out["loss_trace"][0]


def test_pack_nm_roundtrip(orc):
    rng = np.random.default_rng(53)
    _, _, _, _, C, mask = rand_state(rng, 8, 16, 4, N=2, M=4)
    vals, idx = orc.pack_nm(C, mask, 2, 4)
    rebuilt = np.zeros_like(C)
    for i in range(8):
        for g in range(4):
            for x in range(2):
                rebuilt[i, g * 4 + idx[i, g * 2 + x]] = vals[i, g * 2 + x]
    np.testing.assert_array_equal(rebuilt, C)
    assert np.all(np.diff(idx.reshape(8, 4, 2).astype(int), axis=-1) > 0)


@pytest.mark.parametrize("M,entries", [(2, 13), (4, 16), (4, 6), (8, 5)])
def test_pack_index_bits_is_a_little_endian_bit_stream(orc, M, entries):
    """The compact index form read back as one integer per row: field e sits at bit e*w."""
    rng = np.random.default_rng(54)
    w = {2: 1, 4: 2, 8: 4}[M]
    idx = rng.integers(0, M, (3, entries)).astype(np.uint8)
    packed = orc.pack_index_bits(idx, M)
    assert packed.shape == (3, (entries * w + 7) // 8)
    for i in range(3):
        as_int = int.from_bytes(packed[i].tobytes(), "little")
        assert [(as_int >> (e * w)) & ((1 << w) - 1) for e in range(entries)] == idx[i].tolist()
        assert as_int >> (entries * w) == 0


# ---------------------------------------------------------------------------------------------
# the factorized layer applied to activations (Sec. 3.1, Sec. 4.4)
# ---------------------------------------------------------------------------------------------
def bf16_round(a):
    return synth.bf16_bits_to_f32(synth.to_bf16_bits(np.asarray(a, dtype=np.float32))).astype(np.float64)


@pytest.mark.parametrize("d_out,d_in,b,N,M", [(12, 16, 4, 2, 4), (16, 24, 8, 3, 8), (8, 8, 4, 1, 2), (8, 16, 8, 5, 8)])
def test_apply_packed_is_the_dense_product(orc, d_out, d_in, b, N, M):
    """Without rounding, y = A(S(Bx)) from the compressed core is X (A S B)^T with dense matrices:
    catches a transposed wrapper, a wrong block, a wrong in-group column."""
    rng = np.random.default_rng(61)
    _, _, A, B, C, mask = rand_state(rng, d_out, d_in, b, N=N, M=M, perturb=0.5)
    X = rng.standard_normal((5, d_in)).astype(np.float32)
    vals, idx = orc.pack_nm(C, mask, N, M)
    Y = orc.apply_packed(X, A, vals, idx, B, N, M, round_bf16=False)
    What = dense(A) @ C.astype(np.float64) @ dense(B)
    np.testing.assert_allclose(Y, X.astype(np.float64) @ What.T, rtol=1e-12, atol=1e-13)
    # identity wrappers: the plain N:M sparse product
    I_A, I_B = orc.identity_blocks(d_out // b, b), orc.identity_blocks(d_in // b, b)
    Y0 = orc.apply_packed(X, I_A, vals, idx, I_B, N, M, round_bf16=False)
    np.testing.assert_allclose(Y0, X.astype(np.float64) @ C.astype(np.float64).T, rtol=1e-12, atol=1e-13)


def test_apply_packed_rounds_the_two_intermediates_to_bf16(orc):
    """With rounding on, u = Bx and v = Su pass through bfloat16 (round to nearest even, checked
    against the input generator's own conversion); y itself is not rounded."""
    rng = np.random.default_rng(62)
    d_out, d_in, b = 16, 24, 8
    _, _, A, B, C, mask = rand_state(rng, d_out, d_in, b, perturb=0.5)
    X = bf16_round(rng.standard_normal((7, d_in))).astype(np.float32)
    vals, idx = orc.pack_nm(C, mask, 2, 4)
    Y = orc.apply_packed(X, A, vals, idx, B, 2, 4, round_bf16=True)
    u = bf16_round(X.astype(np.float64) @ dense(B).T)
    v = bf16_round(u @ C.astype(np.float64).T)
    np.testing.assert_allclose(Y, v @ dense(A).T, rtol=1e-9, atol=1e-12)
    exact = orc.apply_packed(X, A, vals, idx, B, 2, 4, round_bf16=False)
    assert 0 < np.abs(Y - exact).max() < 2.0 ** -6 * np.abs(exact).max()


# ---------------------------------------------------------------------------------------------
# Gram (Sec. 2 / Eq. 2)
# ---------------------------------------------------------------------------------------------
def test_gram_is_textbook_syrk(orc):
    X = synth.make_calibration(70, 24, seed=5, outlier_frac=0.1, outlier_scale=20.0)
    H = orc.gram(X)
    ref = X.astype(np.float64).T @ X.astype(np.float64)
    np.testing.assert_allclose(H, ref, rtol=1e-12, atol=1e-12)
    np.testing.assert_array_equal(H, H.T)
    assert np.linalg.eigvalsh(H).min() > -1e-9 * np.trace(H)
    np.testing.assert_allclose(np.diag(H), (X.astype(np.float64) ** 2).sum(0), rtol=1e-12)
    rows, cols = np.array([0, 3, 23, 7]), np.array([0, 5, 23, 2])
    np.testing.assert_allclose(orc.gram_entries(X, rows, cols), ref[rows, cols], rtol=1e-12)
    bits = synth.to_bf16_bits(X)
    Xb = synth.bf16_bits_to_f32(bits).astype(np.float64)
    np.testing.assert_allclose(orc.gram_entries(bits, rows, cols), (Xb.T @ Xb)[rows, cols], rtol=1e-12)


def test_bf16_rounding_helper():
    import torch
    x = np.random.default_rng(0).standard_normal(1000).astype(np.float32)
    bits = synth.to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(bits, ref)


# ---------------------------------------------------------------------------------------------
# joint Adam continuous step (Sec. 3.3.1, App. F)
# ---------------------------------------------------------------------------------------------
def _np_adam(theta, m, v, g, t, lr, b1, b2, eps):
    """Independent restatement of the published Adam update (with bias correction), fp64."""
    m = b1 * m + (1 - b1) * g
    v = b2 * v + (1 - b2) * g * g
    mhat, vhat = m / (1 - b1 ** t), v / (1 - b2 ** t)
    return theta - lr * mhat / (np.sqrt(vhat) + eps), m, v


def test_adam_step_matches_published_update_rule(orc):
    rng = np.random.default_rng(61)
    d_out, d_in, b = 8, 12, 4
    Wbar, D, A, B, C, mask = rand_state(rng, d_out, d_in, b, perturb=0.2)
    st = orc.adam_state(d_out, d_in, b)
    lr, b1, b2, eps = 1e-2, 0.9, 0.999, 1e-8
    A64, B64, C64 = A.astype(np.float64), B.astype(np.float64), C.astype(np.float64)
    m = {k: np.zeros_like(x) for k, x in (("A", A64), ("B", B64), ("C", C64))}
    v = {k: np.zeros_like(x) for k, x in (("A", A64), ("B", B64), ("C", C64))}
    Ao, Co, Bo = A, C, B
    for t in (1, 2, 3):
        # gradients of all three at the same point (pinned above by finite differences)
        gA, _ = orc.grad_A(Wbar, Ao, Co, Bo, D)
        gB, _ = orc.grad_B(Wbar, Ao, Co, Bo, D)
        gC, _ = orc.grad_core(Wbar, Ao, Co, Bo, D)
        gC = gC * mask
        eA, m["A"], v["A"] = _np_adam(Ao.astype(np.float64), m["A"], v["A"], gA, t, lr, b1, b2, eps)
        eB, m["B"], v["B"] = _np_adam(Bo.astype(np.float64), m["B"], v["B"], gB, t, lr, b1, b2, eps)
        eC, m["C"], v["C"] = _np_adam(Co.astype(np.float64), m["C"], v["C"], gC, t, lr, b1, b2, eps)
        eC = np.where(mask == 1, eC, 0.0)                       # pruned entries stay exactly zero
        Ao, Co, Bo, st = orc.adam_update(Wbar, D, mask, Ao, Co, Bo, st, t, lr=lr, b1=b1, b2=b2, eps=eps)
        np.testing.assert_allclose(Ao, eA, rtol=2e-6, atol=1e-7)
        np.testing.assert_allclose(Bo, eB, rtol=2e-6, atol=1e-7)
        np.testing.assert_allclose(Co, eC, rtol=2e-6, atol=1e-7)
        assert np.all(Co[mask == 0] == 0)
        np.testing.assert_allclose(st["mC"], m["C"], rtol=2e-6, atol=1e-9)
        np.testing.assert_allclose(st["vA"], v["A"], rtol=2e-6, atol=1e-12)
        m = {k: st["m" + k].astype(np.float64) for k in m}      # moments are fp32 state between steps
        v = {k: st["v" + k].astype(np.float64) for k in v}


def test_adam_first_step_moves_by_lr_against_the_gradient_sign(orc):
    """t = 1: m_hat = g, v_hat = g^2, so every entry with |g| >> eps moves by lr * sign(-g)."""
    rng = np.random.default_rng(67)
    d_out, d_in, b = 8, 8, 4
    Wbar, D, A, B, C, mask = rand_state(rng, d_out, d_in, b, perturb=0.2)
    gA, _ = orc.grad_A(Wbar, A, C, B, D)
    lr = 1e-3
    A1, C1, B1, _ = orc.adam_update(Wbar, D, mask, A, C, B, orc.adam_state(d_out, d_in, b), 1, lr=lr)
    big = np.abs(gA) > 1e-3
    np.testing.assert_allclose((A1.astype(np.float64) - A)[big], -lr * np.sign(gA[big]), rtol=1e-3)


def test_factorize_adam_reduces_loss_and_keeps_structure(orc):
    d_out, d_in, b = 32, 48, 16
    W = synth.make_weight(d_out, d_in, seed=1, outlier_frac=0.05)
    X = synth.make_calibration(96, d_in, seed=1)
    D = np.diag(orc.gram(X)).astype(np.float32)
    out = orc.factorize_layer_adam(W, D, b, 2, 4, n_iters=40, seed=3, lr=1e-3)
    tr, ct = out["loss_trace"], out["loss_cont_trace"]
    assert tr[-1] < 0.9 * tr[0]                                  # moves far faster than the 1/beta steps
    assert np.all(tr[1:] <= ct * (1 + 1e-9))                     # Lemma 2 still holds for the sparse step
    assert np.all(out["mask"].reshape(d_out, d_in // 4, 4).sum(-1) == 2)
    assert np.all(out["C"][out["mask"] == 0] == 0)
    assert tr[-1] == pytest.approx(dense_loss(out["Wbar"], out["A"], out["C"], out["B"], D), rel=1e-9)
    gd = orc.factorize_layer(W, D, b, 2, 4, n_iters=40, seed=3)
    assert tr[0] == gd["loss_trace"][0]                          # same initial point
