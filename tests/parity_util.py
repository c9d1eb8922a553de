"""Shared assertions of the GPU parity tests.

The bars the task states (A, S, B relative Frobenius error <= 1e-3, mask agreement >= 99.9 %, loss
within 0.5 %) are applied to what an iteration CHANGES, not to the iterate: under the global step
sizes of Eq. 9-11 a multi-block layer moves by 1e-5 .. 1e-3 of its norm in a few iterations, so a
bar on the iterate itself would also pass for a kernel that never moves.  For every parameter
theta in {A, S, B} with starting value theta_0:

    || (theta_gpu - theta_0) - (theta_ref - theta_0) ||_F  <=  1e-3 ||theta_ref - theta_0||_F + floor

floor = sqrt(t) * 2^-24 * ||theta_ref||_F: both sides keep the optimiser state in fp32 between
sub-steps; the oracle rounds an fp64 result, the kernels an fp32 one, so after each of the t
iterations an entry may land on the neighbouring fp32 value (half an ulp rms; this also covers the
fp32 cancellation in R = W-bar - A S B next to the initial point, where R is ~1e-6 of W-bar on the
kept entries).  The floor only matters where an update is a few ulps of what it moves: from the
initial point of Eq. 3 a layer with thousands of blocks moves its core by less than one ulp per
entry in its first iteration, which no fp32 implementation can resolve; the tests of such layers
therefore start both sides from a generic feasible point (theta_0 is an input of Alg. 1), where every
sub-step moves its parameter by 0.1 .. 20 %.  Where the two sides' starting values themselves differ by rounding (the core of Eq. 3 is the normalised weight, which the
kernels form with fp32 reciprocals), each side's update is taken from its own start.  The test prints how
far theta_0 itself is from the oracle's result in units of the tolerance and requires >= 10, i.e.
not moving fails by an order of magnitude.  Losses: the trace agrees to 2e-6 relative (fp32 block
sums) and every decrease L_0 - L_t to 0.5 % (+ 2e-6 L_0); the step sizes of Eq. 9-11 agree to 1e-5;
the per-iteration count of changed groups is an integer and must be equal.
"""
import sys

import numpy as np


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def relfro(a, b):
    a, b = np.asarray(a, dtype=np.float64), np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def identity_blocks(n, b):
    return np.tile(np.eye(b, dtype=np.float32), (n, 1, 1))


def assert_update_parity(name, got, ref, start, n_iters, min_margin=10.0, start_got=None):
    """The bar on the update of one parameter (see the module docstring).  Returns a report string."""
    if n_iters == 0:
        return "%s: no iterations" % name
    got, ref, start = (np.asarray(x, dtype=np.float64) for x in (got, ref, start))
    start_got = start if start_got is None else np.asarray(start_got, dtype=np.float64)
    upd = float(np.linalg.norm(ref - start))
    err = float(np.linalg.norm((got - start_got) - (ref - start)))
    floor = np.sqrt(n_iters) * 2.0 ** -24 * float(np.linalg.norm(ref))
    tol = 1e-3 * upd + floor
    rep = "%s: |update| %.3e  |gpu-ref| %.3e (%.2e of the update)  tol %.3e  start is %.0f tol away" % (
        name, upd, err, err / max(upd, 1e-300), tol, upd / tol)
    assert err <= tol, rep
    if min_margin is not None:
        assert upd >= min_margin * tol, "not discriminating: " + rep
    return rep


def assert_trace_parity(tr, ref_tr, what="loss trace"):
    tr, ref_tr = np.asarray(tr, dtype=np.float64), np.asarray(ref_tr, dtype=np.float64)
    np.testing.assert_allclose(tr, ref_tr, rtol=2e-6, err_msg=what)
    if tr.size > 1:
        dec, rdec = tr[0] - tr[1:], ref_tr[0] - ref_tr[1:]
        np.testing.assert_allclose(dec, rdec, rtol=5e-3, atol=2e-6 * ref_tr[0], err_msg=what + " decreases")
        return float(np.max(np.abs(dec - rdec) / np.maximum(np.abs(rdec), 1e-300)))
    return 0.0


def assert_diagnostics_parity(out, ref, n_iters, n_blocks):
    """Step sizes of Eq. 9-11 and the number of groups each sparse-core step changed (one group per
    block is refit; a draw or a pattern decided by a near-tie in fp32 may differ in at most 0.1 % of
    the blocks, the same allowance as the mask agreement bar: none below 1000 blocks)."""
    if n_iters == 0:
        return
    eta = out["eta_trace"].cpu().numpy()
    np.testing.assert_allclose(eta, ref["etas"], rtol=1e-5, err_msg="eta_A, eta_B, eta_W'")
    assert np.all(eta > 0)
    got = out["mask_changes"].cpu().numpy().astype(np.int64)
    assert np.all(np.abs(got - ref["mask_changes"]) <= n_blocks // 1000), (got, ref["mask_changes"])
