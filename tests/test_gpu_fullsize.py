"""Parity at the full size and launch configuration that bench.py times (BASELINE config 2:
Llama-7B-shaped 4096x4096 bf16 weight, 262144 x 4096 bf16 calibration tokens, d_block 128, 2:4).

The oracle cannot run 50 iterations of this layer in seconds, so:
  * Gram: full diagonal + sampled off-diagonal entries, each computed one by one by the oracle;
  * first two BCD iterations: full element-wise parity of A, S, B, mask and the loss trace;
  * 50 iterations: properties that hold at any size (N:M structure, monotone trace, closed-form
    L_0) and the oracle's evaluation of the loss of the returned factors.
"""
import sys

import numpy as np
import pytest

from paper_2510_05528_amd import synth

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def relfro(a, b):
    return float(np.linalg.norm(a.astype(np.float64) - b.astype(np.float64)) / np.linalg.norm(b.astype(np.float64)))


def test_config2_full_size(orc):
    import torch
    import paper_2510_05528_amd as armor
    armor.load_library()
    dev = torch.device("cuda:0")
    d_out = d_in = 4096
    n_tok, b, N, M = 262144, 128, 2, 4
    say("config2: generating inputs")
    W = synth.torch_weight(d_out, d_in, 0, dev, bf16=True)
    X = synth.torch_calibration(n_tok, d_in, 0, dev, outlier_frac=0.005, outlier_scale=20.0)
    say("config2: gram")
    H = armor.gram(X)
    D = armor.gram_diag(H)
    torch.cuda.synchronize()
    Hh = H.cpu().numpy()
    Xbits = X.view(torch.int16).cpu().numpy().view(np.uint16)
    rng = np.random.default_rng(0)
    rows = np.concatenate([np.arange(d_in), rng.integers(0, d_in, 4096)])
    cols = np.concatenate([np.arange(d_in), rng.integers(0, d_in, 4096)])
    say("config2: oracle gram entries", rows.size)
    ref = orc.gram_entries(Xbits, rows, cols)
    diag = ref[:d_in]
    scale = np.sqrt(diag[rows] * diag[cols])
    assert np.max(np.abs(Hh[rows, cols] - ref) / scale) < 2e-5
    np.testing.assert_array_equal(Hh[rows, cols], Hh[cols, rows])
    del Xbits

    Wh = W.float().cpu().numpy()
    Dh = D.cpu().numpy()
    ws = torch.empty(armor.factorize_workspace_bytes(d_out, d_in, b, N, M), device=dev, dtype=torch.uint8)
    say("config2: 2 iterations on GPU and oracle")
    out2 = armor.factorize_layer(W, D, b, N, M, 2, seed=0, ws=ws, want_cont_trace=True)
    torch.cuda.synchronize()
    ref2 = orc.factorize_layer(Wh, Dh, b, N, M, 2, seed=0)
    mask2 = armor.unpack_mask(out2["mask_bits"].cpu().numpy(), M)
    agree = float((mask2 == ref2["mask"]).mean())
    eA, eB = relfro(out2["A"].cpu().numpy(), ref2["A"]), relfro(out2["B"].cpu().numpy(), ref2["B"])
    eS = relfro(out2["S"].cpu().numpy(), ref2["C"])
    say("   mask agreement %.7f relF A %.2e B %.2e S %.2e" % (agree, eA, eB, eS))
    assert agree >= 0.999 and eA <= 1e-3 and eB <= 1e-3 and eS <= 1e-3
    np.testing.assert_allclose(out2["loss_trace"].cpu().numpy(), ref2["loss_trace"], rtol=1e-5)
    np.testing.assert_allclose(out2["loss_cont_trace"].cpu().numpy(), ref2["loss_cont_trace"], rtol=1e-5)

    say("config2: 50 iterations on GPU")
    out = armor.factorize_layer(W, D, b, N, M, 50, seed=0, ws=ws, want_cont_trace=True)
    torch.cuda.synchronize()
    tr = out["loss_trace"].cpu().numpy()
    ct = out["loss_cont_trace"].cpu().numpy()
    mask = armor.unpack_mask(out["mask_bits"].cpu().numpy(), M)
    S = out["S"].cpu().numpy()
    assert np.all(mask.reshape(d_out, d_in // M, M).sum(-1) == N)           # bit-exact structure
    assert np.all(S[mask == 0] == 0)
    tol = 1e-6 * tr[0]
    assert np.all(np.diff(tr) <= tol) and np.all(ct <= tr[:-1] + tol) and np.all(tr[1:] <= ct + tol)
    assert tr[-1] < tr[0]
    Wbar = ref2["Wbar"]
    imp = (Wbar.astype(np.float64) ** 2) * Dh.astype(np.float64)[None, :]
    l0 = np.sort(imp.reshape(d_out, d_in // M, M), axis=-1)[..., : M - N].sum()
    assert tr[0] == pytest.approx(l0, rel=1e-5)                               # plain 2:4 pruning loss
    say("config2: oracle loss of the returned factors")
    lref = orc.proxy_loss(Wbar, out["A"].cpu().numpy(), S, out["B"].cpu().numpy(), Dh)
    assert tr[-1] == pytest.approx(lref, rel=1e-5)
    # the first two iterations of the long run are the short run (same seed, deterministic)
    np.testing.assert_array_equal(tr[:2], out2["loss_trace"].cpu().numpy()[:2])
