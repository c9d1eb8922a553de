"""Parity on the shapes of BASELINE configs 3-5 (Llama-7B MLP, Llama-3-8B GQA projections,
Llama-3-70B-shaped d_block = 256 stress with 2:4 / 4:8 / unstructured), at sizes the oracle can
follow: real layer shapes with one oracle iteration where the layer is large, or the reduced layer
of the same law (1024 x 8192 at d_block 256) with several iterations."""
import sys

import numpy as np
import pytest

from paper_2510_05528_amd import synth

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def relfro(a, b):
    return float(np.linalg.norm(a.astype(np.float64) - b.astype(np.float64)) / max(np.linalg.norm(b.astype(np.float64)), 1e-300))


@pytest.fixture(scope="module")
def env():
    import torch
    import paper_2510_05528_amd as armor
    armor.load_library()
    return armor, torch, torch.device("cuda:0")


def compare(armor, torch, orc, W, D, b, N, M, n_iters, seed, sparsity=0, keep=0, long_iters=0):
    """Element-wise parity after n_iters; then (optionally) properties of a longer run."""
    d_out, d_in = W.shape
    dev = W.device
    Wh, Dh = W.float().cpu().numpy(), D.cpu().numpy()
    mg = 8 if sparsity else M
    out = armor.factorize_layer(W, D, b, N, M, n_iters, seed=seed, sparsity=sparsity, unstructured_keep=keep,
                                want_cont_trace=True)
    torch.cuda.synchronize()
    ref = orc.factorize_layer(Wh, Dh, b, N, M, n_iters, seed=seed, sparsity=sparsity, keep=keep)
    mask = armor.unpack_mask(out["mask_bits"].cpu().numpy(), mg)
    S = out["S"].cpu().numpy()
    agree = float((mask == ref["mask"]).mean())
    eA, eB, eS = relfro(out["A"].cpu().numpy(), ref["A"]), relfro(out["B"].cpu().numpy(), ref["B"]), relfro(S, ref["C"])
    say("   %dx%d b=%d %d:%d sparsity=%d iters=%d: mask agreement %.7f relF A %.2e B %.2e S %.2e" %
        (d_out, d_in, b, N, M, sparsity, n_iters, agree, eA, eB, eS))
    if sparsity == 0:
        assert np.all(mask.reshape(d_out, d_in // M, M).sum(-1) == N)
    else:
        assert int(mask.sum()) == keep
    assert np.all(S[mask == 0] == 0)
    assert agree >= 0.999 and eA <= 1e-3 and eB <= 1e-3 and eS <= 1e-3
    np.testing.assert_allclose(out["loss_trace"].cpu().numpy(), ref["loss_trace"], rtol=5e-3)
    if long_iters:
        lo = armor.factorize_layer(W, D, b, N, M, long_iters, seed=seed, sparsity=sparsity, unstructured_keep=keep,
                                   want_cont_trace=True)
        torch.cuda.synchronize()
        tr, ct = lo["loss_trace"].cpu().numpy(), lo["loss_cont_trace"].cpu().numpy()
        tol = 1e-6 * tr[0]
        assert np.all(np.diff(tr) <= tol) and np.all(ct <= tr[:-1] + tol) and np.all(tr[1:] <= ct + tol)
        lmask = armor.unpack_mask(lo["mask_bits"].cpu().numpy(), mg)
        if sparsity == 0:
            assert np.all(lmask.reshape(d_out, d_in // M, M).sum(-1) == N)
        lref = orc.proxy_loss(ref["Wbar"], lo["A"].cpu().numpy(), lo["S"].cpu().numpy(), lo["B"].cpu().numpy(), Dh)
        assert tr[-1] == pytest.approx(lref, rel=1e-4)
    return out, ref


def test_config3_mlp_shapes(env, orc):
    """Llama-7B MLP: gate/up 11008x4096 on the shared 4096-wide Gram, down 4096x11008 on the Gram of
    SiLU(gate)*up activations (heavy-tailed).  One oracle iteration each, 10-iteration properties."""
    armor, torch, dev = env
    n_tok = 8192
    say("config3: inputs")
    X = synth.torch_calibration(n_tok, 4096, 3, dev, outlier_frac=0.005, outlier_scale=20.0)
    Wg = synth.torch_weight(11008, 4096, 31, dev)
    Wu = synth.torch_weight(11008, 4096, 32, dev)
    Wd = synth.torch_weight(4096, 11008, 33, dev)
    H = armor.gram(X)
    D = armor.gram_diag(H)
    say("config3: gate_proj 11008x4096")
    compare(armor, torch, orc, Wg, D, 128, 2, 4, 1, seed=0, long_iters=10)
    say("config3: down_proj 4096x11008")
    Xd = synth.torch_mlp_down_inputs(X, Wg * 8.0, Wu * 8.0)       # x8: keep activations O(1) at init scale 0.02
    Hd = armor.gram(Xd)
    Dd = armor.gram_diag(Hd)
    # Gram of the heavy-tailed activations: diagonal against the oracle, one entry at a time
    bits = Xd.view(torch.int16).cpu().numpy().view(np.uint16)
    idx = np.random.default_rng(1).integers(0, 11008, 512)
    ref = orc.gram_entries(bits, idx, idx)
    np.testing.assert_allclose(Dd.cpu().numpy()[idx], ref, rtol=2e-5)
    compare(armor, torch, orc, Wd, Dd, 128, 2, 4, 1, seed=0, long_iters=10)


def test_adam_multi_block_chunks(env, orc):
    """Joint-Adam variant where a workgroup of the forward/backward chain walks more than one block
    (18 x 32 blocks of 128 on 512 workgroup slots: chunks of two column blocks) and the core-gradient
    chain more than one block per workgroup.  One iteration from theta_0 is determined to rounding."""
    armor, torch, dev = env
    d_out, d_in, b = 2304, 4096, 128
    W = synth.torch_weight(d_out, d_in, 51, dev)
    D = (torch.rand(d_in, device=dev, generator=torch.Generator(device=dev).manual_seed(7)) + 0.5).float()
    Wh, Dh = W.float().cpu().numpy(), D.cpu().numpy()
    say("adam, chunks of two: %dx%d" % (d_out, d_in))
    out = armor.factorize_layer(W, D, b, 2, 4, 1, seed=3, variant=1, lr=1e-3)
    torch.cuda.synchronize()
    ref = orc.factorize_layer_adam(Wh, Dh, b, 2, 4, 1, seed=3, lr=1e-3)
    # Adam's first step is lr * sign(g) on every entry: an entry whose gradient is zero up to rounding may
    # take either sign in any implementation.  Everything else agrees to rounding.
    lr = 1e-3
    for k, rk in (("A", "A"), ("B", "B"), ("S", "C")):
        d = np.abs(out[k].cpu().numpy().astype(np.float64) - ref[rk])
        nbad = int((d > 1e-6).sum())
        say("   %s: max diff %.2e, entries off by more than 1e-6: %d of %d" % (k, d.max(), nbad, d.size))
        assert d.max() <= 2 * lr * (1 + 1e-3) and nbad <= max(4, d.size // 100000), k
    agree = float((armor.unpack_mask(out["mask_bits"].cpu().numpy(), 4) == ref["mask"]).mean())
    assert agree >= 0.99999
    np.testing.assert_allclose(out["loss_trace"].cpu().numpy(), ref["loss_trace"], rtol=1e-5)


def test_config4_gqa_kv_shape(env, orc):
    """Llama-3-8B k/v projection: 1024x4096 (8 x 32 blocks), full parity over 3 iterations."""
    armor, torch, dev = env
    X = synth.torch_calibration(8192, 4096, 4, dev, outlier_frac=0.005, outlier_scale=20.0)
    D = armor.gram_diag(armor.gram(X))
    W = synth.torch_weight(1024, 4096, 41, dev)
    compare(armor, torch, orc, W, D, 128, 2, 4, 3, seed=0, long_iters=20)


@pytest.mark.parametrize("N,M,sparsity", [(2, 4, 0), (4, 8, 0), (2, 4, 1)])
def test_config5_reduced_block256(env, orc, N, M, sparsity):
    """Llama-3-70B-shaped stress at the reduced layer of the same law: 1024x8192, d_block 256,
    2:4, 4:8 and 50 % unstructured, 3 iterations of full parity + 10-iteration properties."""
    armor, torch, dev = env
    X = synth.torch_calibration(4096, 8192, 5, dev, outlier_frac=0.005, outlier_scale=20.0)
    D = armor.gram_diag(armor.gram(X))
    W = synth.torch_weight(1024, 8192, 51, dev)
    keep = (1024 * 8192) // 2 if sparsity else 0
    compare(armor, torch, orc, W, D, 256, N, M, 3, seed=0, sparsity=sparsity, keep=keep, long_iters=10)
