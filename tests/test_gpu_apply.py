"""The factorized layer applied to activations (Sec. 3.1 / Sec. 4.4): armor_apply_packed against the
oracle's y = A (S (B x)) with the same bf16 rounding points, through the C ABI.

Tolerance (derived from the arithmetic; bf16 keeps 8 significant bits, so one ulp is at most 2^-7
and a rounding error at most 2^-8, relative).  Both sides round u = Bx and v = Su to bf16 at the same
points; they differ by fp32-vs-fp64 accumulation (~1e-6 relative), which now and then straddles a
rounding boundary and moves one intermediate by a whole ulp, and the GPU result is rounded to bf16
once more.  With wrappers near the identity the dominant term of y_p is A_pp v_p, so one such flip
moves y_p by up to 2^-7 |y_p|.  Hence for every element
    |y_gpu - y_ref|_p <= 2^-8 |y_ref|_p + 1.1 * 2^-7 (|A| |v|)_p    (final rounding; every v_q off by an
                                                                    ulp, 10 % on top for flips in u),
at least 99 % of the elements see the final rounding alone, 2^-8 |y_ref| + 2^-10 rms(y_ref), and the
relative Frobenius error stays <= 3e-3."""
import sys

import numpy as np
import pytest

from paper_2510_05528_amd import synth

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def env():
    import torch
    import paper_2510_05528_amd as armor
    armor.load_library()
    return armor, torch, torch.device("cuda:0")


def make_factors(rng, d_out, d_in, b, perturb=0.2):
    A = np.stack([np.eye(b) + perturb * rng.standard_normal((b, b)) / np.sqrt(b) for _ in range(d_out // b)]).astype(np.float32)
    B = np.stack([np.eye(b) + perturb * rng.standard_normal((b, b)) / np.sqrt(b) for _ in range(d_in // b)]).astype(np.float32)
    scores = rng.random((d_out, d_in // 4, 4))
    keep = np.argsort(-scores, axis=-1)[..., :2]
    mask = np.zeros((d_out, d_in // 4, 4), dtype=np.uint8)
    np.put_along_axis(mask, keep, 1, axis=-1)
    mask = mask.reshape(d_out, d_in)
    S = (rng.standard_normal((d_out, d_in)) * 0.05 * mask).astype(np.float32)
    return A, B, S, mask


def bf16_to_np(torch, t):
    return t.float().cpu().numpy()


def run_case(armor, torch, orc, dev, n, d_out, d_in, b, seed):
    rng = np.random.default_rng(seed)
    A, B, S, mask = make_factors(rng, d_out, d_in, b)
    X = rng.standard_normal((n, d_in)).astype(np.float32)
    X[:, :: 37] *= 6.0  # a few large channels, as in the calibration recipe
    bits = (mask.reshape(d_out, d_in // 4, 4).astype(np.uint32) << np.arange(4, dtype=np.uint32)).sum(-1).astype(np.uint8)
    Sd = torch.from_numpy(S).to(dev)
    vals, meta = armor.pack_nm(Sd, torch.from_numpy(bits).to(dev), 2, 4, bf16=True)
    Ab, Bb = armor.to_bf16(torch.from_numpy(A).to(dev)), armor.to_bf16(torch.from_numpy(B).to(dev))
    Xb = torch.from_numpy(X).to(dev).to(torch.bfloat16)
    say("apply n=%d d_out=%d d_in=%d b=%d" % (n, d_out, d_in, b))
    prepared = armor.apply_prepare(vals, meta, 2, 4)
    Y = armor.apply_packed(Xb, Ab, prepared, Bb, 2, 4)
    torch.cuda.synchronize()
    # the oracle sees exactly the bf16 operands the kernels saw
    ev, ei = orc.pack_nm(S, mask, 2, 4)
    ev_bf = synth.bf16_bits_to_f32(synth.to_bf16_bits(ev))
    np.testing.assert_array_equal(bf16_to_np(torch, vals), ev_bf)
    ref = orc.apply_packed(bf16_to_np(torch, Xb), bf16_to_np(torch, Ab), ev_bf, ei, bf16_to_np(torch, Bb), 2, 4,
                           round_bf16=True)
    got = bf16_to_np(torch, Y).astype(np.float64)
    assert got.shape == ref.shape
    err = np.abs(got - ref)
    rms = np.sqrt((ref ** 2).mean())
    eye = np.stack([np.eye(b, dtype=np.float32)] * (d_out // b))
    v = orc.apply_packed(bf16_to_np(torch, Xb), eye, ev_bf, ei, bf16_to_np(torch, Bb), 2, 4, round_bf16=True)
    absA = np.abs(bf16_to_np(torch, Ab).astype(np.float64))
    Av = np.einsum("ipq,tiq->tip", absA, np.abs(v).reshape(n, d_out // b, b)).reshape(n, d_out)
    bound = 2.0 ** -8 * np.abs(ref) + 1.1 * 2.0 ** -7 * Av
    typical = 2.0 ** -8 * np.abs(ref) + 2.0 ** -10 * rms
    frac_in = float((err <= typical).mean())
    relf = float(np.linalg.norm(got - ref) / np.linalg.norm(ref))
    say("   relF %.2e, final-rounding-only fraction %.5f, worst err/bound %.2f" % (relf, frac_in, float((err / bound).max())))
    assert relf <= 3e-3
    assert frac_in >= 0.99
    assert np.all(err <= bound)


@pytest.mark.parametrize("n,d_out,d_in,b", [(300, 512, 768, 128), (1000, 384, 640, 64), (64, 96, 128, 32),
                                            (257, 256, 64, 32), (5, 128, 192, 64), (513, 640, 256, 128),
                                            (300, 512, 768, 256), (700, 768, 256, 256)])
def test_apply_packed_matches_oracle(env, orc, n, d_out, d_in, b):
    """Several row tiles and token tiles, ragged tails in both, every wrapper block size, one-stage K."""
    armor, torch, dev = env
    run_case(armor, torch, orc, dev, n, d_out, d_in, b, seed=n + d_out)


def test_apply_after_factorization(env, orc):
    """End to end: factorize a layer (denormalised wrappers), pack, apply; the result approximates
    X W^T as well as the factorization's proxy loss says, and matches the oracle's apply."""
    armor, torch, dev = env
    d_out, d_in, b, n = 256, 384, 128, 200
    W = synth.make_weight(d_out, d_in, seed=21)
    Xc = synth.make_calibration(512, d_in, seed=22)
    D = (Xc.astype(np.float64) ** 2).sum(0).astype(np.float32)
    out = armor.factorize_layer(torch.from_numpy(W).to(dev), torch.from_numpy(D).to(dev), b, 2, 4, 5, seed=3, denormalize=True)
    vals, meta = armor.pack_nm(out["S"], out["mask_bits"], 2, 4, bf16=True)
    Ab, Bb = armor.to_bf16(out["A"]), armor.to_bf16(out["B"])
    Xb = torch.from_numpy(Xc[:n]).to(dev).to(torch.bfloat16)
    Y = armor.apply_packed(Xb, Ab, armor.apply_prepare(vals, meta, 2, 4), Bb, 2, 4)
    torch.cuda.synchronize()
    mask = armor.unpack_mask(out["mask_bits"].cpu().numpy(), 4)
    ev, ei = orc.pack_nm(out["S"].cpu().numpy(), mask, 2, 4)
    ref = orc.apply_packed(Xb.float().cpu().numpy(), Ab.float().cpu().numpy(), synth.bf16_bits_to_f32(synth.to_bf16_bits(ev)),
                           ei, Bb.float().cpu().numpy(), 2, 4, round_bf16=True)
    got = Y.float().cpu().numpy().astype(np.float64)
    assert np.linalg.norm(got - ref) / np.linalg.norm(ref) <= 3e-3
    dense = Xb.float().cpu().numpy().astype(np.float64) @ W.astype(np.float64).T
    # 2:4 pruning keeps most of the layer's action on calibration-like inputs
    assert np.linalg.norm(got - dense) / np.linalg.norm(dense) < 0.9


def test_apply_edge_cases(env):
    armor, torch, dev = env
    b, d_out, d_in = 32, 64, 64
    A = torch.zeros((d_out // b, b, b), device=dev, dtype=torch.bfloat16)
    Bw = torch.zeros((d_in // b, b, b), device=dev, dtype=torch.bfloat16)
    vals = torch.zeros((d_out, d_in // 2), device=dev, dtype=torch.bfloat16)
    meta = torch.zeros((d_out, d_in // 8), device=dev, dtype=torch.uint8)
    prepared = armor.apply_prepare(vals, meta, 2, 4)
    X0 = torch.zeros((0, d_in), device=dev, dtype=torch.bfloat16)
    assert armor.apply_packed(X0, A, prepared, Bw, 2, 4).shape == (0, d_out)       # no tokens: no-op
    X = torch.ones((3, d_in), device=dev, dtype=torch.bfloat16)
    with pytest.raises(armor.ArmorError):
        armor.apply_packed(X, A, prepared, Bw, 4, 8)                                 # only 2:4 on this path
    Y = armor.apply_packed(X, A, prepared, Bw, 2, 4)                                 # all-zero factors
    torch.cuda.synchronize()
    assert float(Y.float().abs().max()) == 0.0
