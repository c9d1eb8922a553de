"""Seeded synthetic inputs shaped like the paper's workloads (LLM linear layers and calibration
activations).  This module holds no arithmetic of the method itself: it only draws weights and
activations.  Both the HIP path and the CPU oracle receive the arrays produced here.

Recipe (stands in for the Llama / Qwen layers and the SlimPajama calibration activations the
paper uses, which are not available offline):
  * W ~ N(0, 0.02^2), with a fraction of the input columns scaled up (outlier channels);
  * calibration tokens x ~ N(0, Sigma), Sigma = Q diag(lambda) Q^T, lambda_i = 1/(1 + i/8), Q a
    random orthogonal matrix (QR of a Gaussian, signs fixed), plus a fraction of channels scaled
    up (outlier activations);
  * MLP down-projection inputs are SiLU(x Wg^T) * (x Wu^T) of such tokens (heavy tailed).
"""
import numpy as np


def make_weight(d_out, d_in, seed=0, outlier_frac=0.02, outlier_scale=8.0, std=0.02):
    rng = np.random.default_rng([seed, 1])
    W = rng.standard_normal((d_out, d_in)).astype(np.float32) * np.float32(std)
    n_out = int(round(outlier_frac * d_in))
    if n_out > 0:
        cols = rng.choice(d_in, size=n_out, replace=False)
        W[:, cols] *= np.float32(outlier_scale)
    return W


def _mixing(d_in, rng):
    G = rng.standard_normal((d_in, d_in))
    Q, Rr = np.linalg.qr(G)
    Q = Q * np.sign(np.diag(Rr))[None, :]
    lam = 1.0 / (1.0 + np.arange(d_in) / 8.0)
    return (np.sqrt(lam)[:, None] * Q.T)  # x = z @ (Lambda^{1/2} Q^T)  =>  cov = Q Lambda Q^T


def make_calibration(n_tokens, d_in, seed=0, outlier_frac=0.0, outlier_scale=1.0):
    """[n_tokens, d_in] fp32; one token per row."""
    rng = np.random.default_rng([seed, 2])
    mix = _mixing(d_in, rng)
    Z = rng.standard_normal((n_tokens, d_in))
    X = Z @ mix
    n_out = int(round(outlier_frac * d_in))
    if n_out > 0:
        cols = rng.choice(d_in, size=n_out, replace=False)
        X[:, cols] *= outlier_scale
    return X.astype(np.float32)


def to_bf16_bits(x):
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns (numpy has no bf16)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    r = ((u >> 16) & 1) + 0x7FFF
    return ((u + r) >> 16).astype(np.uint16)


def bf16_bits_to_f32(h):
    return (np.ascontiguousarray(h, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


# ------------------------------------------------------------------------------------------------
# Full-size inputs are drawn directly in device memory with torch's seeded generator (harness
# work, outside every timed region); the same tensors are copied to the host for the oracle.
# ------------------------------------------------------------------------------------------------
def torch_weight(d_out, d_in, seed, device, outlier_frac=0.02, outlier_scale=8.0, std=0.02, bf16=True):
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(1000 + seed)
    W = torch.randn((d_out, d_in), generator=g, device=device, dtype=torch.float32) * std
    n_out = int(round(outlier_frac * d_in))
    if n_out > 0:
        cols = torch.randperm(d_in, generator=g, device=device)[:n_out]
        W[:, cols] *= outlier_scale
    return W.to(torch.bfloat16) if bf16 else W


def torch_mixing(d_in, seed, device):
    """Lambda^{1/2} Q^T on the device; the QR itself runs on the host (numpy, seeded)."""
    import torch
    rng = np.random.default_rng([seed, 3])
    return torch.from_numpy(_mixing(d_in, rng).astype(np.float32)).to(device)


def torch_calibration(n_tokens, d_in, seed, device, outlier_frac=0.005, outlier_scale=20.0,
                      chunk=16384, dtype=None):
    """[n_tokens, d_in] activations in device memory (bf16 by default), drawn chunk by chunk."""
    import torch
    dtype = dtype or torch.bfloat16
    mix = torch_mixing(d_in, seed, device)
    g = torch.Generator(device=device)
    g.manual_seed(3000 + seed)
    n_out = int(round(outlier_frac * d_in))
    cols = torch.randperm(d_in, generator=g, device=device)[:n_out]
    X = torch.empty((n_tokens, d_in), device=device, dtype=dtype)
    for s in range(0, n_tokens, chunk):
        e = min(n_tokens, s + chunk)
        Z = torch.randn((e - s, d_in), generator=g, device=device, dtype=torch.float32)
        Y = Z @ mix
        if n_out > 0:
            Y[:, cols] *= outlier_scale
        X[s:e] = Y.to(dtype)
    return X


def torch_mlp_down_inputs(X, Wg, Wu, chunk=8192):
    """SiLU(x Wg^T) * (x Wu^T) for MLP down-projection calibration inputs (same dtype as X)."""
    import torch
    out = torch.empty((X.shape[0], Wg.shape[0]), device=X.device, dtype=X.dtype)
    for s in range(0, X.shape[0], chunk):
        x = X[s:s + chunk].float()
        out[s:s + chunk] = (torch.nn.functional.silu(x @ Wg.float().T) * (x @ Wu.float().T)).to(X.dtype)
    return out


def make_state(d_out, d_in, b, N, M, seed=0, perturb=0.3, core_std=None):
    """A generic feasible starting point for the iteration (not the initial point of the method):
    wrappers I + perturb/sqrt(b) * N(0,1) (so their spectrum stays near 1 at any block size), a
    uniformly random N-of-M mask per group and N(0, core_std^2) values on the kept entries
    (core_std defaults to 1/sqrt(d_in), the scale of a row-normalised weight).
    Returns (A [d_out/b,b,b], B [d_in/b,b,b], C [d_out,d_in], mask [d_out,d_in] uint8)."""
    rng = np.random.default_rng([seed, 4])
    sc = perturb / np.sqrt(b)
    A = (np.eye(b)[None] + sc * rng.standard_normal((d_out // b, b, b))).astype(np.float32)
    B = (np.eye(b)[None] + sc * rng.standard_normal((d_in // b, b, b))).astype(np.float32)
    order = np.argsort(rng.random((d_out, d_in // M, M), dtype=np.float32), axis=-1)
    mask = (order < N).astype(np.uint8).reshape(d_out, d_in)
    std = core_std if core_std is not None else 1.0 / np.sqrt(d_in)
    C = rng.standard_normal((d_out, d_in), dtype=np.float32) * np.float32(std) * mask
    return A, B, C, mask
