"""The allocation-free entry point (armor_proxy_loss_noalloc: scratch in a fixed array of the library's device
image) against armor_proxy_loss, through the C ABI: two calls in a row, the second on a smaller input, so the
second call sees the first call's leftovers in the shared scratch."""
import numpy as np
import pytest

from paper_2510_05528_amd import synth

pytestmark = pytest.mark.gpu


def test_noalloc_proxy_loss_matches_the_workspace_entry_point(orc):
    import torch
    import paper_2510_05528_amd as armor
    armor.load_library()
    dev = torch.device("cuda:0")

    def case(d_out, d_in, b, wrappers, seed):
        W = synth.make_weight(d_out, d_in, seed=seed)
        Wbar, _, _ = orc.normalize(W)
        D = (np.random.default_rng(seed).random(d_in) * 3 + 0.2).astype(np.float32)
        A, B, C, _ = synth.make_state(d_out, d_in, b, 2, 4, seed=seed)
        t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
        return dict(Wbar=Wbar, D=D, A=A, B=B, C=C, b=b, wrappers=wrappers,
                    dev=(t(Wbar), t(A) if wrappers else None, t(C), t(B) if wrappers else None, t(D)))

    # first a larger problem, then smaller ones (all share the library's scratch), then the large one again
    cases = [case(512, 768, 128, True, 1), case(128, 192, 64, False, 2), case(512, 768, 256, True, 3),
             case(256, 256, 256, False, 4), case(96, 160, 32, True, 5)]
    out = torch.zeros(1, device=dev, dtype=torch.float64)
    for c in cases + cases[:1]:
        Wd, Ad, Cd, Bd, Dd = c["dev"]
        want = armor.proxy_loss(Wd, Ad, Cd, Bd, Dd, d_block=c["b"]).item()
        got = armor.proxy_loss_noalloc(Wd, Ad, Cd, Bd, Dd, d_block=c["b"], out=out).item()
        assert got == want, (c["b"], got, want)                       # same kernels, same order of sums
        eye = lambda n: np.tile(np.eye(c["b"], dtype=np.float32), (n, 1, 1))
        A = c["A"] if c["wrappers"] else eye(c["Wbar"].shape[0] // c["b"])
        B = c["B"] if c["wrappers"] else eye(c["Wbar"].shape[1] // c["b"])
        assert got == pytest.approx(orc.proxy_loss(c["Wbar"], A, c["C"], B, c["D"]), rel=2e-5)
    # H as a full matrix: only its diagonal is read
    c = cases[1]
    Wd, _, Cd, _, Dd = c["dev"]
    H = torch.diag(Dd) + 0.01
    H.diagonal().copy_(Dd)
    assert armor.proxy_loss_noalloc(Wd, None, Cd, None, H, d_block=c["b"], out=out).item() == \
        armor.proxy_loss(Wd, None, Cd, None, H, d_block=c["b"]).item()
    # beyond the fixed scratch: the identity wrappers of a 16384 x 16384 layer at d_block 256 alone take 32 MiB
    lib = armor.load_library()
    p = Wd.data_ptr()
    assert lib.armor_proxy_loss_noalloc(p, None, p, None, p, 0, 16384, 16384, 256, out.data_ptr(), None) == 9
