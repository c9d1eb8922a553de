"""The C-ABI library loads on a machine without a GPU and exports every symbol the header declares."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "armor.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(armor_[a-z_0-9]+)\s*\(", text)))


def test_header_symbols_are_exported():
    from paper_2510_05528_amd import binding
    lib = binding.load_library()
    names = _declared_symbols()
    assert set(names) == set(binding.EXPORTED), (names, binding.EXPORTED)
    for n in names:
        assert getattr(lib, n) is not None


def test_status_strings_and_host_side_validation():
    """Argument errors are detected on the host before any launch (no GPU needed)."""
    from paper_2510_05528_amd import binding
    lib = binding.load_library()
    assert lib.armor_status_string(0) == b"ok"
    assert lib.armor_status_string(2) == b"bad shape"
    # workspace queries are pure host arithmetic; bad shapes give 0
    assert lib.armor_factorize_workspace_bytes(256, 256, 32, 2, 4, None) > 2 * 256 * 256 * 4
    assert lib.armor_factorize_workspace_bytes(256, 250, 32, 2, 4, None) == 0      # b does not divide d_in
    assert lib.armor_factorize_workspace_bytes(256, 256, 48, 2, 4, None) == 0      # unsupported block size
    assert lib.armor_factorize_workspace_bytes(256, 256, 32, 4, 4, None) == 0      # N >= M
    assert lib.armor_factorize_workspace_bytes(256, 256, 32, 2, 3, None) == 0      # M not 2/4/8
    assert lib.armor_factorize_workspace_bytes(128, 1 << 23, 128, 2, 4, None) == 0  # d_block * d_in beyond 2^29
    assert lib.armor_factorize_workspace_bytes(128, 1 << 22, 128, 2, 4, None) > 0
    assert lib.armor_proxy_loss_workspace_bytes(128, 128, 64) > 0
    # null pointers / bad shapes are rejected without touching the device
    assert lib.armor_gram(None, 0, 16, 64, 64, None, 64, 0, None, 0, None) == 1
    buf = (ctypes.c_float * 64)()
    p = ctypes.cast(buf, ctypes.c_void_p)
    assert lib.armor_gram(p, 0, 16, 48, 48, p, 48, 0, None, 0, None) == 2                   # d_in not a multiple of 32
    assert lib.armor_gram(p, 7, 16, 64, 64, p, 64, 0, None, 0, None) == 3                   # dtype
    assert lib.armor_factorize_layer(None, 0, None, 0, 64, 64, 32, 2, 4, 1, None, None, None, None, None, None, None,
                                     None, None, None, None, None, 0, None) == 1
    assert lib.armor_factorize_layer(p, 0, p, 0, 64, 64, 32, 2, 4, 1, None, p, p, p, None, None, None, None, None, None,
                                     None, None, 0, None) == 4                    # no workspace
    assert lib.armor_factorize_layer(p, 0, p, 0, 64, 60, 32, 2, 4, 1, None, p, p, p, None, None, None, None, None, None,
                                     None, p, 1 << 30, None) == 2
    # starting from the caller's state needs its mask; negative / absurd iteration offsets are rejected
    o = binding.ArmorOpts(init_from_outputs=1)
    assert lib.armor_factorize_layer(p, 0, p, 0, 64, 64, 32, 2, 4, 1, ctypes.byref(o), p, p, p, None, None, None, None,
                                     None, None, None, p, 1 << 30, None) == 1
    for bad in (binding.ArmorOpts(iter_offset=-1), binding.ArmorOpts(iter_offset=1 << 31),
                binding.ArmorOpts(init_from_outputs=2), binding.ArmorOpts(check_finite=-1),
                binding.ArmorOpts(tol=-1e-3), binding.ArmorOpts(tol=float("nan")), binding.ArmorOpts(tol=2.0)):
        assert lib.armor_factorize_layer(p, 0, p, 0, 64, 64, 32, 2, 4, 1, ctypes.byref(bad), p, p, p, p, None, None,
                                         None, None, None, None, p, 1 << 30, None) == 2
    tol_adam = binding.ArmorOpts(tol=1e-3, variant=1)   # the joint-Adam variant cannot discard a forward pass
    assert lib.armor_factorize_layer(p, 0, p, 0, 64, 64, 32, 2, 4, 1, ctypes.byref(tol_adam), p, p, p, p, None, None,
                                     None, None, None, None, p, 1 << 30, None) == 7
    assert lib.armor_status_string(8).startswith(b"non-finite")
    # the loss against the whole Gram matrix: its workspace also holds the residual
    assert lib.armor_proxy_loss_full_h_workspace_bytes(128, 128, 64) > lib.armor_proxy_loss_workspace_bytes(128, 128, 64) + 4 * 128 * 128
    assert lib.armor_proxy_loss_full_h_workspace_bytes(128, 100, 64) == 0
    assert lib.armor_proxy_loss_full_h(None, None, None, None, None, 64, 64, 64, 32, None, None, 0, None) == 1
    assert lib.armor_proxy_loss_full_h(p, None, p, None, p, 63, 64, 64, 32, p, p, 1 << 30, None) == 2   # ldh < d_in
    assert lib.armor_proxy_loss_full_h(p, None, p, None, p, 66, 64, 64, 32, p, p, 1 << 30, None) == 2   # ldh not a multiple of 4
    assert lib.armor_proxy_loss_full_h(p, None, p, None, p, 64, 64, 64, 32, p, p, 16, None) == 4        # workspace too small
    # the allocation-free loss: argument errors and the fixed-scratch limit are host-side checks
    assert lib.armor_proxy_loss_noalloc(None, None, None, None, None, 0, 64, 64, 32, None, None) == 1
    assert lib.armor_proxy_loss_noalloc(p, None, p, None, p, 0, 64, 60, 32, p, None) == 2
    assert lib.armor_proxy_loss_noalloc(p, None, p, None, p, 0, 16384, 16384, 256, p, None) == 9   # 2 x 16 MiB of identities
    assert b"fixed scratch" in lib.armor_status_string(9)
    assert lib.armor_pack_nm(p, p, 4, 16, 2, 5, p, 0, p, None) == 2
    assert lib.armor_pack_meta_row_bytes(4096, 2, 4) == 512 and lib.armor_pack_meta_row_bytes(72, 5, 8) == 23
    assert lib.armor_pack_meta_row_bytes(70, 1, 2) == 5 and lib.armor_pack_meta_row_bytes(70, 2, 4) == 0
    # the apply entry point: workspace = one bf16 activation matrix; unsupported patterns / shapes say so
    assert lib.armor_apply_workspace_bytes(100, 64) >= 256 * 64 * 2               # tokens padded to 256
    assert lib.armor_apply_prepared_bytes(300, 128) == 2 * 512 * 72 and lib.armor_apply_prepared_bytes(300, 96) == 0
    assert lib.armor_apply_prepare(p, p, 64, 64, 4, 8, p, 1 << 20, None) == 7                     # only 2:4
    assert lib.armor_apply_prepare(p, p, 64, 64, 2, 4, p, 16, None) == 4                          # buffer too small
    assert lib.armor_apply_packed(None, 1, p, p, p, 64, 64, 32, 2, 4, p, p, 1 << 20, None) == 1
    assert lib.armor_apply_packed(p, 1, p, p, p, 64, 64, 32, 4, 8, p, p, 1 << 20, None) == 7      # only 2:4
    assert lib.armor_apply_packed(p, 1, p, p, p, 64, 96, 32, 2, 4, p, p, 1 << 20, None) == 7      # d_in % 64
    assert lib.armor_apply_packed(p, 1, p, p, p, 192, 192, 96, 2, 4, p, p, 1 << 20, None) == 2     # block size
    assert lib.armor_apply_packed(p, 1, p, p, p, 64, 64, 48, 2, 4, p, p, 1 << 20, None) == 2
    assert lib.armor_apply_packed(p, 4, p, p, p, 64, 64, 32, 2, 4, p, p, 16, None) == 4            # workspace too small


def test_product_package_does_not_import_the_oracle():
    """The product path must not route through the CPU oracle."""
    pkg = os.path.join(ROOT, "paper_2510_05528_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                src = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in src and "from oracle" not in src and "liboracle" not in src, f


def test_profiler_host_side():
    """Switching the per-kernel timing on and off and reading it with nothing recorded touch no device."""
    from paper_2510_05528_amd import binding
    lib = binding.load_library()
    assert lib.armor_profile_read(None, None) == 1
    assert lib.armor_profile_enable(0) == 0
    ms = (ctypes.c_double * len(binding.PROF_KINDS))(*([7.0] * len(binding.PROF_KINDS)))
    cnt = (ctypes.c_int64 * len(binding.PROF_KINDS))(*([7] * len(binding.PROF_KINDS)))
    assert lib.armor_profile_read(ms, cnt) == 0
    assert list(ms) == [0.0] * len(binding.PROF_KINDS) and list(cnt) == [0] * len(binding.PROF_KINDS)
