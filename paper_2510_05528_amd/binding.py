"""ctypes binding of libarmor.so.  Function names mirror the C entry points (armor_<name>)."""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libarmor.so")

ARMOR_F32, ARMOR_BF16 = 0, 1

PROF_KINDS = ["gram", "phase_A", "phase_B", "phase_WS", "sparse_step", "phase_FB", "phase_GS", "normalize", "init",
              "pack_nm", "small_kernels", "apply_pre", "apply_main", "gram_diag_x", "residual", "full_gram_loss"]

EXPORTED = ["armor_status_string", "armor_last_hip_error", "armor_last_iteration_count", "armor_profile_enable", "armor_profile_read",
            "armor_gram_workspace_bytes", "armor_gram", "armor_gram_diag",
            "armor_gram_diag_x_workspace_bytes", "armor_gram_diag_x",
            "armor_normalize_workspace_bytes", "armor_normalize", "armor_proxy_loss_workspace_bytes",
            "armor_proxy_loss", "armor_proxy_loss_noalloc", "armor_proxy_loss_full_h_workspace_bytes",
            "armor_proxy_loss_full_h", "armor_factorize_workspace_bytes", "armor_factorize_layer", "armor_pack_nm",
            "armor_pack_meta_row_bytes", "armor_to_bf16", "armor_apply_prepared_bytes", "armor_apply_prepare",
            "armor_apply_workspace_bytes", "armor_apply_packed"]


class ArmorError(RuntimeError):
    pass


class ArmorOpts(ctypes.Structure):
    _fields_ = [("selection", ctypes.c_int32), ("sparsity", ctypes.c_int32), ("unstructured_keep", ctypes.c_int64),
                ("seed", ctypes.c_uint64), ("denormalize", ctypes.c_int32), ("variant", ctypes.c_int32),
                ("lr", ctypes.c_double), ("adam_beta1", ctypes.c_double), ("adam_beta2", ctypes.c_double),
                ("adam_eps", ctypes.c_double), ("init_from_outputs", ctypes.c_int32), ("check_finite", ctypes.c_int32),
                ("iter_offset", ctypes.c_int64), ("tol", ctypes.c_double)]


_lib = None
_vp, _i64, _int, _sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_size_t


def load_library():
    """Load libarmor.so (built by __graft_entry__.build()).  Raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ArmorError("libarmor.so is not built (%s); run __graft_entry__.build()" % _LIB_PATH)
    lib = ctypes.CDLL(_LIB_PATH)
    lib.armor_status_string.restype = ctypes.c_char_p
    lib.armor_status_string.argtypes = [_int]
    lib.armor_last_hip_error.restype = _int
    lib.armor_last_iteration_count.restype = _i64
    lib.armor_profile_enable.argtypes = [_int]
    lib.armor_profile_read.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int64)]
    lib.armor_gram_workspace_bytes.restype = _sz
    lib.armor_gram_workspace_bytes.argtypes = [_i64, _i64, _int]
    lib.armor_gram.argtypes = [_vp, _int, _i64, _i64, _i64, _vp, _i64, _int, _vp, _sz, _vp]
    lib.armor_gram_diag.argtypes = [_vp, _i64, _i64, _vp, _vp]
    lib.armor_gram_diag_x_workspace_bytes.restype = _sz
    lib.armor_gram_diag_x_workspace_bytes.argtypes = [_i64, _i64]
    lib.armor_gram_diag_x.argtypes = [_vp, _int, _i64, _i64, _i64, _vp, _int, _vp, _sz, _vp]
    lib.armor_normalize_workspace_bytes.restype = _sz
    lib.armor_normalize_workspace_bytes.argtypes = [_i64, _i64]
    lib.armor_normalize.argtypes = [_vp, _int, _i64, _i64, _vp, _vp, _vp, _vp, _sz, _vp]
    lib.armor_proxy_loss_workspace_bytes.restype = _sz
    lib.armor_proxy_loss_workspace_bytes.argtypes = [_i64, _i64, _i64]
    lib.armor_proxy_loss.argtypes = [_vp, _vp, _vp, _vp, _vp, _i64, _i64, _i64, _i64, _vp, _vp, _sz, _vp]
    lib.armor_proxy_loss_noalloc.argtypes = [_vp, _vp, _vp, _vp, _vp, _i64, _i64, _i64, _i64, _vp, _vp]
    lib.armor_proxy_loss_full_h_workspace_bytes.restype = _sz
    lib.armor_proxy_loss_full_h_workspace_bytes.argtypes = [_i64, _i64, _i64]
    lib.armor_proxy_loss_full_h.argtypes = [_vp, _vp, _vp, _vp, _vp, _i64, _i64, _i64, _i64, _vp, _vp, _sz, _vp]
    lib.armor_factorize_workspace_bytes.restype = _sz
    lib.armor_factorize_workspace_bytes.argtypes = [_i64, _i64, _i64, _int, _int, ctypes.POINTER(ArmorOpts)]
    lib.armor_factorize_layer.argtypes = [_vp, _int, _vp, _i64, _i64, _i64, _i64, _int, _int, _int,
                                          ctypes.POINTER(ArmorOpts), _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp,
                                          _vp, _sz, _vp]
    lib.armor_pack_meta_row_bytes.argtypes = [_i64, _int, _int]
    lib.armor_pack_meta_row_bytes.restype = _i64
    lib.armor_pack_nm.argtypes = [_vp, _vp, _i64, _i64, _int, _int, _vp, _int, _vp, _vp]
    lib.armor_to_bf16.argtypes = [_vp, _i64, _vp, _vp]
    lib.armor_apply_workspace_bytes.restype = _sz
    lib.armor_apply_workspace_bytes.argtypes = [_i64, _i64]
    lib.armor_apply_prepared_bytes.restype = _sz
    lib.armor_apply_prepared_bytes.argtypes = [_i64, _i64]
    lib.armor_apply_prepare.argtypes = [_vp, _vp, _i64, _i64, _int, _int, _vp, _sz, _vp]
    lib.armor_apply_packed.argtypes = [_vp, _i64, _vp, _vp, _vp, _i64, _i64, _i64, _int, _int, _vp, _vp, _sz, _vp]
    _lib = lib
    return lib


def _check(status):
    if status != 0:
        lib = load_library()
        msg = lib.armor_status_string(status).decode()
        if status == 6:
            msg += " (hipError %d)" % lib.armor_last_hip_error()
        raise ArmorError("armor status %d: %s" % (status, msg))


def _torch():
    import torch
    return torch


def _stream():
    return _vp(_torch().cuda.current_stream().cuda_stream)


def _ptr(t):
    return _vp(t.data_ptr()) if t is not None else _vp(0)


def _dtype_code(t):
    torch = _torch()
    if t.dtype == torch.float32:
        return ARMOR_F32
    if t.dtype == torch.bfloat16:
        return ARMOR_BF16
    raise ArmorError("unsupported dtype %s" % t.dtype)


def _dev_f32(t, name):
    torch = _torch()
    if not (t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()):
        raise ArmorError("%s must be a contiguous fp32 device tensor" % name)
    return t


def profile_enable(on=True):
    _check(load_library().armor_profile_enable(int(on)))


def profile_read():
    """{kind: (total_ms, launches)} since the last read; waits for the recorded events."""
    ms = (ctypes.c_double * len(PROF_KINDS))()
    cnt = (ctypes.c_int64 * len(PROF_KINDS))()
    _check(load_library().armor_profile_read(ms, cnt))
    return {k: (ms[i], cnt[i]) for i, k in enumerate(PROF_KINDS)}


def gram_workspace_bytes(n_tokens, d_in, bf16=True):
    return load_library().armor_gram_workspace_bytes(n_tokens, d_in, ARMOR_BF16 if bf16 else ARMOR_F32)


def gram(X, H=None, accumulate=False, ws=None):
    """H (+)= X^T X.  X [n_tokens, d_in] fp32/bf16 on the device; returns H [d_in, d_in] fp32.
    ws: optional uint8 device tensor of gram_workspace_bytes() bytes (allocated here if None)."""
    torch = _torch()
    lib = load_library()
    if not (X.is_cuda and X.dim() == 2 and X.stride(1) == 1):
        raise ArmorError("X must be a 2-D device tensor with unit column stride")
    n, d_in = X.shape
    if H is None:
        if accumulate:
            raise ArmorError("accumulate needs an existing H")
        H = torch.empty((d_in, d_in), device=X.device, dtype=torch.float32)
    _dev_f32(H, "H")
    need = lib.armor_gram_workspace_bytes(n, d_in, _dtype_code(X))
    if need > 0 and (ws is None or ws.numel() < need):
        ws = torch.empty(need, device=X.device, dtype=torch.uint8)
    _check(lib.armor_gram(_ptr(X), _dtype_code(X), n, d_in, X.stride(0), _ptr(H), H.stride(0), int(accumulate),
                          _ptr(ws) if need > 0 else _vp(0), ws.numel() if need > 0 else 0, _stream()))
    return H


def gram_diag(H):
    torch = _torch()
    lib = load_library()
    _dev_f32(H, "H")
    D = torch.empty(H.shape[0], device=H.device, dtype=torch.float32)
    _check(lib.armor_gram_diag(_ptr(H), H.shape[0], H.stride(0), _ptr(D), _stream()))
    return D


def gram_diag_x(X, D=None, accumulate=False, ws=None):
    """D[j] (+)= sum_t X[t][j]^2 straight from the activations (armor_gram_diag_x)."""
    torch = _torch()
    lib = load_library()
    if not (X.is_cuda and X.dim() == 2 and (X.numel() == 0 or X.stride(1) == 1)):
        raise ArmorError("X must be a 2-D device tensor with unit column stride")
    n, d_in = X.shape
    if D is None:
        D = torch.zeros(d_in, device=X.device, dtype=torch.float32)
    if ws is None:
        ws = torch.empty(int(lib.armor_gram_diag_x_workspace_bytes(n, d_in)), device=X.device, dtype=torch.uint8)
    _check(lib.armor_gram_diag_x(_ptr(X), _dtype_code(X), n, d_in, X.stride(0) if n > 0 else d_in, _ptr(D), 1 if accumulate else 0, _ptr(ws),
                                 ws.numel(), _stream()))
    return D


def normalize(W):
    """Returns (Wbar, r1, r2) of the row/column normalisation."""
    torch = _torch()
    lib = load_library()
    if not (W.is_cuda and W.is_contiguous()):
        raise ArmorError("W must be a contiguous device tensor")
    d_out, d_in = W.shape
    Wbar = torch.empty((d_out, d_in), device=W.device, dtype=torch.float32)
    r1 = torch.empty(d_in, device=W.device, dtype=torch.float32)
    r2 = torch.empty(d_out, device=W.device, dtype=torch.float32)
    nbytes = lib.armor_normalize_workspace_bytes(d_out, d_in)
    ws = torch.empty(nbytes, device=W.device, dtype=torch.uint8)
    _check(lib.armor_normalize(_ptr(W), _dtype_code(W), d_out, d_in, _ptr(Wbar), _ptr(r1), _ptr(r2), _ptr(ws), nbytes,
                               _stream()))
    return Wbar, r1, r2


def _h_args(H, d_in):
    """H is either the Gram matrix [d_in, d_in] or the vector D [d_in]."""
    _dev_f32(H, "H")
    if H.dim() == 2:
        return H.stride(0)
    if H.dim() == 1 and H.shape[0] == d_in:
        return 0
    raise ArmorError("H must be [d_in, d_in] or [d_in]")


def proxy_loss(Wbar, A, S, B, H, d_block=None):
    """Proxy loss as a 1-element float64 device tensor.  A or B may be None (identity)."""
    torch = _torch()
    lib = load_library()
    _dev_f32(Wbar, "Wbar"), _dev_f32(S, "S")
    d_out, d_in = Wbar.shape
    b = d_block or (A.shape[-1] if A is not None else B.shape[-1])
    ldh = _h_args(H, d_in)
    out = torch.zeros(1, device=Wbar.device, dtype=torch.float64)
    nbytes = lib.armor_proxy_loss_workspace_bytes(d_out, d_in, b)
    ws = torch.empty(max(nbytes, 256), device=Wbar.device, dtype=torch.uint8)
    _check(lib.armor_proxy_loss(_ptr(Wbar), _ptr(A), _ptr(S), _ptr(B), _ptr(H), ldh, d_out, d_in, b, _ptr(out), _ptr(ws),
                                nbytes, _stream()))
    return out


def proxy_loss_noalloc(Wbar, A, S, B, H, d_block=None, out=None):
    """armor_proxy_loss_noalloc: the proxy loss with the library's own fixed scratch.  `out`: an existing
    1-element float64 device tensor (so that the call itself allocates nothing); created if None."""
    torch = _torch()
    lib = load_library()
    _dev_f32(Wbar, "Wbar"), _dev_f32(S, "S")
    d_out, d_in = Wbar.shape
    b = d_block or (A.shape[-1] if A is not None else B.shape[-1])
    ldh = _h_args(H, d_in)
    if out is None:
        out = torch.zeros(1, device=Wbar.device, dtype=torch.float64)
    _check(lib.armor_proxy_loss_noalloc(_ptr(Wbar), _ptr(A), _ptr(S), _ptr(B), _ptr(H), ldh, d_out, d_in, b, _ptr(out),
                                        _stream()))
    return out


def proxy_loss_full_h(Wbar, A, S, B, H, d_block=None, ws=None):
    """armor_proxy_loss_full_h: tr(R H R^T) with R = Wbar - A S B and the whole Gram matrix H [d_in, d_in]
    (row stride a multiple of 4), as a 1-element float64 device tensor.  A or B may be None (identity)."""
    torch = _torch()
    lib = load_library()
    _dev_f32(Wbar, "Wbar"), _dev_f32(S, "S")
    d_out, d_in = Wbar.shape
    b = d_block or (A.shape[-1] if A is not None else B.shape[-1])
    if not (H.is_cuda and H.dtype == torch.float32 and H.dim() == 2 and H.shape == (d_in, d_in) and H.stride(1) == 1):
        raise ArmorError("H must be a [d_in, d_in] fp32 device tensor with unit column stride")
    out = torch.zeros(1, device=Wbar.device, dtype=torch.float64)
    nbytes = lib.armor_proxy_loss_full_h_workspace_bytes(d_out, d_in, b)
    if ws is None:
        ws = torch.empty(max(nbytes, 256), device=Wbar.device, dtype=torch.uint8)
    _check(lib.armor_proxy_loss_full_h(_ptr(Wbar), _ptr(A), _ptr(S), _ptr(B), _ptr(H), H.stride(0), d_out, d_in, b,
                                       _ptr(out), _ptr(ws), ws.numel(), _stream()))
    return out


def factorize_workspace_bytes(d_out, d_in, d_block, N, M, sparsity=0, variant=0):
    lib = load_library()
    o = ArmorOpts(sparsity=sparsity, variant=variant)
    return lib.armor_factorize_workspace_bytes(d_out, d_in, d_block, N, M, ctypes.byref(o))


def factorize_layer(W, H, d_block, N, M, n_iters, seed=0, selection=0, sparsity=0, unstructured_keep=0,
                    denormalize=False, ws=None, want_cont_trace=False, variant=0, lr=0.0, adam_beta1=0.0,
                    adam_beta2=0.0, adam_eps=0.0, init=None, iter_offset=0, check_finite=False, want_diagnostics=False,
                    tol=0.0):
    """Run the BCD loop.  Returns dict(A, S, B, mask_bits, r1, r2, loss_trace, iters_done[, loss_cont_trace]
    [, eta_trace, mask_changes]).  init: optional dict(A, S, B, mask_bits) of device tensors to start from (they
    are copied; the copies are updated and returned) instead of the initialisation of Eq. 3.  tol > 0: the
    tolerance of Alg. 1 (the loop ends after the first iteration whose loss decrease is <= tol * L_0); the
    traces are then cut to the iterations that ran."""
    torch = _torch()
    lib = load_library()
    if not (W.is_cuda and W.is_contiguous()):
        raise ArmorError("W must be a contiguous device tensor")
    d_out, d_in = W.shape
    ldh = _h_args(H, d_in)
    dev = W.device
    o = ArmorOpts(selection=selection, sparsity=sparsity, unstructured_keep=unstructured_keep, seed=seed,
                  denormalize=int(denormalize), variant=variant, lr=lr, adam_beta1=adam_beta1, adam_beta2=adam_beta2,
                  adam_eps=adam_eps, init_from_outputs=0 if init is None else 1, check_finite=int(check_finite),
                  iter_offset=iter_offset, tol=tol)
    nbytes = lib.armor_factorize_workspace_bytes(d_out, d_in, d_block, N, M, ctypes.byref(o))
    if nbytes == 0:
        _check(2)
    if ws is None or ws.numel() < nbytes:
        ws = torch.empty(nbytes, device=dev, dtype=torch.uint8)
    mg = 8 if sparsity == 1 else M
    shapes = dict(A=(d_out // d_block, d_block, d_block), B=(d_in // d_block, d_block, d_block), S=(d_out, d_in),
                  mask_bits=(d_out, d_in // mg))
    if init is None:
        A, B, S = (torch.empty(shapes[k], device=dev, dtype=torch.float32) for k in ("A", "B", "S"))
        mask_bits = torch.empty(shapes["mask_bits"], device=dev, dtype=torch.uint8)
    else:
        for k, shp in shapes.items():
            t = init[k]
            want = torch.uint8 if k == "mask_bits" else torch.float32
            if not (t.is_cuda and t.dtype == want and tuple(t.shape) == shp):
                raise ArmorError("init[%r] must be a %s device tensor of shape %s" % (k, want, shp))
        A, B, S, mask_bits = (init[k].contiguous().clone() for k in ("A", "B", "S", "mask_bits"))
    r1 = torch.empty(d_in, device=dev, dtype=torch.float32)
    r2 = torch.empty(d_out, device=dev, dtype=torch.float32)
    trace = torch.zeros(n_iters + 1, device=dev, dtype=torch.float64)
    ctrace = torch.zeros(max(n_iters, 1), device=dev, dtype=torch.float64) if want_cont_trace else None
    etas = torch.zeros((max(n_iters, 1), 3), device=dev, dtype=torch.float64) if want_diagnostics else None
    changes = torch.zeros(max(n_iters, 1), device=dev, dtype=torch.int32) if want_diagnostics else None
    _check(lib.armor_factorize_layer(_ptr(W), _dtype_code(W), _ptr(H), ldh, d_out, d_in, d_block, N, M, n_iters,
                                     ctypes.byref(o), _ptr(A), _ptr(S), _ptr(B), _ptr(mask_bits), _ptr(r1), _ptr(r2),
                                     _ptr(trace), _ptr(ctrace), _ptr(etas), _ptr(changes), _ptr(ws), ws.numel(),
                                     _stream()))
    done = int(lib.armor_last_iteration_count())
    out = dict(A=A, S=S, B=B, mask_bits=mask_bits, r1=r1, r2=r2, loss_trace=trace[:done + 1], ws=ws, iters_done=done)
    if want_cont_trace:
        out["loss_cont_trace"] = ctrace[:done]
    if want_diagnostics:
        out["eta_trace"] = etas[:done]
        out["mask_changes"] = changes[:done]
    return out


def pack_mask(mask, M):
    """Host helper: [d_out, d_in] 0/1 array -> [d_out, d_in/M] bytes (bit p = column p of the group kept)."""
    m = np.asarray(mask, dtype=np.uint8)
    g = m.reshape(m.shape[0], m.shape[1] // M, M).astype(np.uint32)
    return (g << np.arange(M, dtype=np.uint32)).sum(-1).astype(np.uint8)


def pack_nm(S, mask_bits, N, M, bf16=False):
    torch = _torch()
    lib = load_library()
    _dev_f32(S, "S")
    d_out, d_in = S.shape
    values = torch.empty((d_out, d_in // M * N), device=S.device, dtype=torch.bfloat16 if bf16 else torch.float32)
    meta_row = int(lib.armor_pack_meta_row_bytes(d_in, N, M))
    if meta_row <= 0:
        raise ArmorError("armor_pack_nm: bad shape")
    meta = torch.empty((d_out, meta_row), device=S.device, dtype=torch.uint8)
    _check(lib.armor_pack_nm(_ptr(S), _ptr(mask_bits), d_out, d_in, N, M, _ptr(values), ARMOR_BF16 if bf16 else ARMOR_F32,
                             _ptr(meta), _stream()))
    return values, meta


def to_bf16(t):
    """fp32 device tensor -> bf16 device tensor of the same shape (armor_to_bf16)."""
    torch = _torch()
    lib = load_library()
    _dev_f32(t, "t")
    out = torch.empty(t.shape, device=t.device, dtype=torch.bfloat16)
    _check(lib.armor_to_bf16(_ptr(t), t.numel(), _ptr(out), _stream()))
    return out


def apply_workspace_bytes(n_tokens, d_in):
    return int(load_library().armor_apply_workspace_bytes(n_tokens, d_in))


def apply_prepare(values, meta, N, M):
    """Compressed core (armor_pack_nm, bf16 values) -> the streaming layout armor_apply_packed takes."""
    torch = _torch()
    lib = load_library()
    if not (values.is_cuda and values.dtype == torch.bfloat16 and values.is_contiguous()):
        raise ArmorError("values must be a contiguous bf16 device tensor")
    if not (meta.is_cuda and meta.dtype == torch.uint8 and meta.is_contiguous()):
        raise ArmorError("meta must be a contiguous uint8 device tensor")
    d_out, d_in = values.shape[0], values.shape[1] * M // N
    nbytes = int(lib.armor_apply_prepared_bytes(d_out, d_in))
    prepared = torch.empty(max(nbytes, 16), device=values.device, dtype=torch.uint8)
    _check(lib.armor_apply_prepare(_ptr(values), _ptr(meta), d_out, d_in, N, M, _ptr(prepared), prepared.numel(), _stream()))
    return prepared


def apply_packed(X, A_bf16, prepared, B_bf16, N, M, Y=None, ws=None):
    """Y[t] = A (S (B X[t])) from the prepared core (armor_apply_packed). X [n, d_in] bf16 -> Y [n, d_out] bf16."""
    torch = _torch()
    lib = load_library()
    for name, t in (("X", X), ("A_bf16", A_bf16), ("B_bf16", B_bf16)):
        if not (t.is_cuda and t.dtype == torch.bfloat16 and t.is_contiguous()):
            raise ArmorError("%s must be a contiguous bf16 device tensor" % name)
    if not (prepared.is_cuda and prepared.dtype == torch.uint8 and prepared.is_contiguous()):
        raise ArmorError("prepared must be a contiguous uint8 device tensor")
    n, d_in = X.shape
    b = A_bf16.shape[-1]
    d_out = A_bf16.shape[0] * b
    if Y is None:
        Y = torch.empty((n, d_out), device=X.device, dtype=torch.bfloat16)
    if ws is None:
        ws = torch.empty(max(apply_workspace_bytes(n, d_in), 16), device=X.device, dtype=torch.uint8)
    _check(lib.armor_apply_packed(_ptr(X), n, _ptr(A_bf16), _ptr(prepared), _ptr(B_bf16), d_out, d_in, b, N, M,
                                  _ptr(Y), _ptr(ws), ws.numel(), _stream()))
    return Y


def unpack_meta(meta, d_in, N, M):
    """Host helper: bit-packed in-group column indices -> [d_out, d_in/M*N] bytes."""
    mb = np.asarray(meta, dtype=np.uint8)
    w = {2: 1, 4: 2, 8: 4}[M]
    per = 8 // w
    fields = (mb[..., None] >> (np.arange(per, dtype=np.uint8) * w)) & ((1 << w) - 1)
    return fields.reshape(mb.shape[0], -1)[:, :d_in // M * N].astype(np.uint8)


def unpack_mask(mask_bits, M):
    """Host helper: [d_out, d_in/M] bytes -> [d_out, d_in] 0/1 array."""
    mb = np.asarray(mask_bits, dtype=np.uint8)
    bits = (mb[..., None] >> np.arange(M, dtype=np.uint8)) & 1
    return bits.reshape(mb.shape[0], mb.shape[1] * M).astype(np.uint8)
