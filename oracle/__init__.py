"""ctypes front-end of the CPU oracle (``armor_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the CPU-baseline leg
of the benchmark.  The product package never imports this module.  It only marshals numpy
arrays; every piece of arithmetic lives in the C file, which cites the paper passage it follows.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "armor_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

_f32p = ctypes.POINTER(ctypes.c_float)
_f64p = ctypes.POINTER(ctypes.c_double)
_u8p = ctypes.POINTER(ctypes.c_uint8)
_u16p = ctypes.POINTER(ctypes.c_uint16)
_i32p = ctypes.POINTER(ctypes.c_int32)
_i64p = ctypes.POINTER(ctypes.c_int64)
_i64 = ctypes.c_int64


def build(force=False):
    """Compile the oracle with gcc -O2 (+OpenMP).  Building the checker is not using it."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB):
            build()
        _lib = ctypes.CDLL(_LIB)
        _lib.oracle_proxy_loss.restype = ctypes.c_double
        _lib.oracle_uniform.restype = ctypes.c_float
        _lib.oracle_uniform.argtypes = [ctypes.c_uint64, _i64, _i64, _i64, _i64, _i64]
    return _lib


def set_threads(n):
    """Number of OpenMP threads the oracle's parallel loops use from now on."""
    ctypes.CDLL("libgomp.so.1").omp_set_num_threads(int(n))


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def _p(a, typ):
    return a.ctypes.data_as(typ) if a is not None else None


def uniform(seed, t, n_blocks, blk, groups_per_block, kappa):
    return float(lib().oracle_uniform(seed, t, n_blocks, blk, groups_per_block, kappa))


def gram(X):
    X = _f32(X)
    n, d = X.shape
    H = np.empty((d, d), dtype=np.float64)
    lib().oracle_gram(_p(X, _f32p), _i64(n), _i64(d), _p(H, _f64p))
    return H


def gram_entries(X, rows, cols):
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    cols = np.ascontiguousarray(cols, dtype=np.int64)
    out = np.empty(rows.shape[0], dtype=np.float64)
    n, d = X.shape
    if X.dtype == np.uint16:  # raw bf16 bit patterns
        X = np.ascontiguousarray(X)
        lib().oracle_gram_entries_bf16(_p(X, _u16p), _i64(n), _i64(d), _p(rows, _i64p), _p(cols, _i64p),
                                       _i64(rows.shape[0]), _p(out, _f64p))
    else:
        X = _f32(X)
        lib().oracle_gram_entries(_p(X, _f32p), _i64(n), _i64(d), _p(rows, _i64p), _p(cols, _i64p),
                                  _i64(rows.shape[0]), _p(out, _f64p))
    return out


def normalize(W):
    W = _f32(W)
    d_out, d_in = W.shape
    Wbar = np.empty_like(W)
    r1 = np.empty(d_in, dtype=np.float32)
    r2 = np.empty(d_out, dtype=np.float32)
    lib().oracle_normalize(_p(W, _f32p), _i64(d_out), _i64(d_in), _p(Wbar, _f32p), _p(r1, _f32p), _p(r2, _f32p))
    return Wbar, r1, r2


def init_nm(Wbar, D, N, M):
    Wbar, D = _f32(Wbar), _f32(D)
    d_out, d_in = Wbar.shape
    C = np.empty_like(Wbar)
    mask = np.empty((d_out, d_in), dtype=np.uint8)
    lib().oracle_init_nm(_p(Wbar, _f32p), _p(D, _f32p), _i64(d_out), _i64(d_in), ctypes.c_int(N),
                         ctypes.c_int(M), _p(C, _f32p), _p(mask, _u8p))
    return C, mask


def init_unstructured(Wbar, D, keep):
    Wbar, D = _f32(Wbar), _f32(D)
    d_out, d_in = Wbar.shape
    C = np.empty_like(Wbar)
    mask = np.empty((d_out, d_in), dtype=np.uint8)
    lib().oracle_init_unstructured(_p(Wbar, _f32p), _p(D, _f32p), _i64(d_out), _i64(d_in), _i64(keep),
                                   _p(C, _f32p), _p(mask, _u8p))
    return C, mask


def identity_blocks(n, b):
    return np.tile(np.eye(b, dtype=np.float32), (n, 1, 1))


def proxy_loss(Wbar, A, C, B, D):
    Wbar, A, C, B, D = _f32(Wbar), _f32(A), _f32(C), _f32(B), _f32(D)
    d_out, d_in = Wbar.shape
    b = A.shape[-1]
    return float(lib().oracle_proxy_loss(_p(Wbar, _f32p), _p(A, _f32p), _p(C, _f32p), _p(B, _f32p),
                                         _p(D, _f32p), _i64(d_out), _i64(d_in), _i64(b)))


def reconstruct(A, C, B):
    A, C, B = _f32(A), _f32(C), _f32(B)
    d_out, d_in = C.shape
    b = A.shape[-1]
    out = np.empty((d_out, d_in), dtype=np.float64)
    lib().oracle_reconstruct(_p(A, _f32p), _p(C, _f32p), _p(B, _f32p), _i64(d_out), _i64(d_in), _i64(b),
                             _p(out, _f64p))
    return out


def factor_sizes(d_out, d_in, b, N=2, M=4):
    """Entry counts of the factorized layer (Sec. 3.1): the wrappers are stored as (d_out/b) x b x b and
    (d_in/b) x b x b tensors, the core keeps N of every M entries of a d_out x d_in matrix.  One multiply-add per
    stored entry and token, so the same counts give the work of y = A (S (B x)) (Sec. 4.4)."""
    assert d_out % b == 0 and d_in % b == 0 and d_in % M == 0
    return dict(wrappers=(d_out // b) * b * b + (d_in // b) * b * b, core=d_out * (d_in // M) * N, dense=d_out * d_in)


def proxy_loss_full_h(Wbar, A, C, B, H):
    """The layer-wise objective against the whole Gram matrix H = X^T X (Sec. 2; Eq. 2 keeps only its
    diagonal):  tr(R H R^T) = ||R X^T||_F^2  with R = Wbar - A C B.  The definition written out in fp64."""
    R = np.asarray(_f32(Wbar), dtype=np.float64) - reconstruct(A, C, B)
    H = np.asarray(H, dtype=np.float64)
    assert H.shape == (R.shape[1], R.shape[1])
    return float(np.sum((R @ H) * R))


def _grad(fn, Wbar, A, C, B, D, shape):
    Wbar, A, C, B, D = _f32(Wbar), _f32(A), _f32(C), _f32(B), _f32(D)
    d_out, d_in = Wbar.shape
    b = A.shape[-1]
    g = np.empty(shape, dtype=np.float64)
    beta = ctypes.c_double(0.0)
    fn(_p(Wbar, _f32p), _p(A, _f32p), _p(C, _f32p), _p(B, _f32p), _p(D, _f32p), _i64(d_out), _i64(d_in),
       _i64(b), _p(g, _f64p), ctypes.byref(beta))
    return g, beta.value


def grad_A(Wbar, A, C, B, D):
    """(grad_A [d_out/b, b, b], beta_A)"""
    return _grad(lib().oracle_grad_A, Wbar, A, C, B, D, np.asarray(A).shape)


def grad_B(Wbar, A, C, B, D):
    """(grad_B [d_in/b, b, b], beta_B)"""
    return _grad(lib().oracle_grad_B, Wbar, A, C, B, D, np.asarray(B).shape)


def grad_core(Wbar, A, C, B, D):
    """(unmasked core gradient [d_out, d_in], beta_W')"""
    return _grad(lib().oracle_grad_core, Wbar, A, C, B, D, np.asarray(Wbar).shape)


def continuous_update(Wbar, D, mask, A, C, B):
    """One pass of the sequential-GD continuous step; returns new (A, C, B, etas[3])."""
    Wbar, D = _f32(Wbar), _f32(D)
    A, C, B = _f32(A).copy(), _f32(C).copy(), _f32(B).copy()
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    d_out, d_in = Wbar.shape
    b = A.shape[-1]
    etas = np.zeros(3, dtype=np.float64)
    lib().oracle_continuous_update(_p(Wbar, _f32p), _p(D, _f32p), _p(mask, _u8p), _i64(d_out), _i64(d_in),
                                   _i64(b), _p(A, _f32p), _p(C, _f32p), _p(B, _f32p), _p(etas, _f64p))
    return A, C, B, etas


def sparse_core_update(Wbar, A, B, D, C, mask, N, M, seed, t, selection=0):
    """One sparse-core step; returns new (C, mask, chosen_kappa[n_blocks], chosen_pattern[n_blocks])."""
    Wbar, A, B, D = _f32(Wbar), _f32(A), _f32(B), _f32(D)
    C = _f32(C).copy()
    mask = np.ascontiguousarray(mask, dtype=np.uint8).copy()
    d_out, d_in = Wbar.shape
    b = A.shape[-1]
    nblk = (d_out // b) * (d_in // b)
    kap = np.zeros(nblk, dtype=np.int32)
    pat = np.zeros(nblk, dtype=np.int32)
    lib().oracle_sparse_core_update(_p(Wbar, _f32p), _p(A, _f32p), _p(B, _f32p), _p(D, _f32p), _i64(d_out),
                                    _i64(d_in), _i64(b), ctypes.c_int(N), ctypes.c_int(M),
                                    ctypes.c_uint64(seed), _i64(t), ctypes.c_int(selection), _p(C, _f32p),
                                    _p(mask, _u8p), _p(kap, _i32p), _p(pat, _i32p))
    return C, mask, kap, pat


def _start_state(init, d_out, d_in, b):
    """Output buffers of the outer loop, pre-filled with the caller's starting point when one is given."""
    if init is None:
        A = np.empty((d_out // b, b, b), dtype=np.float32)
        B = np.empty((d_in // b, b, b), dtype=np.float32)
        C = np.empty((d_out, d_in), dtype=np.float32)
        mask = np.empty((d_out, d_in), dtype=np.uint8)
    else:
        A, B, C = _f32(init["A"]).copy(), _f32(init["B"]).copy(), _f32(init["C"]).copy()
        mask = np.ascontiguousarray(init["mask"], dtype=np.uint8).copy()
        assert A.shape == (d_out // b, b, b) and B.shape == (d_in // b, b, b)
        assert C.shape == (d_out, d_in) and mask.shape == (d_out, d_in)
    return A, B, C, mask


def factorize_layer(W, D, b, N, M, n_iters, seed=0, selection=0, sparsity=0, keep=0, init=None, iter_offset=0, tol=0.0):
    """Whole outer loop.  Returns a dict with A, C (=S), B, mask, Wbar, r1, r2, loss_trace, loss_cont_trace,
    etas [n_iters, 3] (eta_A, eta_B, eta_W' of each iteration), mask_changes [n_iters] and iters_done.
    init: optional dict(A, C, B, mask) to start from instead of Eq. 3; iter_offset: iterations already done.
    tol: the tolerance input of Alg. 1 (stop after the first iteration t with L_{t-1} - L_t <= tol * L_0; 0 = never);
    the traces are cut to the iterations that ran."""
    W, D = _f32(W), _f32(D)
    d_out, d_in = W.shape
    A, B, C, mask = _start_state(init, d_out, d_in, b)
    Wbar = np.empty((d_out, d_in), dtype=np.float32)
    r1 = np.empty(d_in, dtype=np.float32)
    r2 = np.empty(d_out, dtype=np.float32)
    trace = np.zeros(n_iters + 1, dtype=np.float64)
    ctrace = np.zeros(max(n_iters, 1), dtype=np.float64)
    etas = np.zeros((max(n_iters, 1), 3), dtype=np.float64)
    changes = np.zeros(max(n_iters, 1), dtype=np.int64)
    done = ctypes.c_int(0)
    lib().oracle_factorize_layer_ex(_p(W, _f32p), _p(D, _f32p), _i64(d_out), _i64(d_in), _i64(b), ctypes.c_int(N),
                                    ctypes.c_int(M), ctypes.c_int(n_iters), ctypes.c_uint64(seed),
                                    ctypes.c_int(selection), ctypes.c_int(sparsity), _i64(keep),
                                    ctypes.c_int(0 if init is None else 1), _i64(iter_offset), _p(A, _f32p),
                                    _p(C, _f32p), _p(B, _f32p), _p(mask, _u8p), _p(Wbar, _f32p), _p(r1, _f32p),
                                    _p(r2, _f32p), _p(trace, _f64p), _p(ctrace, _f64p), _p(etas, _f64p),
                                    _p(changes, _i64p), ctypes.c_double(tol), ctypes.byref(done))
    n = done.value
    return dict(A=A, C=C, B=B, mask=mask, Wbar=Wbar, r1=r1, r2=r2, loss_trace=trace[:n + 1],
                loss_cont_trace=ctrace[:n], etas=etas[:n], mask_changes=changes[:n], iters_done=n)


def adam_update(Wbar, D, mask, A, C, B, state, t, lr=1e-4, b1=0.9, b2=0.999, eps=1e-8):
    """One joint Adam step at iteration t (1-based).  state: dict of mA, vA, mB, vB, mC, vC (fp32 arrays,
    updated in place on copies).  Returns new (A, C, B, state)."""
    Wbar, D = _f32(Wbar), _f32(D)
    A, C, B = _f32(A).copy(), _f32(C).copy(), _f32(B).copy()
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    st = {k: _f32(v).copy() for k, v in state.items()}
    d_out, d_in = Wbar.shape
    b = A.shape[-1]
    lib().oracle_adam_update(_p(Wbar, _f32p), _p(D, _f32p), _p(mask, _u8p), _i64(d_out), _i64(d_in), _i64(b),
                             _p(A, _f32p), _p(C, _f32p), _p(B, _f32p), _p(st["mA"], _f32p), _p(st["vA"], _f32p),
                             _p(st["mB"], _f32p), _p(st["vB"], _f32p), _p(st["mC"], _f32p), _p(st["vC"], _f32p),
                             ctypes.c_double(lr), ctypes.c_double(b1), ctypes.c_double(b2), ctypes.c_double(eps),
                             _i64(t))
    return A, C, B, st


def adam_state(d_out, d_in, b):
    z = lambda *shape: np.zeros(shape, dtype=np.float32)
    return dict(mA=z(d_out // b, b, b), vA=z(d_out // b, b, b), mB=z(d_in // b, b, b), vB=z(d_in // b, b, b),
                mC=z(d_out, d_in), vC=z(d_out, d_in))


def factorize_layer_adam(W, D, b, N, M, n_iters, seed=0, selection=0, sparsity=0, keep=0, lr=1e-4, b1=0.9, b2=0.999,
                         eps=1e-8, init=None, iter_offset=0):
    """Outer loop with the joint Adam continuous step; same outputs as factorize_layer (no etas)."""
    W, D = _f32(W), _f32(D)
    d_out, d_in = W.shape
    A, B, C, mask = _start_state(init, d_out, d_in, b)
    Wbar = np.empty((d_out, d_in), dtype=np.float32)
    r1 = np.empty(d_in, dtype=np.float32)
    r2 = np.empty(d_out, dtype=np.float32)
    trace = np.zeros(n_iters + 1, dtype=np.float64)
    ctrace = np.zeros(max(n_iters, 1), dtype=np.float64)
    changes = np.zeros(max(n_iters, 1), dtype=np.int64)
    lib().oracle_factorize_layer_adam_ex(_p(W, _f32p), _p(D, _f32p), _i64(d_out), _i64(d_in), _i64(b),
                                         ctypes.c_int(N), ctypes.c_int(M), ctypes.c_int(n_iters),
                                         ctypes.c_uint64(seed), ctypes.c_int(selection), ctypes.c_int(sparsity),
                                         _i64(keep), ctypes.c_double(lr), ctypes.c_double(b1), ctypes.c_double(b2),
                                         ctypes.c_double(eps), ctypes.c_int(0 if init is None else 1),
                                         _i64(iter_offset), _p(A, _f32p), _p(C, _f32p), _p(B, _f32p),
                                         _p(mask, _u8p), _p(Wbar, _f32p), _p(r1, _f32p), _p(r2, _f32p),
                                         _p(trace, _f64p), _p(ctrace, _f64p), _p(changes, _i64p))
    return dict(A=A, C=C, B=B, mask=mask, Wbar=Wbar, r1=r1, r2=r2, loss_trace=trace,
                loss_cont_trace=ctrace[:n_iters], mask_changes=changes[:n_iters])


def denormalize(A, B, r1, r2):
    A, B = _f32(A).copy(), _f32(B).copy()
    r1, r2 = _f32(r1), _f32(r2)
    b = A.shape[-1]
    lib().oracle_denormalize(_p(A, _f32p), _p(B, _f32p), _p(r1, _f32p), _p(r2, _f32p), _i64(r2.shape[0]),
                             _i64(r1.shape[0]), _i64(b))
    return A, B


def pack_nm(C, mask, N, M):
    C = _f32(C)
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    d_out, d_in = C.shape
    values = np.zeros((d_out, d_in // M * N), dtype=np.float32)
    index = np.zeros((d_out, d_in // M * N), dtype=np.uint8)
    lib().oracle_pack_nm(_p(C, _f32p), _p(mask, _u8p), _i64(d_out), _i64(d_in), ctypes.c_int(N), ctypes.c_int(M),
                         _p(values, _f32p), _p(index, _u8p))
    return values, index


def pack_index_bits(index, M):
    """Byte-per-entry indices [d_out, entries] -> compact bit fields [d_out, ceil(entries*w/8)]."""
    index = np.ascontiguousarray(index, dtype=np.uint8)
    d_out, entries = index.shape
    w = {2: 1, 4: 2, 8: 4}[M]
    row_bytes = (entries * w + 7) // 8
    packed = np.zeros((d_out, row_bytes), dtype=np.uint8)
    lib().oracle_pack_index_bits(_p(index, _u8p), _i64(d_out), _i64(entries), ctypes.c_int(w), _p(packed, _u8p),
                                 _i64(row_bytes))
    return packed


def apply_packed(X, A, values, index, B, N, M, round_bf16=True):
    """y = A (S (B x)) for every row x of X, from the compressed core (Sec. 3.1 / Sec. 4.4). fp64 out."""
    X, A, B, values = _f32(X), _f32(A), _f32(B), _f32(values)
    index = np.ascontiguousarray(index, dtype=np.uint8)
    n, d_in = X.shape
    b = A.shape[-1]
    d_out = A.shape[0] * b
    Y = np.zeros((n, d_out), dtype=np.float64)
    lib().oracle_apply_packed(_p(X, _f32p), _i64(n), _p(A, _f32p), _p(values, _f32p), _p(index, _u8p), _p(B, _f32p),
                              _i64(d_out), _i64(d_in), _i64(b), ctypes.c_int(N), ctypes.c_int(M),
                              ctypes.c_int(1 if round_bf16 else 0), Y.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    return Y
