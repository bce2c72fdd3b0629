"""ctypes front end of the CPU oracle (``sparse_conv_oracle.c``) -- TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the benchmark's cpu_baseline leg may import this module.  It
shares no code with the HIP library.  Floating-point operands (fp32 or fp16 storage) are widened to
double exactly, all arithmetic happens in double, and the result is rounded once to the storage
type; integer operands (int8 storage) are widened to int32 and accumulated in int32.

Definitions follow the paper's section on convolution via a sparse operation: CSR rows are output
channels, columns are filter taps flattened as (c, r, s), rows are padded to a common non-zero
count, column indices are stretched to offsets into the zero-padded NCHW input, and Algorithm 3
gathers and accumulates one output pixel at a time.
"""
from __future__ import annotations

import ctypes
import math
import os
import subprocess
from typing import Dict, Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sparse_conv_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (-O2, OpenMP, no hand vectorisation)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall",
                               "-Wextra", "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build()
    lib = ctypes.CDLL(_LIB)
    i, i64, sz, vp = ctypes.c_int, ctypes.c_int64, ctypes.c_size_t, ctypes.c_void_p
    lib.oracle_num_threads.restype = i
    for name in ("oracle_dense_conv_f64", "oracle_dense_conv_i32"):
        getattr(lib, name).argtypes = [vp, vp, vp] + [i] * 11
        getattr(lib, name).restype = None
    lib.oracle_unified_nnz.argtypes = [vp, i]
    lib.oracle_unified_nnz.restype = i
    for name in ("oracle_unify_rows_f64", "oracle_unify_rows_i32"):
        getattr(lib, name).argtypes = [vp, vp, vp, i, i, vp, vp]
        getattr(lib, name).restype = None
    lib.oracle_stretch.argtypes = [vp, sz, i, i, i, i, vp]
    lib.oracle_stretch.restype = None
    for name in ("oracle_pad_input_f64", "oracle_pad_input_i32"):
        getattr(lib, name).argtypes = [vp, i, i, i, i, i, i, vp]
        getattr(lib, name).restype = None
    for name in ("oracle_gather_mac_f64", "oracle_gather_mac_i32"):
        getattr(lib, name).argtypes = [vp, vp, vp, vp, i, i64, i, i, i, i, i, i, i]
        getattr(lib, name).restype = None
    lib.oracle_decode_codebook.argtypes = [vp, sz, vp, vp]
    lib.oracle_decode_codebook.restype = None
    lib.oracle_decode_codebook_f64.argtypes = [vp, sz, vp, vp]
    lib.oracle_decode_codebook_f64.restype = None
    _lib = lib
    return lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def _p(a: np.ndarray) -> ctypes.c_void_p:
    return ctypes.c_void_p(a.ctypes.data)


def out_shape(H, W, R, S, stride, pad) -> Tuple[int, int]:
    return ((H + 2 * pad[0] - R) // stride[0] + 1, (W + 2 * pad[1] - S) // stride[1] + 1)


def _is_int(a: np.ndarray) -> bool:
    return np.issubdtype(a.dtype, np.integer)


def _round_out(y: np.ndarray, dtype: np.dtype) -> np.ndarray:
    """Single rounding from the accumulator type to the storage type."""
    return y.astype(dtype)


def dense_conv(x: np.ndarray, wt: np.ndarray, stride=(1, 1), pad=(0, 0), out_dtype=None
               ) -> np.ndarray:
    """Textbook direct convolution.  x [N,C,H,W], wt [D,C,R,S] -> y [N,D,P,Q]."""
    lib = _load()
    N, C, H, W = x.shape
    D, C2, R, S = wt.shape
    assert C == C2
    P, Q = out_shape(H, W, R, S, stride, pad)
    assert P > 0 and Q > 0
    if _is_int(x):
        xa = np.ascontiguousarray(x, dtype=np.int32)
        wa = np.ascontiguousarray(wt, dtype=np.int32)
        y = np.empty((N, D, P, Q), dtype=np.int32)
        lib.oracle_dense_conv_i32(_p(xa), _p(wa), _p(y), N, C, H, W, D, R, S, stride[0], stride[1],
                                  pad[0], pad[1])
        return y
    xa = np.ascontiguousarray(x, dtype=np.float64)
    wa = np.ascontiguousarray(wt, dtype=np.float64)
    y = np.empty((N, D, P, Q), dtype=np.float64)
    lib.oracle_dense_conv_f64(_p(xa), _p(wa), _p(y), N, C, H, W, D, R, S, stride[0], stride[1],
                              pad[0], pad[1])
    return y if out_dtype is None else _round_out(y, out_dtype)


def dense_from_csr(rowptr, colidx, values, D, C, R, S) -> np.ndarray:
    """Scatter CSR rows (output channel x flattened (c,r,s)) into a dense [D,C,R,S] tensor.
    Duplicate columns in a row add up."""
    dt = np.int32 if _is_int(np.asarray(values)) else np.float64
    w = np.zeros((D, C * R * S), dtype=dt)
    for d in range(D):
        for k in range(rowptr[d], rowptr[d + 1]):
            w[d, colidx[k]] += values[k]
    return w.reshape(D, C, R, S)


def sparse_conv_steps(x: np.ndarray, rowptr: np.ndarray, colidx: np.ndarray, values: np.ndarray,
                      R: int, S: int, stride=(1, 1), pad=(0, 0),
                      codebook: Optional[np.ndarray] = None) -> Dict[str, object]:
    """Run the four steps of the sparse method and return every intermediate.

    values: fp32/fp16 weights, int8 weights, or (with ``codebook``: int8 centroids for integer
    activations, floating-point centroids otherwise) uint8 centroid indices.
    Returns dict(n, col [D,n], theta [D,n], lam [D,n] int64, xp [N,C,Hp,Wp], y [N,D,P,Q]) with y in
    the accumulator type (float64 or int32).
    """
    lib = _load()
    N, C, H, W = x.shape
    D = rowptr.shape[0] - 1
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int32)
    colidx = np.ascontiguousarray(colidx, dtype=np.int32)
    K = C * R * S
    assert rowptr[0] == 0 and rowptr[-1] == colidx.shape[0] == np.asarray(values).shape[0]
    assert np.all(np.diff(rowptr) >= 0)
    assert colidx.size == 0 or (colidx.min() >= 0 and colidx.max() < K)
    P, Q = out_shape(H, W, R, S, stride, pad)
    assert P > 0 and Q > 0
    Hp, Wp = H + 2 * pad[0], W + 2 * pad[1]
    X_size = C * Hp * Wp
    integer = _is_int(x)

    if codebook is not None and integer:
        idx = np.ascontiguousarray(values, dtype=np.uint8)
        assert idx.size == 0 or idx.max() < 16
        cb = np.ascontiguousarray(codebook, dtype=np.int32)
        assert cb.shape == (16,)
        vals = np.empty(idx.shape[0], dtype=np.int32)
        lib.oracle_decode_codebook(_p(idx), idx.shape[0], _p(cb), _p(vals))
    elif codebook is not None:
        # sixteen-bit centroids with floating-point activations (the 4b/16b configuration of the
        # quantisation-results table): the same index -> centroid mapping, centroid values exact
        idx = np.ascontiguousarray(values, dtype=np.uint8)
        assert idx.size == 0 or idx.max() < 16
        cb = np.ascontiguousarray(codebook, dtype=np.float64)
        assert cb.shape == (16,)
        vals = np.empty(idx.shape[0], dtype=np.float64)
        lib.oracle_decode_codebook_f64(_p(idx), idx.shape[0], _p(cb), _p(vals))
    elif integer:
        vals = np.ascontiguousarray(values, dtype=np.int32)
    else:
        vals = np.ascontiguousarray(values, dtype=np.float64)
    assert integer == _is_int(vals), "integer activations need integer weights and vice versa"
    wtype = np.int32 if integer else np.float64

    # step 1: unify the row lengths
    n = int(lib.oracle_unified_nnz(_p(rowptr), D))
    col = np.zeros((D, n), dtype=np.int32)
    theta = np.zeros((D, n), dtype=wtype)
    unify = lib.oracle_unify_rows_i32 if integer else lib.oracle_unify_rows_f64
    unify(_p(rowptr), _p(colidx), _p(vals), D, n, _p(col), _p(theta))
    # step 2: stretch columns to padded-input offsets
    lam = np.zeros((D, n), dtype=np.int64)
    lib.oracle_stretch(_p(col), D * n, R, S, Hp, Wp, _p(lam))
    # step 3: padded input
    xa = np.ascontiguousarray(x, dtype=wtype)
    xp = np.empty((N, C, Hp, Wp), dtype=wtype)
    (lib.oracle_pad_input_i32 if integer else lib.oracle_pad_input_f64)(
        _p(xa), N, C, H, W, pad[0], pad[1], _p(xp))
    # step 4: gather-multiply-accumulate
    y = np.empty((N, D, P, Q), dtype=wtype)
    (lib.oracle_gather_mac_i32 if integer else lib.oracle_gather_mac_f64)(
        _p(xp), _p(theta), _p(lam), _p(y), N, X_size, D, n, P, Q, stride[0], stride[1], Wp)
    return {"n": n, "col": col, "theta": theta, "lam": lam, "xp": xp, "y": y}


def sparse_conv(x, rowptr, colidx, values, R, S, stride=(1, 1), pad=(0, 0), codebook=None,
                out_dtype=None) -> np.ndarray:
    """Direct sparse convolution; result rounded once to ``out_dtype`` (default: accumulator type)."""
    y = sparse_conv_steps(x, rowptr, colidx, values, R, S, stride, pad, codebook)["y"]
    return y if out_dtype is None else _round_out(y, out_dtype)


def quantise_pow2(x: np.ndarray, total_bits: int = 8, saturate_at: float = 1.0) -> Tuple[np.ndarray, int]:
    """The paper's linear fixed-point quantiser (section "Quantisation": q = sigma * round(x / sigma)
    with mu = 0, sigma = 2^-frac_bits, int_bits = ceil(log2 max|x|), frac_bits = total_bits -
    int_bits - 1), per tensor.  Returns (integer codes round(x / sigma) as int8, frac_bits).

    Readings taken where the text is silent: "round" is round-to-nearest with ties to even; codes
    saturate to the two's-complement range of total_bits (a maximum that is an exact power of two
    would otherwise need one more bit); the activation saturation threshold (0.99 in the paper's
    experiments) scales the maximum before int_bits is taken and clips the data to it; an all-zero
    tensor gets int_bits = 0.
    """
    xd = np.asarray(x, dtype=np.float64)
    assert np.all(np.isfinite(xd)) and 2 <= total_bits <= 8 and 0.0 < saturate_at <= 1.0
    m = float(saturate_at) * (float(np.max(np.abs(xd))) if xd.size else 0.0)
    int_bits = int(math.ceil(math.log2(m))) if m > 0.0 else 0
    # log2 of an exact power of two is exact in IEEE double; guard the neighbours against a last-bit error
    if m > 0.0:
        while 2.0 ** int_bits < m:
            int_bits += 1
        while 2.0 ** (int_bits - 1) >= m:
            int_bits -= 1
    frac_bits = total_bits - int_bits - 1
    sigma = 2.0 ** (-frac_bits)
    code = np.rint(np.clip(xd, -m, m) / sigma)
    code = np.clip(code, -(2 ** (total_bits - 1)), 2 ** (total_bits - 1) - 1)
    return code.astype(np.int8), frac_bits


def epilogue(y: np.ndarray, relu: bool = False, pool: int = 0, requant_scale: Optional[np.ndarray] = None,
             out_dtype=None) -> np.ndarray:
    """What follows the convolution inside one layer of a VGG-shaped stack (the network the paper's
    main scheme configures layer by layer), applied to the accumulator-type output ``y`` [N, D, P, Q]
    of ``sparse_conv_steps``: ReLU ``max(0, .)``; 2 x 2 max-pooling with stride 2 (an odd last row /
    column is dropped); then either one rounding to ``out_dtype`` or, for integer accumulators,
    requantisation to 8-bit codes for the next layer,
    ``clip(round_half_even(float32(acc) * float32(scale[d])), -127, 127)``: the paper's linear
    quantiser q = round(x / sigma) applied to the real value acc * s_w[d] * s_x with
    scale[d] = s_w[d] * s_x / sigma_next, evaluated in single precision -- the conversion of the
    accumulator, the product and the rounding are each one IEEE operation, so the code is a
    deterministic function of (acc, scale[d])."""
    v = np.asarray(y)
    assert v.ndim == 4 and pool in (0, 2)
    if relu:
        v = np.maximum(v, 0)
    if pool == 2:
        N, D, P, Q = v.shape
        Po, Qo = P // 2, Q // 2
        out = np.empty((N, D, Po, Qo), dtype=v.dtype)
        for pp in range(Po):
            for qq in range(Qo):
                win = v[:, :, 2 * pp:2 * pp + 2, 2 * qq:2 * qq + 2]
                out[:, :, pp, qq] = win.reshape(N, D, 4).max(axis=2)
        v = out
    if requant_scale is not None:
        assert np.issubdtype(v.dtype, np.integer)
        sc = np.asarray(requant_scale, dtype=np.float32).reshape(1, -1, 1, 1)
        q = np.rint(v.astype(np.float32) * sc)              # float32 x float32 -> float32, ties to even
        return np.clip(q, -127.0, 127.0).astype(np.int8)
    return v if out_dtype is None else _round_out(v, out_dtype)
