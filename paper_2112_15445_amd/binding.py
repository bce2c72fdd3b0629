"""Thin ctypes binding of libsparseconv.so (argument marshalling only).

Every step of the path -- the offset-stretching pass, the LDS staging, the gather-MAC kernels, the
autotuner -- runs inside the HIP library.  PyTorch appears only as the owner of device memory and
streams: tensors are passed down as raw device pointers.  There is no CPU fallback: if the shared
library is missing, importing the symbols fails loudly.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsparseconv.so")

SC_OK = 0
STATUS_NAMES = {0: "SC_OK", 1: "SC_ERR_NULL", 2: "SC_ERR_SHAPE", 3: "SC_ERR_CSR",
                4: "SC_ERR_UNSUPPORTED", 5: "SC_ERR_RANGE", 6: "SC_ERR_OOM", 7: "SC_ERR_WORKSPACE",
                8: "SC_ERR_HIP"}
SC_F32, SC_F16, SC_I8, SC_CB4_I8, SC_CB4_F16 = 0, 1, 2, 3, 4
DTYPES = {"f32": SC_F32, "f16": SC_F16, "i8": SC_I8, "cb4": SC_CB4_I8, "cb4h": SC_CB4_F16}
SC_VARIANT_AUTO, SC_VARIANT_GATHER, SC_VARIANT_SLAB, SC_VARIANT_DENSE = 0, 1, 2, 3
SC_STATIC_WORKSPACE_BYTES = 32 << 20
SC_PATH_SPARSE, SC_PATH_DENSE, SC_PATH_LIBRARY = 0, 1, 2

# every symbol include/sparse_conv.h declares
EXPORTS = [
    "sparse_conv_plan_create_csr", "sparse_conv_plan_create_ell", "sparse_conv_plan_destroy",
    "sparse_conv_plan_info", "sparse_conv_plan_debug_offsets", "sparse_conv_plan_set_tuning", "sparse_conv_plan_set_epilogue",
    "sparse_conv_plan_get_tuning", "sparse_conv_workspace_size", "sparse_conv_workspace_size_max",
    "sparse_conv_forward", "sparse_conv_forward_static", "sparse_conv_plan_autotune", "sparse_conv_autotune_workspace_size", "sparse_conv_plan_dispatch", "sparse_conv_plan_set_path",
    "sparse_conv_plan_num_candidates",
    "sparse_conv_plan_candidate", "sparse_conv_quantize_pow2", "sparse_conv_status_string",
]


class sc_layer_t(ctypes.Structure):
    _fields_ = [(k, ctypes.c_int32) for k in
                ("C", "D", "H", "W", "R", "S", "stride_h", "stride_w", "pad_h", "pad_w")]


class sc_tuning_t(ctypes.Structure):
    _fields_ = [("variant", ctypes.c_int32), ("wg_threads", ctypes.c_int32),
                ("sub_batch", ctypes.c_int32), ("tile_p", ctypes.c_int32),
                ("tile_q", ctypes.c_int32), ("wg_per_cu", ctypes.c_int32),
                ("wsrc", ctypes.c_int32), ("split_n", ctypes.c_int32),
                ("pipeline", ctypes.c_int32), ("producers", ctypes.c_int32),
                ("chunk_c", ctypes.c_int32), ("tile_d", ctypes.c_int32), ("ragged", ctypes.c_int32), ("pack", ctypes.c_int32),
                ("waves_m", ctypes.c_int32), ("buffers", ctypes.c_int32),
                ("stage_rows", ctypes.c_int32)]

    def as_dict(self):
        return {k: int(getattr(self, k)) for k, _ in self._fields_}


class sc_dispatch_t(ctypes.Structure):
    _fields_ = [("choice", ctypes.c_int32), ("sparse_ms", ctypes.c_float), ("dense_ms", ctypes.c_float),
                ("library_ms", ctypes.c_float), ("sparse_tuning", sc_tuning_t), ("dense_tuning", sc_tuning_t)]

    def as_dict(self):
        return {"choice": ("sparse", "dense", "library")[self.choice], "sparse_ms": self.sparse_ms,
                "dense_ms": self.dense_ms, "library_ms": self.library_ms,
                "sparse_tuning": self.sparse_tuning.as_dict(), "dense_tuning": self.dense_tuning.as_dict()}


class sc_plan_info_t(ctypes.Structure):
    _fields_ = [("n", ctypes.c_int32), ("P", ctypes.c_int32), ("Q", ctypes.c_int32),
                ("X_size", ctypes.c_int64), ("true_nnz", ctypes.c_int64),
                ("macs_per_sample", ctypes.c_int64), ("useful_macs_per_sample", ctypes.c_int64),
                ("act_bytes_per_sample", ctypes.c_int64), ("weight_bytes", ctypes.c_int64),
                ("lds_bytes", ctypes.c_int32), ("grid_size", ctypes.c_int32),
                ("tuning", sc_tuning_t), ("out_P", ctypes.c_int32), ("out_Q", ctypes.c_int32),
                ("out_elem_bytes", ctypes.c_int32)]


class sc_epilogue_t(ctypes.Structure):
    _fields_ = [("relu", ctypes.c_int32), ("pool", ctypes.c_int32), ("requant", ctypes.c_int32)]


class SparseConvError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib().sparse_conv_status_string(status).decode()
        super().__init__(f"{where}: {STATUS_NAMES.get(status, status)} ({msg})")


_lib = None


def lib() -> ctypes.CDLL:
    """Load libsparseconv.so; raises if it has not been built (no fallback)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'`")
    # PyTorch bundles its own HIP runtime.  Import it before the library so that both bind to the one
    # runtime already in the process; loaded the other way round the process ends up with two runtimes
    # and the second to initialise reports that it sees no GPU.
    import torch  # noqa: F401
    L = ctypes.CDLL(LIB_PATH)
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    P = ctypes.POINTER
    L.sparse_conv_plan_create_csr.argtypes = [P(sc_layer_t), ctypes.c_int, vp, vp, vp, vp, vp, vp, P(vp)]
    L.sparse_conv_plan_create_ell.argtypes = [P(sc_layer_t), ctypes.c_int, i32, vp, vp, vp, vp, vp, P(vp)]
    L.sparse_conv_plan_destroy.argtypes = [vp]
    L.sparse_conv_plan_destroy.restype = None
    L.sparse_conv_plan_info.argtypes = [vp, P(sc_plan_info_t)]
    L.sparse_conv_plan_debug_offsets.argtypes = [vp, vp]
    L.sparse_conv_plan_set_tuning.argtypes = [vp, P(sc_tuning_t), vp]
    L.sparse_conv_plan_get_tuning.argtypes = [vp, P(sc_tuning_t)]
    L.sparse_conv_plan_set_epilogue.argtypes = [vp, P(sc_epilogue_t), vp, vp]
    L.sparse_conv_workspace_size.argtypes = [vp, i32, P(sz)]
    L.sparse_conv_workspace_size_max.argtypes = [vp, i32, P(sz)]
    L.sparse_conv_forward.argtypes = [vp, vp, vp, i32, vp, sz, vp]
    L.sparse_conv_forward_static.argtypes = [vp, vp, vp, i32, vp]
    L.sparse_conv_plan_autotune.argtypes = [vp, vp, vp, i32, vp, sz, vp]
    L.sparse_conv_autotune_workspace_size.argtypes = [vp, i32, P(sz)]
    L.sparse_conv_plan_dispatch.argtypes = [vp, vp, vp, i32, vp, sz, vp, P(sc_dispatch_t)]
    L.sparse_conv_plan_set_path.argtypes = [vp, i32, vp]
    L.sparse_conv_plan_num_candidates.argtypes = [vp, P(i32)]
    L.sparse_conv_plan_candidate.argtypes = [vp, i32, P(sc_tuning_t)]
    L.sparse_conv_quantize_pow2.argtypes = [vp, sz, i32, ctypes.c_float, vp, P(i32)]
    L.sparse_conv_status_string.argtypes = [ctypes.c_int]
    L.sparse_conv_status_string.restype = ctypes.c_char_p
    for name in EXPORTS:
        if name not in ("sparse_conv_plan_destroy", "sparse_conv_status_string"):
            getattr(L, name).restype = ctypes.c_int
    _lib = L
    return L


def _check(status: int, where: str):
    if status != SC_OK:
        raise SparseConvError(status, where)


def _host(a: Optional[np.ndarray], dtype) -> Optional[np.ndarray]:
    return None if a is None else np.ascontiguousarray(a, dtype=dtype)


def _hp(a: Optional[np.ndarray]):
    return None if a is None else ctypes.c_void_p(a.ctypes.data)


_VALUE_NP = {SC_F32: np.float32, SC_F16: np.float16, SC_I8: np.int8, SC_CB4_I8: np.uint8, SC_CB4_F16: np.uint8}
_CODEBOOK_NP = {SC_CB4_I8: np.int8, SC_CB4_F16: np.float16}


def quantize_pow2(x: np.ndarray, total_bits: int = 8, saturate_at: float = 1.0):
    """sparse_conv_quantize_pow2: (codes int8 with the shape of x, frac_bits)."""
    xa = np.ascontiguousarray(x, dtype=np.float32)
    codes = np.empty(xa.shape, dtype=np.int8)
    fb = ctypes.c_int32(0)
    _check(lib().sparse_conv_quantize_pow2(_hp(xa) if xa.size else None, xa.size, total_bits, saturate_at,
                                           _hp(codes) if xa.size else None, ctypes.byref(fb)),
           "sparse_conv_quantize_pow2")
    return codes, int(fb.value)


def make_layer(C, D, H, W, R, S, stride=(1, 1), pad=(0, 0)) -> sc_layer_t:
    return sc_layer_t(C, D, H, W, R, S, stride[0], stride[1], pad[0], pad[1])


class Plan:
    """Owner of one sparse_conv_plan_t.  Same calls as the C ABI, same names."""

    def __init__(self, handle: int, layer: sc_layer_t, dtype: int):
        self._h = ctypes.c_void_p(handle)
        self.layer = layer
        self.dtype = dtype

    # -- construction -------------------------------------------------------------------------
    @staticmethod
    def create_csr(layer: sc_layer_t, dtype: int, rowptr, colidx, values, scales=None,
                   codebook=None, stream: int = 0) -> "Plan":
        rp = _host(rowptr, np.int32)
        ci = _host(colidx, np.int32)
        va = _host(values, _VALUE_NP.get(dtype, np.uint8))
        sc_ = _host(scales, np.float32)
        cb = _host(codebook, _CODEBOOK_NP.get(dtype, np.int8))
        out = ctypes.c_void_p()
        st = lib().sparse_conv_plan_create_csr(ctypes.byref(layer), dtype, _hp(rp), _hp(ci), _hp(va),
                                               _hp(sc_), _hp(cb), ctypes.c_void_p(stream),
                                               ctypes.byref(out))
        _check(st, "sparse_conv_plan_create_csr")
        return Plan(out.value, layer, dtype)

    @staticmethod
    def create_ell(layer: sc_layer_t, dtype: int, n: int, colidx, values, scales=None,
                   codebook=None, stream: int = 0) -> "Plan":
        ci = _host(colidx, np.int32)
        va = _host(values, _VALUE_NP.get(dtype, np.uint8))
        sc_ = _host(scales, np.float32)
        cb = _host(codebook, _CODEBOOK_NP.get(dtype, np.int8))
        out = ctypes.c_void_p()
        st = lib().sparse_conv_plan_create_ell(ctypes.byref(layer), dtype, n, _hp(ci), _hp(va),
                                               _hp(sc_), _hp(cb), ctypes.c_void_p(stream),
                                               ctypes.byref(out))
        _check(st, "sparse_conv_plan_create_ell")
        return Plan(out.value, layer, dtype)

    def destroy(self):
        if self._h:
            lib().sparse_conv_plan_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    # -- queries ------------------------------------------------------------------------------
    def info(self) -> sc_plan_info_t:
        inf = sc_plan_info_t()
        _check(lib().sparse_conv_plan_info(self._h, ctypes.byref(inf)), "sparse_conv_plan_info")
        return inf

    def debug_offsets(self) -> np.ndarray:
        inf = self.info()
        out = np.zeros((self.layer.D, inf.n), dtype=np.int32)
        _check(lib().sparse_conv_plan_debug_offsets(self._h, _hp(out)), "sparse_conv_plan_debug_offsets")
        return out

    def get_tuning(self) -> sc_tuning_t:
        t = sc_tuning_t()
        _check(lib().sparse_conv_plan_get_tuning(self._h, ctypes.byref(t)), "sparse_conv_plan_get_tuning")
        return t

    def set_tuning(self, tuning: Optional[sc_tuning_t] = None, stream: int = 0, **fields):
        t = tuning if tuning is not None else sc_tuning_t()
        for k, v in fields.items():
            setattr(t, k, v)
        _check(lib().sparse_conv_plan_set_tuning(self._h, ctypes.byref(t), ctypes.c_void_p(stream)),
               "sparse_conv_plan_set_tuning")

    def set_epilogue(self, relu: bool = False, pool: int = 0, requant_scale=None, stream: int = 0):
        ep = sc_epilogue_t(int(bool(relu)), int(pool), int(requant_scale is not None))
        rq = _host(requant_scale, np.float32)
        _check(lib().sparse_conv_plan_set_epilogue(self._h, ctypes.byref(ep), _hp(rq), ctypes.c_void_p(stream)),
               "sparse_conv_plan_set_epilogue")

    def workspace_size(self, N: int) -> int:
        b = ctypes.c_size_t()
        _check(lib().sparse_conv_workspace_size(self._h, N, ctypes.byref(b)), "sparse_conv_workspace_size")
        return int(b.value)

    def workspace_size_max(self, N: int) -> int:
        b = ctypes.c_size_t()
        _check(lib().sparse_conv_workspace_size_max(self._h, N, ctypes.byref(b)),
               "sparse_conv_workspace_size_max")
        return int(b.value)

    def dispatch(self, x_ptr: int, y_ptr: int, N: int, ws_ptr: int = 0, ws_bytes: int = 0, stream: int = 0):
        rec = sc_dispatch_t()
        _check(lib().sparse_conv_plan_dispatch(self._h, ctypes.c_void_p(x_ptr), ctypes.c_void_p(y_ptr), N,
                                               ctypes.c_void_p(ws_ptr), ws_bytes, ctypes.c_void_p(stream),
                                               ctypes.byref(rec)),
               "sparse_conv_plan_dispatch")
        return rec

    def set_path(self, path: int, stream: int = 0):
        _check(lib().sparse_conv_plan_set_path(self._h, path, ctypes.c_void_p(stream)), "sparse_conv_plan_set_path")

    def autotune_workspace_size(self, N: int) -> int:
        b = ctypes.c_size_t()
        _check(lib().sparse_conv_autotune_workspace_size(self._h, N, ctypes.byref(b)),
               "sparse_conv_autotune_workspace_size")
        return int(b.value)

    def num_candidates(self) -> int:
        c = ctypes.c_int32()
        _check(lib().sparse_conv_plan_num_candidates(self._h, ctypes.byref(c)),
               "sparse_conv_plan_num_candidates")
        return int(c.value)

    def candidate(self, i: int) -> sc_tuning_t:
        t = sc_tuning_t()
        _check(lib().sparse_conv_plan_candidate(self._h, i, ctypes.byref(t)), "sparse_conv_plan_candidate")
        return t

    # -- execution (raw device pointers) --------------------------------------------------------
    def forward(self, x_ptr: int, y_ptr: int, N: int, ws_ptr: int = 0, ws_bytes: int = 0,
                stream: int = 0):
        _check(lib().sparse_conv_forward(self._h, ctypes.c_void_p(x_ptr), ctypes.c_void_p(y_ptr), N,
                                         ctypes.c_void_p(ws_ptr), ws_bytes, ctypes.c_void_p(stream)),
               "sparse_conv_forward")

    def forward_static(self, x_ptr: int, y_ptr: int, N: int, stream: int = 0):
        _check(lib().sparse_conv_forward_static(self._h, ctypes.c_void_p(x_ptr), ctypes.c_void_p(y_ptr), N,
                                                ctypes.c_void_p(stream)),
               "sparse_conv_forward_static")

    def autotune(self, x_ptr: int, y_ptr: int, N: int, ws_ptr: int = 0, ws_bytes: int = 0,
                 stream: int = 0):
        _check(lib().sparse_conv_plan_autotune(self._h, ctypes.c_void_p(x_ptr), ctypes.c_void_p(y_ptr),
                                               N, ctypes.c_void_p(ws_ptr), ws_bytes,
                                               ctypes.c_void_p(stream)),
               "sparse_conv_plan_autotune")


# -------------------------------------------------------------------------------------------------
# torch conveniences used by the tests and the benchmark (device memory and streams only)
# -------------------------------------------------------------------------------------------------
def torch_out_dtype(dtype: int):
    import torch
    return {SC_F32: torch.float32, SC_F16: torch.float16, SC_I8: torch.int32, SC_CB4_I8: torch.int32,
            SC_CB4_F16: torch.float16}[dtype]


def forward_torch(plan: Plan, x, y=None, workspace=None):
    """Run sparse_conv_forward on torch CUDA tensors on torch's current stream."""
    import torch
    assert x.is_cuda and x.is_contiguous()
    N = x.shape[0]
    inf = plan.info()
    if y is None:
        y = torch.empty((N, plan.layer.D, inf.P, inf.Q), dtype=torch_out_dtype(plan.dtype), device=x.device)
    need = plan.workspace_size(N)
    if need and (workspace is None or workspace.numel() * workspace.element_size() < need):
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
    stream = torch.cuda.current_stream(x.device).cuda_stream
    plan.forward(x.data_ptr(), y.data_ptr(), N,
                 workspace.data_ptr() if workspace is not None else 0,
                 workspace.numel() * workspace.element_size() if workspace is not None else 0, stream)
    return y
