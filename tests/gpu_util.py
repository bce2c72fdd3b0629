"""Helpers for the GPU parity tests: run one layer through the C ABI and through the oracle."""
from __future__ import annotations

import numpy as np

import oracle
from paper_2112_15445_amd import binding as B
from paper_2112_15445_amd import workloads as wl

TOL = {"f32": 1e-5, "f16": 2e-2, "i8": 0.0, "cb4": 0.0, "cb4h": 2e-2}   # max|y - ref| / max|ref|, per layer
NP_OUT = {"f32": np.float32, "f16": np.float16, "i8": np.int32, "cb4": np.int32, "cb4h": np.float16}


def layer_desc(l: wl.Layer):
    return B.make_layer(l.C, l.D, l.H, l.W, l.R, l.S, (l.stride_h, l.stride_w), (l.pad_h, l.pad_w))


def make_plan(l: wl.Layer, data) -> B.Plan:
    return B.Plan.create_csr(layer_desc(l), B.DTYPES[l.dtype], data["rowptr"], data["colidx"],
                             data["values"], data["scales"], data["codebook"])


def oracle_out(l: wl.Layer, data, samples=None) -> np.ndarray:
    x = data["x"] if samples is None else data["x"][samples]
    return oracle.sparse_conv(x, data["rowptr"], data["colidx"], data["values"], l.R, l.S,
                              (l.stride_h, l.stride_w), (l.pad_h, l.pad_w),
                              codebook=data["codebook"], out_dtype=NP_OUT[l.dtype])


def to_device(x: np.ndarray):
    import torch
    if x.dtype == np.float16:
        return torch.from_numpy(x.view(np.int16)).cuda().view(torch.float16)
    return torch.from_numpy(x).cuda()


def to_host(y) -> np.ndarray:
    import torch
    if y.dtype == torch.float16:
        return y.view(torch.int16).cpu().numpy().view(np.float16)
    return y.cpu().numpy()


def rel_err(y: np.ndarray, ref: np.ndarray) -> float:
    den = float(np.max(np.abs(ref.astype(np.float64)))) if ref.size else 0.0
    num = float(np.max(np.abs(y.astype(np.float64) - ref.astype(np.float64)))) if ref.size else 0.0
    return num / den if den > 0 else num


def check(l: wl.Layer, y: np.ndarray, ref: np.ndarray, what: str = ""):
    assert y.shape == ref.shape, (what, y.shape, ref.shape)
    if l.dtype in ("i8", "cb4"):
        assert np.array_equal(y, ref), f"{what}: integer outputs differ in {np.count_nonzero(y != ref)} places"
    else:
        assert np.all(np.isfinite(y.astype(np.float64))), what
        e = rel_err(y, ref)
        assert e <= TOL[l.dtype], f"{what}: rel err {e:.3e} > {TOL[l.dtype]:.1e}"


def run_gpu(plan: B.Plan, x: np.ndarray, poison: bool = True) -> np.ndarray:
    import torch
    xd = to_device(np.ascontiguousarray(x))
    inf = plan.info()
    y = torch.empty((x.shape[0], plan.layer.D, inf.P, inf.Q), dtype=B.torch_out_dtype(plan.dtype),
                    device="cuda")
    if poison:   # make unwritten outputs visible
        y.view(torch.uint8).fill_(0x7f)
    B.forward_torch(plan, xd, y)
    torch.cuda.synchronize()
    return to_host(y)
