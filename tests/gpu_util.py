"""Helpers for the GPU parity tests: run one layer through the C ABI and through the oracle."""
from __future__ import annotations

import numpy as np

import oracle
from paper_2112_15445_amd import binding as B
from paper_2112_15445_amd import workloads as wl

# Floating-point tolerance per layer, applied three ways (check): max|y - ref| / max|ref|, relative
# L2 error, and element by element |y - ref| <= tol * |ref| + tol * rms(ref).  Integer paths: exact.
TOL = {"f32": 1e-5, "f16": 2e-2, "i8": 0.0, "cb4": 0.0, "cb4h": 2e-2}
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


def check(l: wl.Layer, y: np.ndarray, ref: np.ndarray, what: str = "", tol=None):
    assert y.shape == ref.shape, (what, y.shape, ref.shape)
    if l.dtype in ("i8", "cb4"):
        assert np.array_equal(y, ref), f"{what}: integer outputs differ in {np.count_nonzero(y != ref)} places"
    else:
        assert np.all(np.isfinite(y.astype(np.float64))), what
        tol = TOL[l.dtype] if tol is None else tol
        e = rel_err(y, ref)
        assert e <= tol, f"{what}: rel err {e:.3e} > {tol:.1e}"
        yd, rd = y.astype(np.float64), ref.astype(np.float64)
        nrm = float(np.sqrt(np.sum(rd * rd)))
        l2 = float(np.sqrt(np.sum((yd - rd) ** 2))) / nrm if nrm > 0 else 0.0
        assert l2 <= tol, f"{what}: relative L2 error {l2:.3e} > {tol:.1e}"
        rms = nrm / np.sqrt(max(rd.size, 1))
        excess = np.abs(yd - rd) - tol * (np.abs(rd) + rms)
        worst = int(np.argmax(excess)) if excess.size else 0
        assert not excess.size or excess.flat[worst] <= 0, (
            f"{what}: element {np.unravel_index(worst, y.shape)}: y {yd.flat[worst]!r} ref {rd.flat[worst]!r} "
            f"(allowed {tol:.1e} * (|ref| + rms {rms:.3e}))")


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


def full_batch_parity(l: wl.Layer, data, plan: B.Plan, x_dev=None, ws=None, group: int = 16, tol=None):
    """The installed launch shape on the FULL batch against the oracle on sampled outputs: samples
    0..group-1 (one whole group of every multi-sample launch shape: up to 16 samples share a
    workgroup) and the last one, every element of those.  Returns {"ok", "samples", "rel_err"} or
    {"ok": False, "samples", "error"}."""
    import torch
    inf = plan.info()
    if x_dev is None:
        x_dev = to_device(np.ascontiguousarray(data["x"]))
    y = torch.empty((l.N, l.D, inf.P, inf.Q), dtype=B.torch_out_dtype(plan.dtype), device="cuda")
    y.view(torch.uint8).fill_(0x7f)
    need = plan.workspace_size(l.N)
    if need and (ws is None or ws.numel() * ws.element_size() < need):
        ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    wsp, wsn = (ws.data_ptr(), ws.numel() * ws.element_size()) if ws is not None else (0, 0)
    plan.forward(x_dev.data_ptr(), y.data_ptr(), l.N, wsp, wsn, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    idx = sorted(set(range(min(group, l.N))) | {l.N - 1})
    got = to_host(y[idx].contiguous())
    ref = oracle_out(l, data, samples=idx)
    try:
        check(l, got, ref, l.name, tol=tol)
    except AssertionError as e:
        return {"ok": False, "samples": idx, "error": str(e)[:300]}
    return {"ok": True, "samples": idx, "rel_err": rel_err(got, ref)}
