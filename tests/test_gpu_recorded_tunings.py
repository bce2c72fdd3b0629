"""Every layer of every workload configuration at FULL batch, in the path and launch shape recorded
for it (paper_2112_15445_amd/tunings/mi355x.json: what the per-layer dispatch installed on an MI355X
and the per-layer report timed -- gather kernels, the densified tile on the matrix cores, or the dense
library), against the CPU oracle: samples 0..15 and the last one, element by element.

The shapes are installed with sparse_conv_plan_set_tuning and sparse_conv_plan_set_path (nothing is
timed here), so that the result the benchmark figures stand for is the one that is checked."""
import json
import os

import pytest

from paper_2112_15445_amd import binding as B
from paper_2112_15445_amd import workloads as wl

import gpu_util as G

pytestmark = pytest.mark.gpu

_PATH = os.path.join(os.path.dirname(os.path.abspath(B.__file__)), "tunings", "mi355x.json")
ROWS = json.load(open(_PATH))
_LAYERS = {(l.name, l.dtype): l for c in wl.CONFIGS for l in wl.CONFIGS[c]()}


def test_every_workload_layer_has_a_recorded_tuning():
    assert {(r["layer"], r["dtype"]) for r in ROWS} == set(_LAYERS)


@pytest.mark.parametrize("row", ROWS, ids=[f"cfg{r['config']}-{r['layer']}-{r['dtype']}" for r in ROWS])
def test_recorded_tuning_at_full_batch(row):
    l = _LAYERS[(row["layer"], row["dtype"])]
    print("case recorded tuning", l.name, l.dtype, "N", l.N, row["tuning"], flush=True)
    data = wl.prepare(l)
    plan = G.make_plan(l, data)
    plan.set_tuning(B.sc_tuning_t(), **row["tuning"])
    got = {k: v for k, v in plan.get_tuning().as_dict().items() if v}
    assert got == row["tuning"], (got, row["tuning"])        # installed exactly as recorded
    tol, x_dev = None, None
    if row.get("path") == "library":
        # the library leg exists once the dispatch has measured it on real buffers; then the recorded
        # shape and path are installed over whatever that run chose.  The dense library chooses its
        # own algorithm and summation order: fp32 layers are held to 1e-3 of the output scale there
        import numpy as np
        import torch
        x_dev = G.to_device(np.ascontiguousarray(data["x"]))
        inf = plan.info()
        y = torch.empty((l.N, l.D, inf.P, inf.Q), dtype=B.torch_out_dtype(plan.dtype), device="cuda")
        ws = torch.empty(max(plan.workspace_size_max(l.N), 16), dtype=torch.uint8, device="cuda")
        plan.dispatch(x_dev.data_ptr(), y.data_ptr(), l.N, ws.data_ptr(), ws.numel(), torch.cuda.current_stream().cuda_stream)
        plan.set_tuning(B.sc_tuning_t(), **row["tuning"])
        plan.set_path(B.SC_PATH_LIBRARY)
        tol = 1e-3 if l.dtype == "f32" else None
    res = G.full_batch_parity(l, data, plan, x_dev=x_dev, tol=tol)
    plan.destroy()
    assert res["ok"], res
