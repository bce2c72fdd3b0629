"""sparse_conv_forward_static (the entry point that allocates nothing and takes no workspace) against
sparse_conv_forward on the same plan: two calls in a row, the second on a smaller batch, so that
what the first call left in the library's static scratch array would show if it were reused."""
import numpy as np
import pytest

from paper_2112_15445_amd import binding as B
from paper_2112_15445_amd import workloads as wl

import gpu_util as G

pytestmark = pytest.mark.gpu


def _both(plan, l, x):
    """(y of sparse_conv_forward with a caller workspace, y of sparse_conv_forward_static)."""
    import torch
    xd = G.to_device(np.ascontiguousarray(x))
    inf = plan.info()
    shape = (x.shape[0], l.D, inf.P, inf.Q)
    y_ref = torch.empty(shape, dtype=B.torch_out_dtype(plan.dtype), device="cuda")
    y_sta = torch.empty(shape, dtype=B.torch_out_dtype(plan.dtype), device="cuda")
    y_ref.view(torch.uint8).fill_(0x7f)
    y_sta.view(torch.uint8).fill_(0x5b)
    B.forward_torch(plan, xd, y_ref)
    st = torch.cuda.current_stream().cuda_stream
    plan.forward_static(xd.data_ptr(), y_sta.data_ptr(), x.shape[0], st)
    torch.cuda.synchronize()
    return G.to_host(y_ref), G.to_host(y_sta)


@pytest.mark.parametrize("dtype", ["f32", "f16", "i8", "cb4"])
def test_static_workspace_forward_matches_forward(dtype):
    (l,) = wl.config1()
    l = l.replace(dtype=dtype, N=5, H=19, W=23)           # padded copy: 5 x 64 x 21 x 25 elements
    data = wl.prepare(l)
    ref = G.oracle_out(l, data)
    plan = G.make_plan(l, data)
    for variant, extra in ((B.SC_VARIANT_GATHER, {"sub_batch": 2}), (B.SC_VARIANT_GATHER, {"split_n": 4}),
                           (B.SC_VARIANT_SLAB, {})):
        plan.set_tuning(B.sc_tuning_t(), variant=variant, **extra)
        need = plan.workspace_size(l.N)
        assert (need > 0) == (variant == B.SC_VARIANT_GATHER)
        for ns in (5, 2):                                  # the second call is the smaller one
            print("case static", dtype, variant, extra, "N", ns, flush=True)
            y_ref, y_sta = _both(plan, l, data["x"][:ns])
            assert np.array_equal(y_ref.view(np.uint8), y_sta.view(np.uint8)), (dtype, variant, ns)
            G.check(l, y_sta, ref[:ns], f"static {dtype} variant {variant} N {ns}")
    plan.destroy()


def test_static_workspace_forward_rejects_what_does_not_fit():
    import torch
    l = wl.Layer("big_pad", 64, 4, 126, 126, N=9, sparsity=0.99, dtype="f32")   # 9 x 64 x 128 x 128 x 4 B = 36 MiB
    data = wl.prepare(l)
    plan = G.make_plan(l, data)
    plan.set_tuning(B.sc_tuning_t(), variant=B.SC_VARIANT_GATHER)
    assert plan.workspace_size(l.N) > B.SC_STATIC_WORKSPACE_BYTES
    xd = G.to_device(data["x"])
    y = torch.zeros((l.N, l.D, l.P, l.Q), dtype=torch.float32, device="cuda")
    with pytest.raises(B.SparseConvError) as e:
        plan.forward_static(xd.data_ptr(), y.data_ptr(), l.N, 0)
    assert e.value.status == 7                             # SC_ERR_WORKSPACE, nothing launched
    torch.cuda.synchronize()
    assert float(y.abs().max()) == 0.0
    # one sample less fits (28 MiB) and runs
    ns = 7
    y_ref, y_sta = _both(plan, l, data["x"][:ns])
    assert np.array_equal(y_ref, y_sta)
    plan.destroy()
