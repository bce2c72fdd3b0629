"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by element.

Tolerances (max|y - ref| / max|ref| per layer): fp32 1e-5, fp16 2e-2, integer paths bit-exact."""
import numpy as np
import pytest

from paper_2112_15445_amd import binding as B
from paper_2112_15445_amd import workloads as wl

import gpu_util as G

pytestmark = pytest.mark.gpu

DT = ["f32", "f16", "i8", "cb4", "cb4h"]


def _both_variants(plan):
    """Yield a label for every kernel family that can run this plan (after installing it)."""
    for variant, extra in ((B.SC_VARIANT_GATHER, {}), (B.SC_VARIANT_SLAB, {"wsrc": 0}),
                           (B.SC_VARIANT_SLAB, {"wsrc": 1}), (B.SC_VARIANT_SLAB, {"wsrc": 2}),
                           (B.SC_VARIANT_SLAB, {"wsrc": 3}),
                           (B.SC_VARIANT_SLAB, {"wsrc": 3, "pipeline": 1, "wg_threads": 512}),
                           (B.SC_VARIANT_SLAB, {"wsrc": 1, "pipeline": 1, "wg_threads": 512, "chunk_c": 5,
                                                "tile_q": 128}),
                           (B.SC_VARIANT_SLAB, {"wsrc": 1, "pipeline": 1, "wg_threads": 256, "chunk_c": 8,
                                                "tile_d": 4, "tile_q": 64, "producers": 1}),
                           (B.SC_VARIANT_SLAB, {"wsrc": 1, "pipeline": 1, "wg_threads": 512, "producers": 1}),
                           (B.SC_VARIANT_SLAB, {"wsrc": 2, "pipeline": 1, "wg_threads": 512, "producers": 4}),
                           (B.SC_VARIANT_SLAB, {"wsrc": 1, "chunk_c": 2, "wg_threads": 256}),
                           (B.SC_VARIANT_SLAB, {"wsrc": 1, "chunk_c": 3, "tile_d": 4, "wg_threads": 128, "tile_p": 2,
                                                "tile_q": 1000}),
                           (B.SC_VARIANT_SLAB, {"wsrc": 1, "chunk_c": 3, "tile_d": 4, "wg_threads": 256, "tile_p": 3,
                                                "tile_q": 16, "sub_batch": 2}),
                           (B.SC_VARIANT_SLAB, {"wsrc": 1, "chunk_c": 2, "wg_threads": 128, "tile_p": 4,
                                                "tile_q": 8, "sub_batch": 3}),
                           (B.SC_VARIANT_SLAB, {"wsrc": 3, "chunk_c": 2, "wg_threads": 256}),
                           (B.SC_VARIANT_SLAB, {"wsrc": 3, "chunk_c": 3, "tile_d": 4, "wg_threads": 128, "tile_p": 2,
                                                "tile_q": 1000}),
                           (B.SC_VARIANT_SLAB, {"wsrc": 3, "chunk_c": 3, "tile_d": 4, "wg_threads": 256, "tile_p": 3,
                                                "tile_q": 16, "sub_batch": 2}),
                           (B.SC_VARIANT_SLAB, {"wsrc": 1, "chunk_c": 2, "wg_threads": 256, "pack": 1}),
                           (B.SC_VARIANT_SLAB, {"wsrc": 1, "chunk_c": 3, "tile_d": 4, "wg_threads": 128, "tile_p": 2,
                                                "tile_q": 1000, "pack": 1}),
                           (B.SC_VARIANT_SLAB, {"wsrc": 1, "chunk_c": 64, "tile_d": 3, "wg_threads": 64, "tile_p": 5,
                                                "tile_q": 37, "pack": 1}),
                           (B.SC_VARIANT_SLAB, {"wsrc": 1, "pipeline": 1, "wg_threads": 512, "chunk_c": 5,
                                                "tile_q": 128, "pack": 1}),
                           (B.SC_VARIANT_SLAB, {"wsrc": 1, "pipeline": 2, "wg_threads": 192, "chunk_c": 7,
                                                "tile_q": 64, "tile_d": 5, "pack": 1}),
                           (B.SC_VARIANT_SLAB, {"wsrc": 1, "chunk_c": 2, "wg_threads": 256, "pack": 2}),
                           (B.SC_VARIANT_SLAB, {"wsrc": 1, "chunk_c": 3, "tile_d": 4, "wg_threads": 128, "tile_p": 2,
                                                "tile_q": 1000, "pack": 2}),
                           (B.SC_VARIANT_SLAB, {"wsrc": 1, "pipeline": 1, "wg_threads": 512, "chunk_c": 5,
                                                "tile_q": 128, "pack": 2}),
                           (B.SC_VARIANT_SLAB, {"wsrc": 1, "pipeline": 2, "wg_threads": 192, "chunk_c": 7,
                                                "tile_q": 64, "tile_d": 5, "pack": 2}),
                           (B.SC_VARIANT_SLAB, {"wsrc": 1, "pipeline": 2, "wg_threads": 1024}),
                           (B.SC_VARIANT_SLAB, {"wsrc": 1, "pipeline": 2, "wg_threads": 192, "tile_q": 64}),
                           (B.SC_VARIANT_SLAB, {"wsrc": 1, "pipeline": 2, "wg_threads": 448, "tile_q": 96}),
                           (B.SC_VARIANT_DENSE, {}),
                           (B.SC_VARIANT_DENSE, {"tile_d": 32, "tile_p": 1, "wg_per_cu": 4, "waves_m": 1}),
                           (B.SC_VARIANT_DENSE, {"tile_d": 32, "tile_p": 2, "chunk_c": 64}),
                           (B.SC_VARIANT_DENSE, {"tile_d": 64, "tile_p": 1000, "sub_batch": 2}),
                           (B.SC_VARIANT_DENSE, {"tile_d": 128, "tile_p": 3, "wg_per_cu": 1})):
        try:
            plan.set_tuning(B.sc_tuning_t(), variant=variant, **extra)
        except B.SparseConvError as e:
            assert e.status == 4      # does not fit / not available for this dtype
            continue
        yield f"variant={variant} {extra}"


@pytest.mark.parametrize("dtype", DT)
def test_config1_layer(dtype):
    (l,) = wl.config1()
    l = l.replace(dtype=dtype)
    data = wl.prepare(l)
    ref = G.oracle_out(l, data)
    plan = G.make_plan(l, data)
    assert plan.info().n == 58
    for label in _both_variants(plan):
        print("case", l.name, dtype, label, flush=True)
        G.check(l, G.run_gpu(plan, data["x"]), ref, label)


def test_stretch_pass_offsets_match_oracle():
    import oracle
    for l in (wl.config1()[0], wl.Layer("t", 5, 7, 9, 11, 3, 2, 2, 1, 1, 2, N=1, sparsity=0.5)):
        data = wl.prepare(l, ragged=True)
        st = oracle.sparse_conv_steps(data["x"], data["rowptr"], data["colidx"], data["values"], l.R,
                                      l.S, (l.stride_h, l.stride_w), (l.pad_h, l.pad_w))
        plan = G.make_plan(l, data)
        lam = plan.debug_offsets()
        assert lam.shape == st["lam"].shape and np.array_equal(lam, st["lam"])


SHAPES = [
    # name, C, D, H, W, R, S, sh, sw, ph, pw, N, sparsity
    ("odd_3x3", 5, 7, 13, 11, 3, 3, 1, 1, 1, 1, 3, 0.6),
    ("stride2_3x3", 6, 5, 14, 15, 3, 3, 2, 2, 1, 1, 2, 0.7),
    ("stride2_nopad", 4, 6, 9, 10, 3, 3, 2, 2, 0, 0, 2, 0.5),
    ("pad2_5x5", 3, 4, 8, 9, 5, 5, 1, 1, 2, 2, 2, 0.8),
    ("rect_filter", 4, 5, 10, 12, 2, 3, 1, 2, 0, 1, 2, 0.5),
    ("pointwise", 24, 10, 7, 9, 1, 1, 1, 1, 0, 0, 3, 0.7),
    ("pointwise_vec", 16, 12, 8, 8, 1, 1, 1, 1, 0, 0, 2, 0.6),
    ("pointwise_s2", 8, 6, 9, 9, 1, 1, 2, 2, 0, 0, 2, 0.5),
    ("conv1d_like", 30, 8, 1, 64, 1, 3, 1, 1, 0, 0, 2, 0.8),
    ("stride3", 3, 4, 11, 13, 3, 3, 3, 3, 1, 1, 2, 0.5),
    ("wide_tiles", 2, 3, 6, 150, 3, 3, 1, 1, 1, 1, 1, 0.5),
]


@pytest.mark.parametrize("dtype", DT)
@pytest.mark.parametrize("shape", SHAPES, ids=[s[0] for s in SHAPES])
def test_shapes_both_variants(shape, dtype):
    name, C, D, H, W, R, S, sh, sw, ph, pw, N, sp = shape
    l = wl.Layer(name, C, D, H, W, R, S, sh, sw, ph, pw, N=N, sparsity=sp, dtype=dtype, seed=4242)
    data = wl.prepare(l)
    ref = G.oracle_out(l, data)
    plan = G.make_plan(l, data)
    ran = 0
    for label in _both_variants(plan):
        print("case", name, dtype, label, flush=True)
        G.check(l, G.run_gpu(plan, data["x"]), ref, f"{name} {label}")
        ran += 1
    assert ran >= 1


@pytest.mark.parametrize("dtype", DT)
def test_ragged_rows_empty_rows_and_extremes(dtype):
    base = wl.Layer("ragged", 6, 9, 10, 9, 3, 3, 1, 1, 1, 1, N=2, sparsity=0.6, dtype=dtype, seed=99)
    cases = {
        "ragged": wl.prepare(base, ragged=True),
        "n=1": wl.prepare(base, n=1),
        "n=K (0% sparsity)": wl.prepare(base, n=base.K),
    }
    # a table with empty rows
    d = wl.prepare(base, ragged=True)
    rp = d["rowptr"].copy()
    keep = np.ones(rp[-1], bool)
    for row in (0, 4):
        keep[rp[row]:rp[row + 1]] = False
    lens = np.diff(rp)
    lens[[0, 4]] = 0
    d["rowptr"] = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    d["colidx"], d["values"] = d["colidx"][keep], d["values"][keep]
    cases["empty rows"] = d
    for what, data in cases.items():
        ref = G.oracle_out(base, data)
        plan = G.make_plan(base, data)
        for label in _both_variants(plan):
            print("case", what, dtype, label, flush=True)
            G.check(base, G.run_gpu(plan, data["x"]), ref, f"{what} {label}")


@pytest.mark.parametrize("dtype", ["f32", "i8"])
def test_all_zero_table_gives_zero_output(dtype):
    l = wl.Layer("empty", 3, 4, 6, 6, 3, 3, 1, 1, 1, 1, N=2, dtype=dtype)
    data = wl.prepare(l, n=0)
    assert data["rowptr"][-1] == 0
    plan = G.make_plan(l, data)
    assert plan.info().n == 0
    for label in _both_variants(plan):
        y = G.run_gpu(plan, data["x"])
        assert y.shape == (2, 4, 6, 6) and not np.any(y), label


@pytest.mark.parametrize("dtype", ["f32", "cb4", "cb4h"])
def test_long_rows_are_chunked(dtype):
    """n larger than one LDS weight stage / one gather row chunk (dense 3x3 over 160 channels)."""
    l = wl.Layer("long", 160, 6, 6, 6, 3, 3, 1, 1, 1, 1, N=1, sparsity=0.0, dtype=dtype, seed=5)
    data = wl.prepare(l)
    assert l.n == 1440
    ref = G.oracle_out(l, data)
    plan = G.make_plan(l, data)
    for label in _both_variants(plan):
        print("case long", dtype, label, flush=True)
        G.check(l, G.run_gpu(plan, data["x"]), ref, label)


@pytest.mark.parametrize("dtype", DT)
def test_wavefront_split_reduction(dtype):
    """Few output positions (batch 1, 3x3 plane): the stored entries of one output are split over
    4 / 16 / 64 lanes and combined by the wavefront-level shuffle reduction."""
    l = wl.Layer("split", 40, 9, 5, 5, 3, 3, 1, 1, 0, 0, N=1, sparsity=0.5, dtype=dtype, seed=77)
    data = wl.prepare(l)
    ref = G.oracle_out(l, data)
    plan = G.make_plan(l, data)
    for ns in (1, 4, 16, 64):
        for sb in (1, 2, 8):
            plan.set_tuning(B.sc_tuning_t(), variant=B.SC_VARIANT_GATHER, split_n=ns, sub_batch=sb)
            t = plan.get_tuning()
            assert (t.split_n, t.sub_batch) == (ns, sb)
            G.check(l, G.run_gpu(plan, data["x"]), ref, f"split_n={ns} sub_batch={sb}")


@pytest.mark.parametrize("dtype", ["f32", "f16", "i8"])
def test_channel_chunked_pipeline(dtype):
    """Pointwise layer through the channel-chunked persistent kernel: chunk sizes that do and do not
    divide C, output-channel blocks, many tiles per workgroup, ragged rows."""
    l = wl.Layer("chunked", 40, 24, 12, 12, 1, 1, 1, 1, 0, 0, N=50, sparsity=0.6, dtype=dtype, seed=5)
    data = wl.prepare(l, ragged=True)
    ref = G.oracle_out(l, data)
    plan = G.make_plan(l, data)
    ran = 0
    for thr, tq, cc, td, npd in ((512, 64, 8, 0, 2), (1024, 128, 16, 16, 2), (1024, 144, 33, 0, 1),
                                 (512, 144, 7, 10, 4), (256, 64, 40, 0, 1)):
        try:
            plan.set_tuning(B.sc_tuning_t(), variant=B.SC_VARIANT_SLAB, wsrc=1, pipeline=1, wg_threads=thr,
                            tile_q=tq, chunk_c=cc, tile_d=td, producers=npd)
        except B.SparseConvError as e:
            assert e.status == 4
            continue
        t = plan.get_tuning()
        assert t.chunk_c == min(cc, 40) and t.pipeline == 1
        G.check(l, G.run_gpu(plan, data["x"]), ref, str(t.as_dict()))
        ran += 1
    assert ran >= 3


@pytest.mark.parametrize("dtype", ["f32", "f16", "i8"])
@pytest.mark.parametrize("D", [24, 10, 1])
def test_symmetric_pipeline(dtype, D):
    """Pointwise layer through the persistent kernel in which every wave copies and multiplies: more
    tiles than workgroups, row counts that do and do not divide the wave count (including waves
    without rows), ragged rows, odd and tiny row lengths, a tile tail."""
    l = wl.Layer("sym", 40, D, 16, 16, 1, 1, 1, 1, 0, 0, N=70, sparsity=0.6, dtype=dtype, seed=7)
    ran = 0
    for n, ragged in ((None, True), (1, False), (3, False)):
        data = wl.prepare(l, n=n, ragged=ragged)
        ref = G.oracle_out(l, data)
        plan = G.make_plan(l, data)
        for thr, tq, cc, td in ((64, 32, 0, 0), (320, 64, 0, 0), (1024, 48, 0, 0), (1024, 128, 0, 0),
                                (704, 256, 0, 0), (1024, 128, 16, 0), (256, 256, 7, 0), (128, 64, 20, 8),
                                (512, 192, 33, 0)):
            try:
                plan.set_tuning(B.sc_tuning_t(), variant=B.SC_VARIANT_SLAB, wsrc=1, pipeline=2,
                                wg_threads=thr, tile_q=tq, chunk_c=cc, tile_d=td)
            except B.SparseConvError as e:
                assert e.status == 4
                continue
            t = plan.get_tuning()
            assert t.pipeline == 2 and t.producers == 0
            G.check(l, G.run_gpu(plan, data["x"]), ref, f"n={n} {t.as_dict()}")
            ran += 1
    assert ran >= 15


@pytest.mark.parametrize("dtype", ["f16", "i8"])
def test_packed_positions_in_the_producer_consumer_kernel(dtype):
    """16- and 8-bit activations through the persistent kernel whose lanes own 2 / 4 adjacent
    positions per LDS dword: one to four dwords per lane, a ragged last tile, ragged rows."""
    l = wl.Layer("packed", 24, 20, 24, 24, 1, 1, 1, 1, 0, 0, N=40, sparsity=0.5, dtype=dtype, seed=13)
    data = wl.prepare(l, ragged=True)
    ref = G.oracle_out(l, data)
    plan = G.make_plan(l, data)
    ran = 0
    for thr, tq, npd in ((1024, 128, 2), (512, 256, 1), (1024, 512, 4), (768, 192, 1), (1024, 64, 2)):
        try:
            plan.set_tuning(B.sc_tuning_t(), variant=B.SC_VARIANT_SLAB, wsrc=1, pipeline=1,
                            wg_threads=thr, tile_q=tq, producers=npd)
        except B.SparseConvError as e:
            assert e.status == 4
            continue
        G.check(l, G.run_gpu(plan, data["x"]), ref, str(plan.get_tuning().as_dict()))
        ran += 1
    assert ran >= 4


@pytest.mark.parametrize("dtype", ["f32", "f16", "i8"])
def test_symmetric_pipeline_rows_not_16_byte_aligned(dtype):
    """7x7 planes (49 elements per channel row): fp32 rows are only 4-byte aligned, so the symmetric
    kernels copy 4 bytes per lane; fp16 / int8 rows of odd length cannot be copied that way and the
    tuning must be refused."""
    l = wl.Layer("sym7", 72, 40, 7, 7, 1, 1, 1, 1, 0, 0, N=9, sparsity=0.7, dtype=dtype, seed=11)
    data = wl.prepare(l, ragged=True)
    ref = G.oracle_out(l, data)
    plan = G.make_plan(l, data)
    ran = 0
    for thr, tq, cc, td in ((1024, 64, 0, 0), (384, 49, 24, 0), (512, 32, 16, 16), (1024, 64, 36, 8)):
        try:
            plan.set_tuning(B.sc_tuning_t(), variant=B.SC_VARIANT_SLAB, wsrc=1, pipeline=2,
                            wg_threads=thr, tile_q=tq, chunk_c=cc, tile_d=td)
        except B.SparseConvError as e:
            assert e.status == 4
            continue
        G.check(l, G.run_gpu(plan, data["x"]), ref, str(plan.get_tuning().as_dict()))
        ran += 1
    assert ran == (4 if dtype == "f32" else 0)


def test_ell_entry_point_and_unsorted_duplicate_columns():
    rng = np.random.default_rng(3)
    l = wl.Layer("ell", 4, 5, 8, 8, 3, 3, 1, 1, 1, 1, N=2, dtype="i8")
    n = 7
    col = rng.integers(0, l.K, size=(l.D, n)).astype(np.int32)       # unsorted, duplicates likely
    col[:, 3] = col[:, 2]
    val = rng.integers(-127, 128, size=(l.D, n)).astype(np.int8)
    x = rng.integers(-127, 128, size=(2, 4, 8, 8)).astype(np.int8)
    import oracle
    rp = (np.arange(l.D + 1) * n).astype(np.int32)
    ref = oracle.sparse_conv(x, rp, col.ravel(), val.ravel(), 3, 3, (1, 1), (1, 1))
    plan = B.Plan.create_ell(G.layer_desc(l), B.SC_I8, n, col, val, scales=np.ones(l.D, np.float32))
    for label in _both_variants(plan):
        assert np.array_equal(G.run_gpu(plan, x), ref), label


@pytest.mark.parametrize("dtype", ["f32", "f16", "i8"])
def test_every_autotune_candidate_on_mid_size_layers(dtype):
    """Layers large enough for the wide-tile, channel-chunked, packed and pipelined candidates to
    fit (planes of 1024 and 784 positions, 96 / 160 input channels, a stride-2 layer): every
    candidate the autotuner would time gives the oracle's result."""
    for l in (wl.Layer("mid1x1", 96, 80, 32, 32, 1, 1, 1, 1, 0, 0, N=3, sparsity=0.85, dtype=dtype, seed=18),
              wl.Layer("mid3x3", 160, 48, 28, 28, 3, 3, 1, 1, 1, 1, N=2, sparsity=0.9, dtype=dtype, seed=19),
              wl.Layer("mid3x3s2", 48, 40, 28, 28, 3, 3, 2, 2, 1, 1, N=2, sparsity=0.8, dtype=dtype, seed=20)):
        data = wl.prepare(l, ragged=True)
        ref = G.oracle_out(l, data)
        plan = G.make_plan(l, data)
        nc = plan.num_candidates()
        kinds = set()
        for i in range(nc):
            t = plan.candidate(i)
            plan.set_tuning(t)
            d = t.as_dict()
            kinds.add((d["variant"], d["pipeline"], d["chunk_c"] > 0, d["pack"], d["wsrc"], d["sub_batch"] > 1))
            G.check(l, G.run_gpu(plan, data["x"]), ref, f"{l.name} candidate {i} {d}")
        print("case", l.name, dtype, nc, "candidates,", len(kinds), "kinds", flush=True)
        assert nc >= 50 and len(kinds) >= 6


def test_every_autotune_candidate_gives_the_same_answer():
    for l in (wl.Layer("cand3x3", 16, 24, 20, 20, 3, 3, 1, 1, 1, 1, N=3, sparsity=0.8, seed=8),
              wl.Layer("cand1x1", 32, 40, 16, 16, 1, 1, 1, 1, 0, 0, N=3, sparsity=0.8, seed=9)):
        data = wl.prepare(l)
        ref = G.oracle_out(l, data)
        plan = G.make_plan(l, data)
        nc = plan.num_candidates()
        assert nc >= 8
        for i in range(nc):
            t = plan.candidate(i)
            plan.set_tuning(t)
            print("candidate", l.name, i, t.as_dict(), flush=True)
            G.check(l, G.run_gpu(plan, data["x"]), ref, f"{l.name} candidate {i} {t.as_dict()}")


def test_autotune_installs_a_valid_tuning():
    import torch
    l = wl.Layer("tune", 32, 32, 28, 28, 3, 3, 1, 1, 1, 1, N=4, sparsity=0.9, seed=10)
    data = wl.prepare(l)
    ref = G.oracle_out(l, data)
    plan = G.make_plan(l, data)
    x = G.to_device(data["x"])
    y = torch.empty((4, 32, 28, 28), device="cuda")
    ws = torch.empty(max(plan.workspace_size_max(4), 1), dtype=torch.uint8, device="cuda")
    plan.autotune(x.data_ptr(), y.data_ptr(), 4, ws.data_ptr(), ws.numel(),
                  torch.cuda.current_stream().cuda_stream)
    t = plan.get_tuning()
    assert t.variant in (B.SC_VARIANT_GATHER, B.SC_VARIANT_SLAB)
    G.check(l, G.run_gpu(plan, data["x"]), ref, str(t.as_dict()))
    assert plan.info().grid_size > 0


@pytest.mark.parametrize("cfg,dtype", [(2, "f32"), (5, "i8"), (5, "cb4"), (7, "cb4h")])
def test_vgg_stack_layers_at_reduced_batch(cfg, dtype):
    layers = [l for l in wl.CONFIGS[cfg]() if l.dtype == dtype]
    assert len(layers) == 13
    for l in layers:
        data = wl.prepare(l, N=2)
        ref = G.oracle_out(l, data)
        plan = G.make_plan(l, data)
        print("case", l.name, plan.get_tuning().as_dict(), flush=True)
        G.check(l, G.run_gpu(plan, data["x"]), ref, l.name)


@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_resnet_layers_full_batch_sampled(dtype):
    """Full-size ResNet-50-shaped layers (batch 32, 90 %) in the default launch configuration;
    the oracle checks the first and last sample completely."""
    layers = [l for l in wl.config3() if l.name.endswith("sp90")]
    for l in layers:
        l = l.replace(dtype=dtype)
        data = wl.prepare(l)
        plan = G.make_plan(l, data)
        print("case", l.name, dtype, plan.get_tuning().as_dict(), flush=True)
        y = G.run_gpu(plan, data["x"])
        for b in (0, l.N - 1):
            ref = G.oracle_out(l, data, samples=[b])
            G.check(l, y[b:b + 1], ref, f"{l.name} sample {b}")


def test_headline_layer_full_size_as_benchmarked():
    """The benchmark's layer at full size in the launch shape the benchmark times: autotuned, then
    the oracle checks the first and the last sample completely; also the three persistent kernel
    families pinned explicitly."""
    import torch
    l = wl.headline_layer()
    data = wl.prepare(l)
    plan = G.make_plan(l, data)
    x = G.to_device(data["x"])
    y = torch.empty((l.N, l.D, l.P, l.Q), device="cuda")
    ws = torch.empty(max(plan.workspace_size_max(l.N), 1), dtype=torch.uint8, device="cuda")
    plan.autotune(x.data_ptr(), y.data_ptr(), l.N, ws.data_ptr(), ws.numel(),
                  torch.cuda.current_stream().cuda_stream)
    refs = {b: G.oracle_out(l, data, samples=[b]) for b in (0, l.N - 1)}
    tuned = plan.get_tuning().as_dict()
    print("autotuned", tuned, flush=True)
    assert tuned["variant"] == B.SC_VARIANT_SLAB and tuned["pipeline"] >= 1
    y = G.run_gpu(plan, data["x"])
    for b, ref in refs.items():
        G.check(l, y[b:b + 1], ref, f"autotuned {tuned} sample {b}")
    for extra in ({"pipeline": 1, "producers": 1, "tile_q": 64}, {"pipeline": 2, "tile_q": 64},
                  {"pipeline": 1, "producers": 2, "tile_q": 256, "chunk_c": 64},
                  {"pipeline": 2, "tile_q": 128, "chunk_c": 128}):
        plan.set_tuning(B.sc_tuning_t(), variant=B.SC_VARIANT_SLAB, wsrc=1, wg_threads=1024, **extra)
        y = G.run_gpu(plan, data["x"])
        for b, ref in refs.items():
            G.check(l, y[b:b + 1], ref, f"{extra} sample {b}")


@pytest.mark.parametrize("name,extra", [
    ("s28_conv3x3_s2_sp90", {"tile_p": 4, "chunk_c": 64, "wg_per_cu": 1}),
    ("s14_conv3x3_sp90", {"tile_p": 7, "chunk_c": 128, "tile_d": 128, "wg_per_cu": 2}),
    ("s7_conv3x3_sp90", {"tile_p": 7, "chunk_c": 64, "tile_d": 128, "sub_batch": 2}),
    ("s7_expand1x1_sp90", {"tile_p": 1, "tile_q": 49, "chunk_c": 128, "tile_d": 128, "sub_batch": 4, "wg_per_cu": 1}),
    ("s14_reduce1x1_sp90", {"tile_p": 1, "tile_q": 128, "chunk_c": 128, "tile_d": 128, "pipeline": 2}),
    ("s7_reduce1x1_sp90", {"tile_p": 1, "tile_q": 49, "chunk_c": 768, "tile_d": 64, "wg_per_cu": 1}),
    ("s7_conv3x3_sp80", {"tile_p": 7, "chunk_c": 192, "tile_d": 32, "sub_batch": 2, "wg_per_cu": 1}),
    ("s7_conv3x3_sp80", {"tile_p": 7, "chunk_c": 64, "tile_d": 16, "wg_per_cu": 1, "pack": 3}),
    ("s56_conv3x3_sp80", {"tile_p": 2, "chunk_c": 32, "tile_d": 64, "wg_per_cu": 1, "pack": 3}),
    ("s14_conv3x3_s2_sp90", {"tile_p": 4, "chunk_c": 32, "tile_d": 32, "wg_per_cu": 1, "pack": 3}),
])
def test_full_size_layers_through_the_chunked_kernels(name, extra):
    """Full-size ResNet-50-shaped layers (batch 32) through the channel-chunked kernels with
    output-channel blocks, several samples per workgroup and samples interleaved in the LDS word;
    first and last sample checked."""
    l = {x.name: x for x in wl.config3()}[name]
    data = wl.prepare(l)
    plan = G.make_plan(l, data)
    plan.set_tuning(B.sc_tuning_t(), variant=B.SC_VARIANT_SLAB, wsrc=1, wg_threads=1024, **extra)
    t = plan.get_tuning().as_dict()
    assert t["chunk_c"] == extra["chunk_c"]
    y = G.run_gpu(plan, data["x"])
    for b in (0, l.N - 1):
        G.check(l, y[b:b + 1], G.oracle_out(l, data, samples=[b]), f"{name} {t} sample {b}")


@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_one_dimensional_convolution_workload(dtype):
    """The 1-D convolution layers (300 channels, length 64, kernels 2 and 3, batch 128) at full
    size, autotuned; the oracle checks three samples completely."""
    import torch
    for l in [x for x in wl.config6() if x.dtype == dtype]:
        data = wl.prepare(l)
        plan = G.make_plan(l, data)
        x = G.to_device(data["x"])
        y = torch.empty((l.N, l.D, l.P, l.Q), device="cuda", dtype=B.torch_out_dtype(plan.dtype))
        ws = torch.empty(max(plan.workspace_size_max(l.N), 1), dtype=torch.uint8, device="cuda")
        plan.autotune(x.data_ptr(), y.data_ptr(), l.N, ws.data_ptr(), ws.numel(),
                      torch.cuda.current_stream().cuda_stream)
        t = plan.get_tuning().as_dict()
        print("case", l.name, t, flush=True)
        out = G.run_gpu(plan, data["x"])
        for b in (0, 77, l.N - 1):
            G.check(l, out[b:b + 1], G.oracle_out(l, data, samples=[b]), f"{l.name} {t} sample {b}")


@pytest.mark.parametrize("dtype", ["f32", "f16", "i8"])
def test_ragged_table_option_matches_the_unified_result(dtype):
    """Rows of different lengths walked over their own entries only (tuning.ragged = 1, the filler
    entries left out of the per-chunk segments) through the three chunked kernels: the result is
    the oracle's, as for the unified table."""
    for l in (wl.Layer("rag3x3", 20, 36, 14, 14, 3, 3, 2, 2, 1, 1, N=5, sparsity=0.7, dtype=dtype, seed=21),
              wl.Layer("rag1x1", 48, 24, 16, 16, 1, 1, 1, 1, 0, 0, N=9, sparsity=0.6, dtype=dtype, seed=22)):
        data = wl.prepare(l, ragged=True)
        ref = G.oracle_out(l, data)
        plan = G.make_plan(l, data)
        ran = 0
        for extra in ({"chunk_c": 6, "tile_p": 4, "tile_d": 16}, {"chunk_c": 16, "tile_p": 2, "sub_batch": 2},
                      {"chunk_c": 16, "pipeline": 1, "tile_q": 128, "producers": 1},
                      {"chunk_c": 12, "pipeline": 2, "tile_q": 64, "tile_d": 8}):
            for ragged in (0, 1):
                try:
                    plan.set_tuning(B.sc_tuning_t(), variant=B.SC_VARIANT_SLAB, wsrc=1, wg_threads=512,
                                    ragged=ragged, **extra)
                except B.SparseConvError as e:
                    assert e.status == 4
                    continue
                t = plan.get_tuning().as_dict()
                assert t["ragged"] == ragged
                G.check(l, G.run_gpu(plan, data["x"]), ref, f"{l.name} {t}")
                ran += 1
        assert ran >= 4


@pytest.mark.parametrize("dtype", ["f16", "i8"])
def test_packed_positions_in_the_chunked_one_shot_kernel(dtype):
    """tuning.pack = 1: a lane owns the 2 (f16) or 4 (i8) adjacent positions of one 32-bit word of the
    staged tile.  Filter taps make the word start at any element (odd offsets), tiles end in the
    middle of a word, stride phases and padding are in play, and tiles of 1..4 words per lane."""
    for l, tunings in (
            (wl.Layer("pk3x3", 20, 24, 28, 28, 3, 3, 1, 1, 1, 1, N=3, sparsity=0.8, dtype=dtype, seed=31),
             [{"tile_p": 4, "chunk_c": 8}, {"tile_p": 7, "chunk_c": 20, "tile_d": 8}, {"tile_p": 16, "chunk_c": 4},
              {"tile_p": 2, "chunk_c": 16, "wg_per_cu": 3}]),
            (wl.Layer("pk3x3s2", 12, 10, 29, 27, 3, 3, 2, 2, 1, 1, N=2, sparsity=0.7, dtype=dtype, seed=32),
             [{"tile_p": 4, "chunk_c": 5}, {"tile_p": 14, "chunk_c": 12}]),
            (wl.Layer("pk1x1", 96, 40, 14, 14, 1, 1, 1, 1, 0, 0, N=5, sparsity=0.9, dtype=dtype, seed=33),
             [{"tile_q": 64, "chunk_c": 32}, {"tile_q": 200, "chunk_c": 16, "tile_d": 16}, {"tile_q": 512, "chunk_c": 64}]),
            (wl.Layer("pk5x1", 9, 6, 40, 7, 5, 1, 1, 1, 2, 0, N=2, sparsity=0.5, dtype=dtype, seed=34),
             [{"tile_p": 9, "chunk_c": 4}])):
        data = wl.prepare(l, ragged=True)
        ref = G.oracle_out(l, data)
        plan = G.make_plan(l, data)
        for extra in tunings:
            plan.set_tuning(B.sc_tuning_t(), variant=B.SC_VARIANT_SLAB, wsrc=1, wg_threads=512, pack=1, **extra)
            t = plan.get_tuning().as_dict()
            assert t["pack"] == 1
            print("case", l.name, dtype, t, flush=True)
            G.check(l, G.run_gpu(plan, data["x"]), ref, f"{l.name} {t}")
    # the pipelined chunked kernels of the pointwise layers (rows and tiles are whole words there)
    l = wl.Layer("pk1x1p", 72, 50, 20, 28, 1, 1, 1, 1, 0, 0, N=4, sparsity=0.8, dtype=dtype, seed=36)
    data = wl.prepare(l, ragged=True)
    ref = G.oracle_out(l, data)
    plan = G.make_plan(l, data)
    for extra in ({"pipeline": 1, "tile_q": 128, "chunk_c": 16, "producers": 1},
                  {"pipeline": 1, "tile_q": 512, "chunk_c": 24, "tile_d": 32, "producers": 2},
                  {"pipeline": 2, "tile_q": 256, "chunk_c": 32}, {"pipeline": 2, "tile_q": 64, "chunk_c": 9, "tile_d": 24},
                  {"pipeline": 2, "tile_q": 384, "chunk_c": 16, "ragged": 1}):
        plan.set_tuning(B.sc_tuning_t(), variant=B.SC_VARIANT_SLAB, wsrc=1, wg_threads=1024, pack=1, **extra)
        t = plan.get_tuning().as_dict()
        assert t["pack"] == 1 and t["pipeline"] == extra["pipeline"]
        print("case", l.name, dtype, t, flush=True)
        G.check(l, G.run_gpu(plan, data["x"]), ref, f"{l.name} {t}")
    # not for 32-bit activations
    l = wl.Layer("pkf32", 8, 8, 8, 8, 1, 1, 1, 1, 0, 0, N=2, sparsity=0.5, dtype="f32", seed=35)
    plan = G.make_plan(l, wl.prepare(l))
    for extra in ({"chunk_c": 4}, ):
        with pytest.raises(B.SparseConvError):
            plan.set_tuning(B.sc_tuning_t(), variant=B.SC_VARIANT_SLAB, wsrc=1, pack=1, **extra)


@pytest.mark.parametrize("dtype", ["f32", "f16", "i8"])
def test_lane_distributed_weights_in_the_chunked_one_shot_kernel(dtype):
    """tuning.wsrc = 3 with chunk_c > 0: segments longer than one batch of 64 entries, empty segments,
    rows of uneven length (with and without the fillers), one and several samples per workgroup."""
    for l, tunings in (
            (wl.Layer("ln1x1", 320, 40, 7, 7, 1, 1, 1, 1, 0, 0, N=6, sparsity=0.3, dtype=dtype, seed=41),
             [{"chunk_c": 160, "tile_q": 49, "sub_batch": 4}, {"chunk_c": 100, "tile_q": 49, "tile_d": 16, "sub_batch": 2},
              {"chunk_c": 64, "tile_q": 49, "ragged": 1}]),
            (wl.Layer("ln3x3", 24, 20, 14, 14, 3, 3, 1, 1, 1, 1, N=3, sparsity=0.5, dtype=dtype, seed=42),
             [{"chunk_c": 24, "tile_p": 7}, {"chunk_c": 5, "tile_p": 4, "tile_d": 8}, {"chunk_c": 12, "tile_p": 14, "ragged": 1}])):
        data = wl.prepare(l, ragged=True)
        ref = G.oracle_out(l, data)
        plan = G.make_plan(l, data)
        for extra in tunings:
            plan.set_tuning(B.sc_tuning_t(), variant=B.SC_VARIANT_SLAB, wsrc=3, wg_threads=512, wg_per_cu=1, **extra)
            t = plan.get_tuning().as_dict()
            assert t["wsrc"] == 3 and t["chunk_c"] > 0
            print("case", l.name, dtype, t, flush=True)
            G.check(l, G.run_gpu(plan, data["x"]), ref, f"{l.name} {t}")


@pytest.mark.parametrize("dtype", ["f32", "f16", "i8"])
def test_pointwise_whole_plane_tiles_staged_as_a_plain_copy(dtype):
    """Pointwise layer, one tile per plane, chunk images that are 16-byte aligned blocks of the input:
    the chunked one-shot kernel copies them with 16-byte loads.  7x7 and 14x14 planes, a last chunk
    with fewer channels, one and several samples per workgroup, a batch that does not divide."""
    for l, tunings in (
            (wl.Layer("flat7", 72, 24, 7, 7, 1, 1, 1, 1, 0, 0, N=5, sparsity=0.8, dtype=dtype, seed=51),
             [{"chunk_c": 16, "tile_q": 49}, {"chunk_c": 32, "tile_q": 49, "sub_batch": 2},
              {"chunk_c": 16, "tile_q": 49, "sub_batch": 4, "tile_d": 8}]),
            (wl.Layer("flat14", 40, 20, 14, 14, 1, 1, 1, 1, 0, 0, N=3, sparsity=0.7, dtype=dtype, seed=52),
             [{"chunk_c": 8, "tile_q": 196}, {"chunk_c": 40, "tile_q": 256, "tile_d": 8}] +
             ([{"chunk_c": 8, "tile_q": 196, "pack": 2, "tile_d": 8}] if dtype == "f32" else []) +
             ([{"chunk_c": 16, "tile_q": 196, "pack": 1}] if dtype != "f32" else []))):
        data = wl.prepare(l, ragged=True)
        ref = G.oracle_out(l, data)
        plan = G.make_plan(l, data)
        for extra in tunings:
            plan.set_tuning(B.sc_tuning_t(), variant=B.SC_VARIANT_SLAB, wsrc=1, wg_threads=512, wg_per_cu=1, **extra)
            t = plan.get_tuning().as_dict()
            assert t["tile_q"] == l.H * l.W and t["chunk_c"] == extra["chunk_c"]
            print("case", l.name, dtype, t, flush=True)
            G.check(l, G.run_gpu(plan, data["x"]), ref, f"{l.name} {t}")


@pytest.mark.parametrize("dtype", ["f32", "f16", "i8"])
def test_full_width_tiles_staged_by_row_runs(dtype):
    """Unit strides and tiles as wide as the plane: the chunked one-shot kernel copies whole input rows
    with 4-, 8- or 16-byte loads and writes the zero padding once.  Widths that give each load size
    (and one that gives none), paddings 0..2, tiles that end below the plane, packed positions."""
    shapes = [("rr56", 12, 10, 13, 56, 3, 3, 1, 1, 1), ("rr24", 10, 12, 9, 24, 3, 3, 1, 1, 1), ("rr20", 9, 8, 11, 20, 5, 5, 2, 2, 1),
              ("rr12", 16, 6, 12, 12, 3, 3, 0, 0, 1), ("rr8", 20, 9, 8, 8, 1, 3, 0, 1, 1), ("rr14", 7, 5, 14, 14, 3, 3, 1, 1, 1),
              ("rr10", 6, 5, 10, 10, 3, 3, 2, 1, 1),
              # strides of two: rows and columns split by parity into the four phase images
              ("rs56", 10, 8, 30, 56, 3, 3, 1, 1, 2), ("rs24", 12, 10, 17, 24, 3, 3, 0, 0, 2), ("rs16", 8, 6, 16, 16, 2, 2, 0, 0, 2),
              ("rs20", 6, 7, 19, 20, 5, 5, 2, 2, 2), ("rs12", 9, 5, 12, 12, 3, 3, 1, 1, 2)]
    for name, C, D, H, W, R, S, ph, pw, st in shapes:
        l = wl.Layer(name, C, D, H, W, R, S, st, st, ph, pw, N=3, sparsity=0.6, dtype=dtype, seed=61)
        data = wl.prepare(l, ragged=True)
        ref = G.oracle_out(l, data)
        plan = G.make_plan(l, data)
        ran = 0
        for extra in ({"tile_p": 4, "chunk_c": 3}, {"tile_p": 3, "chunk_c": 64, "tile_d": 4},
                      {"tile_p": 5, "chunk_c": 4, "pack": 1}, {"tile_p": 8, "chunk_c": 2, "pack": 1, "tile_d": 3}):
            try:
                plan.set_tuning(B.sc_tuning_t(), variant=B.SC_VARIANT_SLAB, wsrc=1, wg_threads=256, wg_per_cu=1,
                                tile_q=10000, **extra)
            except B.SparseConvError as e:
                assert e.status == 4 and extra.get("pack") and dtype == "f32"    # packing: 16- and 8-bit only
                continue
            t = plan.get_tuning().as_dict()
            print("case", name, dtype, t, flush=True)
            G.check(l, G.run_gpu(plan, data["x"]), ref, f"{name} {t}")
            ran += 1
        assert ran >= 2


@pytest.mark.parametrize("name,extra", [
    ("s56_conv3x3_sp80", {"tile_p": 7, "chunk_c": 64, "wg_per_cu": 1, "pack": 1}),
    ("s28_conv3x3_sp80", {"tile_p": 7, "chunk_c": 128, "tile_d": 64, "wg_per_cu": 1, "pack": 1}),
    ("s14_conv3x3_s2_sp90", {"tile_p": 7, "chunk_c": 64, "tile_d": 64, "wg_per_cu": 1, "pack": 1}),
    ("s28_reduce1x1_sp80", {"pipeline": 1, "producers": 1, "tile_q": 256, "chunk_c": 128, "tile_d": 64, "pack": 1}),
    ("s14_reduce1x1_sp90", {"pipeline": 2, "tile_q": 128, "chunk_c": 256, "tile_d": 64, "pack": 1}),
    ("s7_reduce1x1_sp90", {"tile_q": 49, "chunk_c": 256, "tile_d": 32, "sub_batch": 2, "wg_per_cu": 1}),
    ("s7_expand1x1_sp90", {"tile_q": 49, "chunk_c": 256, "tile_d": 64, "sub_batch": 4, "wg_per_cu": 1, "wsrc": 3}),
    ("s7_reduce1x1_sp80", {"tile_q": 49, "chunk_c": 768, "tile_d": 32, "sub_batch": 2, "wg_per_cu": 1}),
    ("s7_expand1x1_sp80", {"tile_q": 49, "chunk_c": 256, "tile_d": 64, "sub_batch": 4, "wg_per_cu": 1, "pack": 1}),
])
def test_full_size_half_precision_layers_packed_and_small_plane_forms(name, extra):
    """Full-size ResNet-50-shaped fp16 layers (batch 32) in the launch shapes the per-layer report
    picks: packed positions (shifted images on the 3x3 layers, row-run staging where the tile spans
    the plane), whole-plane copies, lane-distributed weights, chunks of 768 channels and the planes
    of four samples end to end in one packed tile on the 7x7 layers.  First and last sample checked
    completely against the oracle."""
    l = {x.name: x for x in wl.config4()}[name]
    data = wl.prepare(l)
    plan = G.make_plan(l, data)
    plan.set_tuning(B.sc_tuning_t(), variant=B.SC_VARIANT_SLAB, wg_threads=1024, **{"wsrc": 1, **extra})
    t = plan.get_tuning().as_dict()
    assert t["chunk_c"] == extra["chunk_c"] and t["pack"] == extra.get("pack", 0)
    y = G.run_gpu(plan, data["x"])
    for b in (0, l.N - 1):
        G.check(l, y[b:b + 1], G.oracle_out(l, data, samples=[b]), f"{name} {t} sample {b}")


def test_power_of_two_quantised_layer_is_bit_exact():
    """The paper's linear quantiser (per-tensor power-of-two step, activations saturated at 0.99)
    applied by the library's plan-time helper, then the int8 path: same codes as the oracle's
    quantiser, same int32 outputs as the oracle's convolution of those codes."""
    import oracle
    l = wl.Layer("pow2", 48, 40, 14, 14, 3, 3, 1, 1, 1, 1, N=4, sparsity=0.85, dtype="f32", seed=71)
    data = wl.prepare(l)
    wq, wf = B.quantize_pow2(data["values"], 8)
    xq, xf = B.quantize_pow2(data["x"], 8, 0.99)
    wo, wfo = oracle.quantise_pow2(data["values"], 8)
    xo, xfo = oracle.quantise_pow2(data["x"], 8, 0.99)
    assert (wf, xf) == (wfo, xfo) == (9, 7) and np.array_equal(wq, wo) and np.array_equal(xq, xo)
    li = l.replace(dtype="i8")
    qd = dict(data, values=wq, x=xq, scales=np.full(l.D, 2.0 ** -wf, np.float32), codebook=None)
    ref = G.oracle_out(li, qd)
    assert ref.dtype == np.int32 and np.any(ref)
    plan = G.make_plan(li, qd)
    for label in _both_variants(plan):
        G.check(li, G.run_gpu(plan, xq), ref, label)
    # dequantised, the result is the fp32 layer's up to the quantisation noise
    y = ref.astype(np.float64) * 2.0 ** -(wf + xf)
    yf = G.oracle_out(l, data).astype(np.float64)
    assert np.max(np.abs(y - yf)) / np.max(np.abs(yf)) < 0.05


@pytest.mark.parametrize("dtype", ["f32", "f16", "i8"])
def test_autotune_and_forward_with_unaligned_device_pointers(dtype):
    """x and y that start one element into their allocations: the launch shapes that need 16-byte
    aligned rows are skipped by the autotuner (forward reports them as unsupported instead of
    launching), and the shape it installs gives the oracle's result."""
    import torch
    l = wl.Layer("unal", 32, 24, 16, 16, 1, 1, 1, 1, 0, 0, N=6, sparsity=0.7, dtype=dtype, seed=81)
    data = wl.prepare(l)
    ref = G.oracle_out(l, data)
    plan = G.make_plan(l, data)
    x0 = G.to_device(data["x"])
    xbuf = torch.empty(x0.numel() + 8, dtype=x0.dtype, device="cuda")
    x = xbuf[1:1 + x0.numel()].view(x0.shape)
    x.copy_(x0)
    ybuf = torch.full((l.N * l.D * l.P * l.Q + 8,), 7, dtype=B.torch_out_dtype(plan.dtype), device="cuda")
    y = ybuf[1:1 + l.N * l.D * l.P * l.Q].view(l.N, l.D, l.P, l.Q)
    assert x.data_ptr() % 16 != 0 and y.data_ptr() % 16 != 0
    ws = torch.empty(max(plan.workspace_size_max(l.N), 16), dtype=torch.uint8, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    plan.autotune(x.data_ptr(), y.data_ptr(), l.N, ws.data_ptr(), ws.numel(), st)
    t = plan.get_tuning().as_dict()
    print("case unaligned", dtype, t, flush=True)
    plan.forward(x.data_ptr(), y.data_ptr(), l.N, ws.data_ptr(), ws.numel(), st)
    torch.cuda.synchronize()
    G.check(l, G.to_host(y), ref, f"unaligned {t}")
    assert int(ybuf[0]) == 7 and int(ybuf[-1]) == 7          # nothing written outside y
    # a pipelined shape asked for explicitly installs, but forward refuses these pointers
    plan.set_tuning(B.sc_tuning_t(), variant=B.SC_VARIANT_SLAB, wsrc=1, wg_threads=512, pipeline=2, tile_q=64, chunk_c=8)
    with pytest.raises(B.SparseConvError) as e:
        plan.forward(x.data_ptr(), y.data_ptr(), l.N, ws.data_ptr(), ws.numel(), st)
    assert e.value.status == 4


@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_positions_packed_in_128_bit_words(dtype):
    """tuning.pack = 2: a lane owns the 4 (f32) or 8 (f16) adjacent positions of one 128-bit word, read
    with one LDS instruction.  Pointwise layers through the one-shot and both pipelined chunked
    kernels (tiles of one and two words per lane, ragged last tile, output-channel blocks), other
    layers through the one-shot kernel with its shifted images (odd offsets, strides, padding)."""
    cases = (
        (wl.Layer("w1x1", 72, 50, 20, 28, 1, 1, 1, 1, 0, 0, N=4, sparsity=0.8, dtype=dtype, seed=91),
         [{"tile_q": 256}, {"tile_q": 512, "wg_threads": 256}, {"tile_q": 128, "wg_per_cu": 2},
          {"chunk_c": 16, "tile_q": 256}, {"chunk_c": 24, "tile_q": 512, "tile_d": 16}, {"chunk_c": 72, "tile_q": 128},
          {"pipeline": 1, "tile_q": 256, "producers": 1}, {"pipeline": 1, "tile_q": 512, "producers": 2},
          {"pipeline": 1, "tile_q": 256, "chunk_c": 16, "producers": 1},
          {"pipeline": 1, "tile_q": 512, "chunk_c": 24, "tile_d": 32, "producers": 2},
          {"pipeline": 2, "tile_q": 256, "chunk_c": 32}, {"pipeline": 2, "tile_q": 128, "chunk_c": 9, "tile_d": 24},
          {"pipeline": 2, "tile_q": 512, "chunk_c": 16, "ragged": 1}]),
        (wl.Layer("w3x3", 20, 24, 28, 28, 3, 3, 1, 1, 1, 1, N=3, sparsity=0.8, dtype=dtype, seed=92),
         [{"tile_p": 4, "chunk_c": 4}, {"tile_p": 8, "chunk_c": 5, "tile_d": 8}, {"tile_p": 2, "chunk_c": 8, "wg_per_cu": 2}]),
        (wl.Layer("w3x3s2", 12, 10, 29, 27, 3, 3, 2, 2, 1, 1, N=2, sparsity=0.7, dtype=dtype, seed=93),
         [{"tile_p": 4, "chunk_c": 3}, {"tile_p": 14, "chunk_c": 4}]),
        (wl.Layer("w1x1odd", 40, 12, 7, 7, 1, 1, 1, 1, 0, 0, N=5, sparsity=0.6, dtype=dtype, seed=94),
         [{"tile_q": 49, "chunk_c": 8}]))
    for l, tunings in cases:
        data = wl.prepare(l, ragged=True)
        ref = G.oracle_out(l, data)
        plan = G.make_plan(l, data)
        ran = 0
        for extra in tunings:
            try:
                plan.set_tuning(B.sc_tuning_t(), variant=B.SC_VARIANT_SLAB, wsrc=1, pack=2,
                                **{"wg_per_cu": 1, "wg_threads": 1024, **extra})
            except B.SparseConvError as e:
                assert e.status == 4
                print("does not fit", l.name, dtype, extra, flush=True)
                continue
            t = plan.get_tuning().as_dict()
            assert t["pack"] == 2 and t["pipeline"] == extra.get("pipeline", 0)
            print("case", l.name, dtype, t, flush=True)
            G.check(l, G.run_gpu(plan, data["x"]), ref, f"{l.name} {t}")
            ran += 1
        assert ran >= 1, l.name


def test_autotune_takes_the_ragged_table_when_rows_are_uneven():
    """Rows with uniform lengths in [0, n] (about half of the unified table is fillers): the
    autotuner's candidates include the chunked shapes with the fillers left out, it installs one of
    them, and the result is the oracle's.  A table with equal rows gets no such candidates."""
    import torch
    l = wl.Layer("ragtune", 128, 64, 28, 28, 3, 3, 1, 1, 1, 1, N=4, sparsity=0.8, seed=95)
    even = G.make_plan(l, wl.prepare(l))
    assert not any(even.candidate(i).ragged for i in range(even.num_candidates()))
    data = wl.prepare(l, ragged=True)
    ref = G.oracle_out(l, data)
    plan = G.make_plan(l, data)
    assert any(plan.candidate(i).ragged for i in range(plan.num_candidates()))
    x = G.to_device(data["x"])
    y = torch.empty((l.N, l.D, l.P, l.Q), device="cuda")
    ws = torch.empty(max(plan.workspace_size_max(l.N), 1), dtype=torch.uint8, device="cuda")
    plan.autotune(x.data_ptr(), y.data_ptr(), l.N, ws.data_ptr(), ws.numel(), torch.cuda.current_stream().cuda_stream)
    t = plan.get_tuning().as_dict()
    print("case ragtune", t, flush=True)
    assert t["ragged"] == 1
    G.check(l, G.run_gpu(plan, data["x"]), ref, str(t))


@pytest.mark.parametrize("dtype", ["f32", "f16", "i8"])
def test_samples_laid_end_to_end_in_one_packed_tile(dtype):
    """Pointwise layers with small planes: sub_batch samples end to end along the position axis of
    one packed tile.  7x7, 5x3 and 14x14 planes (channel pitches that need rounding up to a word),
    batches that leave a short last group, a last chunk with fewer channels, output-channel blocks,
    one and two slots per lane, 32- and 128-bit words."""
    packs = {"f32": [2], "f16": [1, 2], "i8": [1]}[dtype]
    for l, shapes in (
            (wl.Layer("e2e7", 72, 24, 7, 7, 1, 1, 1, 1, 0, 0, N=11, sparsity=0.8, dtype=dtype, seed=61),
             [{"sub_batch": 2, "chunk_c": 16}, {"sub_batch": 4, "chunk_c": 32, "tile_d": 8},
              {"sub_batch": 5, "chunk_c": 72}, {"sub_batch": 10, "chunk_c": 16, "tile_d": 16}]),
            (wl.Layer("e2e53", 33, 10, 5, 3, 1, 1, 1, 1, 0, 0, N=9, sparsity=0.6, dtype=dtype, seed=62),
             [{"sub_batch": 3, "chunk_c": 8}, {"sub_batch": 16, "chunk_c": 16}]),
            (wl.Layer("e2e14", 40, 20, 14, 14, 1, 1, 1, 1, 0, 0, N=3, sparsity=0.7, dtype=dtype, seed=63),
             [{"sub_batch": 2, "chunk_c": 8, "tile_d": 8}])):
        data = wl.prepare(l, ragged=True)
        ref = G.oracle_out(l, data)
        plan = G.make_plan(l, data)
        for extra in shapes:
            for pack in packs:
                plan.set_tuning(B.sc_tuning_t(), variant=B.SC_VARIANT_SLAB, wsrc=1, wg_threads=256, wg_per_cu=1,
                                tile_q=l.H * l.W, pack=pack, **extra)
                t = plan.get_tuning().as_dict()
                assert t["sub_batch"] == extra["sub_batch"] and t["pack"] == pack and t["chunk_c"] == extra["chunk_c"]
                print("case", l.name, dtype, t, flush=True)
                G.check(l, G.run_gpu(plan, data["x"]), ref, f"{l.name} {t}")


@pytest.mark.parametrize("dtype", ["f32", "f16", "i8"])
def test_samples_interleaved_in_the_lds_word(dtype):
    """tuning.pack = 3: an LDS word holds the same position of 4 (f32, i8) or 8 (f16) consecutive
    samples, so the wide reads work on any layer shape.  3x3 with padding, stride 2, a 1x3 filter, a
    pointwise layer; batches that leave a short last group (and one smaller than a word); a last
    chunk with fewer channels; one and two slots per lane; output-channel blocks."""
    for l, shapes in (
            (wl.Layer("si3x3", 40, 24, 7, 7, 3, 3, 1, 1, 1, 1, N=11, sparsity=0.8, dtype=dtype, seed=71),
             [{"tile_p": 7, "chunk_c": 16}, {"tile_p": 7, "chunk_c": 8, "tile_d": 8}, {"tile_p": 3, "chunk_c": 40}]),
            (wl.Layer("si14", 24, 12, 14, 14, 3, 3, 1, 1, 1, 1, N=5, sparsity=0.7, dtype=dtype, seed=72),
             [{"tile_p": 4, "chunk_c": 8}] + ([{"tile_p": 8, "chunk_c": 8, "tile_d": 4}] if dtype != "f16" else [])),
            (wl.Layer("sis2", 20, 16, 15, 13, 3, 3, 2, 2, 1, 1, N=3, sparsity=0.6, dtype=dtype, seed=73),
             [{"tile_p": 4, "chunk_c": 8}, {"tile_p": 8, "chunk_c": 4}]),
            (wl.Layer("si1x3", 30, 10, 1, 40, 1, 3, 1, 1, 0, 1, N=9, sparsity=0.5, dtype=dtype, seed=74),
             [{"tile_p": 1, "chunk_c": 16}]),
            (wl.Layer("sipw", 32, 16, 6, 5, 1, 1, 1, 1, 0, 0, N=6, sparsity=0.5, dtype=dtype, seed=75),
             [{"tile_p": 1, "tile_q": 30, "chunk_c": 8}])):
        data = wl.prepare(l, ragged=True)
        ref = G.oracle_out(l, data)
        plan = G.make_plan(l, data)
        for extra in shapes:
            plan.set_tuning(B.sc_tuning_t(), variant=B.SC_VARIANT_SLAB, wsrc=1, wg_threads=256, wg_per_cu=1,
                            pack=3, **{"tile_q": l.Q if l.R * l.S > 1 else l.H * l.W, **extra})
            t = plan.get_tuning().as_dict()
            assert t["pack"] == 3 and t["chunk_c"] == extra["chunk_c"]
            print("case", l.name, dtype, t, flush=True)
            G.check(l, G.run_gpu(plan, data["x"]), ref, f"{l.name} {t}")


@pytest.mark.parametrize("dtype", ["f16", "i8", "cb4", "cb4h"])
def test_dense_variant_on_the_matrix_cores(dtype):
    """The densified tile (MFMA) against the oracle: several channel blocks and LDS chunks, output
    channels that do not fill a 16-row block, batches that do not fill a sample group, strides,
    paddings, rectangular filters; integer dtypes bit-exact."""
    shapes = [("deep_3x3", 150, 70, 9, 11, 3, 3, 1, 1, 1, 1, 5, 0.8),
              ("deep_pointwise", 200, 37, 7, 7, 1, 1, 1, 1, 0, 0, 7, 0.7),
              ("stride2", 70, 20, 13, 12, 3, 3, 2, 2, 1, 1, 3, 0.5),
              ("rect_pad", 40, 130, 6, 17, 2, 3, 1, 2, 0, 2, 2, 0.6),
              ("tiny_plane", 96, 48, 2, 2, 3, 3, 1, 1, 1, 1, 19, 0.9),
              ("one_step", 24, 40, 9, 8, 1, 1, 1, 1, 0, 0, 3, 0.5)]      # one channel block, one tap: a single step
    for name, C, D, H, W, R, S, sh, sw, ph, pw, N, sp in shapes:
        l = wl.Layer(name, C, D, H, W, R, S, sh, sw, ph, pw, N=N, sparsity=sp, dtype=dtype, seed=777)
        data = wl.prepare(l)
        ref = G.oracle_out(l, data)
        plan = G.make_plan(l, data)
        ran = piped = 0
        for extra in ({}, {"tile_d": 16}, {"tile_d": 32, "tile_p": 1}, {"tile_d": 64, "tile_p": 2, "chunk_c": 64},
                      {"tile_d": 128, "wg_per_cu": 1}, {"tile_d": 64, "tile_p": 1000, "sub_batch": 4},
                      {"tile_d": 128, "waves_m": 2, "tile_p": 2}, {"tile_d": 128, "waves_m": 4}, {"tile_d": 64, "waves_m": 1, "tile_p": 3},
                      {"tile_d": 64, "waves_m": 2, "chunk_c": 64},
                      {"tile_d": 32, "waves_m": 2, "tile_p": 1000, "sub_batch": 3},
                      {"tile_d": 32, "tile_p": 1000, "sub_batch": 16, "chunk_c": 128, "wg_per_cu": 1},
                      # several blocks of output channels per workgroup, one after the other on the resident tile
                      {"tile_d": 16, "split_n": 2}, {"tile_d": 32, "tile_p": 2, "split_n": 3}, {"tile_d": 16, "tile_p": 1, "split_n": 16},
                      {"tile_d": 64, "waves_m": 2, "split_n": 2, "tile_p": 1000, "sub_batch": 2}):
            # four waves, and eight (two groups that split the steps of the contraction and meet in LDS);
            # one-shot staging, and the pipelined form (staging waves of their own, two chunk buffers)
            cb = 64 if dtype in ("i8", "cb4") else 32
            for threads in (256, 512):
                for pipe in ({}, {"pipeline": 1}, {"pipeline": 1, "producers": 4, "chunk_c": cb}, {"pipeline": 1, "producers": 1, "chunk_c": 3 * cb}):
                    if pipe and "chunk_c" in extra and "chunk_c" in pipe:
                        continue
                    kw = {**extra, **pipe}
                    try:
                        plan.set_tuning(B.sc_tuning_t(), variant=B.SC_VARIANT_DENSE, wg_threads=threads, **kw)
                    except B.SparseConvError as e:
                        assert e.status == 4
                        continue
                    t = plan.get_tuning()
                    assert t.variant == B.SC_VARIANT_DENSE and t.wg_threads == threads and t.pipeline == pipe.get("pipeline", 0)
                    assert t.producers == (pipe.get("producers", 2) if pipe else 0)
                    print("case dense", name, dtype, t.as_dict(), flush=True)
                    G.check(l, G.run_gpu(plan, data["x"]), ref, f"{name} dense {kw} {threads}")
                    ran += 1
                    piped += 1 if pipe else 0
        assert ran >= 6 and piped >= 6, (name, ran, piped)
        plan.destroy()


def test_dense_variant_is_refused_where_it_does_not_apply():
    l = wl.Layer("refuse", 8, 4, 6, 6, N=1, sparsity=0.5, dtype="f32", seed=5)
    data = wl.prepare(l)
    plan = G.make_plan(l, data)
    with pytest.raises(B.SparseConvError) as e:
        plan.set_tuning(B.sc_tuning_t(), variant=B.SC_VARIANT_DENSE)       # 32-bit activations
    assert e.value.status == 4
    plan.destroy()
    # a column stored twice in one row adds up in the gather kernels; it has no exact dense image
    l = l.replace(dtype="i8")
    data = wl.prepare(l)
    rp, ci, va = data["rowptr"], data["colidx"].copy(), data["values"]
    ci[rp[1] + 1] = ci[rp[1]]
    plan = B.Plan.create_csr(G.layer_desc(l), B.DTYPES["i8"], rp, ci, va, data["scales"], None)
    before = plan.get_tuning().as_dict()
    with pytest.raises(B.SparseConvError) as e:
        plan.set_tuning(B.sc_tuning_t(), variant=B.SC_VARIANT_DENSE)
    assert e.value.status == 4 and plan.get_tuning().as_dict() == before
    plan.destroy()


@pytest.mark.parametrize("dtype,sparsity", [("f16", 0.5), ("f32", 0.9), ("i8", 0.8)])
def test_per_layer_dispatch_records_three_contenders_and_forward_honours_the_choice(dtype, sparsity):
    """sparse_conv_plan_dispatch: the gather kernels, the densified MFMA tile and the dense library timed
    on one layer; every contender that was available gives the oracle's result through
    sparse_conv_forward."""
    import torch
    l = wl.Layer("dispatch", 96, 80, 14, 14, 3, 3, 1, 1, 1, 1, N=8, sparsity=sparsity, dtype=dtype, seed=31)
    data = wl.prepare(l)
    ref = G.oracle_out(l, data)
    plan = G.make_plan(l, data)
    with pytest.raises(B.SparseConvError) as e:
        plan.set_path(B.SC_PATH_SPARSE)                      # nothing measured yet
    assert e.value.status == 4
    xd = G.to_device(data["x"])
    y = torch.empty((l.N, l.D, l.P, l.Q), dtype=B.torch_out_dtype(plan.dtype), device="cuda")
    ws = torch.empty(plan.autotune_workspace_size(l.N), dtype=torch.uint8, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    rec = plan.dispatch(xd.data_ptr(), y.data_ptr(), l.N, ws.data_ptr(), ws.numel(), st)
    print("dispatch", dtype, rec.as_dict(), flush=True)
    assert rec.sparse_ms > 0
    assert (rec.dense_ms > 0) == (dtype != "f32")
    if dtype == "i8":
        assert rec.library_ms < 0                            # the dense library is used for floating point only
    times = {B.SC_PATH_SPARSE: rec.sparse_ms}
    if rec.dense_ms > 0:
        times[B.SC_PATH_DENSE] = rec.dense_ms
    best = min(times, key=times.get)
    assert rec.choice in (best, B.SC_PATH_LIBRARY)
    if rec.choice == B.SC_PATH_LIBRARY:
        assert 0 < rec.library_ms < 0.9 * times[best]

    def run():
        y.view(torch.uint8).fill_(0x7f)
        need = plan.workspace_size(l.N)
        w2 = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")
        plan.forward(xd.data_ptr(), y.data_ptr(), l.N, w2.data_ptr(), w2.numel(), st)
        torch.cuda.synchronize()
        return G.to_host(y)

    if rec.choice != B.SC_PATH_LIBRARY:
        G.check(l, run(), ref, f"dispatch {dtype}: installed choice {rec.choice}")
    for path in (B.SC_PATH_SPARSE, B.SC_PATH_DENSE, B.SC_PATH_LIBRARY):
        try:
            plan.set_path(path)
        except B.SparseConvError as e:
            assert e.status == 4
            assert path != B.SC_PATH_SPARSE
            continue
        print("case dispatch path", dtype, path, flush=True)
        if path == B.SC_PATH_LIBRARY:
            # the dense library picks its own algorithm (possibly a transform-domain one): its
            # rounding is its own, so this leg is held to 1e-3 (fp32) / 2e-2 (fp16), not to the
            # library's own kernels' 1e-5
            got = run()
            assert G.rel_err(got, ref) <= (1e-3 if dtype == "f32" else 2e-2), G.rel_err(got, ref)
        else:
            G.check(l, run(), ref, f"dispatch {dtype}: path {path}")
    plan.destroy()


def _run_epi(plan, l, x, out_np_dtype):
    import torch
    inf = plan.info()
    xd = G.to_device(np.ascontiguousarray(x))
    tdt = {np.int8: torch.int8, np.int32: torch.int32, np.float16: torch.float16, np.float32: torch.float32}[out_np_dtype]
    y = torch.empty((x.shape[0], l.D, inf.out_P, inf.out_Q), dtype=tdt, device="cuda")
    y.view(torch.uint8).fill_(0x7f)
    assert inf.out_elem_bytes == y.element_size()
    need = plan.workspace_size(x.shape[0])
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")
    plan.forward(xd.data_ptr(), y.data_ptr(), x.shape[0], ws.data_ptr(), ws.numel(), torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    return G.to_host(y)


@pytest.mark.parametrize("dtype", DT)
def test_fused_epilogue_relu_pool_requantise(dtype):
    """ReLU / 2x2 max-pool / requantisation fused into the store of the GATHER and DENSE kernels,
    against the oracle's epilogue applied to the oracle's accumulators; requantised codes bit-exact."""
    import oracle
    shapes = [("even", 20, 24, 8, 12, 3, 3, 1, 1, 1, 1, 5, 0.6),
              ("odd_plane", 40, 36, 7, 9, 3, 3, 1, 1, 1, 1, 3, 0.7),
              ("pointwise", 70, 18, 6, 6, 1, 1, 1, 1, 0, 0, 4, 0.5),
              ("stride2", 12, 20, 13, 11, 3, 3, 2, 2, 1, 1, 2, 0.5),
              ("tiny", 96, 33, 2, 2, 3, 3, 1, 1, 1, 1, 9, 0.9)]
    integer = dtype in ("i8", "cb4")
    rng = np.random.default_rng(3)
    for name, C, D, H, W, R, S, sh, sw, ph, pw, N, sp in shapes:
        l = wl.Layer(name, C, D, H, W, R, S, sh, sw, ph, pw, N=N, sparsity=sp, dtype=dtype, seed=123)
        data = wl.prepare(l)
        acc = oracle.sparse_conv_steps(data["x"], data["rowptr"], data["colidx"], data["values"], R, S, (sh, sw), (ph, pw),
                                       codebook=data["codebook"])["y"]
        plan = G.make_plan(l, data)
        # multipliers that spread the codes over the int8 range
        rq = (100.0 / max(1.0, float(np.abs(acc).max())) * (0.5 + rng.random(D))).astype(np.float32)
        for relu, pool, requant in ((1, 0, 0), (0, 2, 0), (1, 2, 0), (1, 2, 1), (0, 0, 1), (1, 0, 1)):
            if requant and not integer:
                with pytest.raises(B.SparseConvError) as e:
                    plan.set_epilogue(relu=relu, pool=pool, requant_scale=rq)
                assert e.value.status == 4
                continue
            plan.set_epilogue(relu=relu, pool=pool, requant_scale=rq if requant else None)
            out_dt = np.int8 if requant else G.NP_OUT[dtype]
            ref = oracle.epilogue(acc, relu=bool(relu), pool=pool, requant_scale=rq if requant else None,
                                  out_dtype=None if requant else G.NP_OUT[dtype])
            with pytest.raises(B.SparseConvError) as e:
                plan.set_tuning(B.sc_tuning_t(), variant=B.SC_VARIANT_SLAB, wsrc=0)      # no epilogue in the slab kernels
            assert e.value.status == 4
            ran = 0
            for variant, extra in ((B.SC_VARIANT_GATHER, {}), (B.SC_VARIANT_GATHER, {"sub_batch": 2}),
                                   (B.SC_VARIANT_DENSE, {}), (B.SC_VARIANT_DENSE, {"tile_d": 32, "tile_p": 2}),
                                   (B.SC_VARIANT_DENSE, {"tile_d": 64, "tile_p": 1000, "sub_batch": 3, "waves_m": 2}),
                                   (B.SC_VARIANT_DENSE, {"tile_d": 128, "tile_p": 4, "waves_m": 4, "chunk_c": 64}),
                                   (B.SC_VARIANT_DENSE, {"wg_threads": 512}), (B.SC_VARIANT_DENSE, {"tile_d": 32, "tile_p": 2, "wg_threads": 512}),
                                   (B.SC_VARIANT_DENSE, {"tile_d": 64, "tile_p": 1000, "sub_batch": 3, "waves_m": 2, "wg_threads": 512}),
                                   # the pipelined form: its staging waves are gone when the epilogue's barriers are met
                                   (B.SC_VARIANT_DENSE, {"pipeline": 1}), (B.SC_VARIANT_DENSE, {"pipeline": 1, "tile_d": 32, "tile_p": 2, "producers": 1}),
                                   (B.SC_VARIANT_DENSE, {"pipeline": 1, "tile_d": 64, "tile_p": 1000, "sub_batch": 3, "waves_m": 2, "wg_threads": 512, "producers": 4}),
                                   (B.SC_VARIANT_DENSE, {"pipeline": 1, "wg_threads": 512, "tile_p": 2, "producers": 3})):
                try:
                    plan.set_tuning(B.sc_tuning_t(), variant=variant, **extra)
                except B.SparseConvError as e:
                    assert e.status == 4
                    continue
                print("case epilogue", name, dtype, (relu, pool, requant), variant, extra, flush=True)
                got = _run_epi(plan, l, data["x"], out_dt)
                assert got.shape == ref.shape, (got.shape, ref.shape)
                if requant or integer:
                    assert np.array_equal(got, ref), (name, relu, pool, requant, variant, extra, np.count_nonzero(got != ref))
                else:
                    G.check(l, got, ref, f"{name} epilogue {(relu, pool)} {variant} {extra}")
                ran += 1
            assert ran >= 2 if dtype != "f32" else ran >= 1
        plan.set_epilogue()                                      # and back to the plain convolution
        G.check(l, G.run_gpu(plan, data["x"]), G.oracle_out(l, data), f"{name} epilogue removed")
        plan.destroy()


@pytest.mark.parametrize("dtype", ["i8", "cb4"])
def test_quantised_vgg_stack_chains_through_the_fused_epilogue(dtype):
    """The VGG-16-shaped stack at batch 4 as ONE chain: every layer's int8 output (ReLU, max-pool at
    the end of a stage, requantisation) is the next layer's input, on the GPU through the DENSE
    kernel (first layer: GATHER) and in the oracle; the codes agree bit for bit after 13 layers."""
    import oracle
    import torch
    layers = [l.replace(N=4) for l in wl.config5() if (l.dtype == dtype)]
    assert len(layers) == 13
    x_ref = wl.prepare(layers[0])["x"]
    x_gpu = G.to_device(x_ref)
    for k, l in enumerate(layers):
        data = wl.prepare(l)
        pool = 2 if (k + 1 < len(layers) and layers[k + 1].H * 2 == l.H) else 0
        acc = oracle.sparse_conv_steps(x_ref, data["rowptr"], data["colidx"], data["values"], l.R, l.S,
                                       (l.stride_h, l.stride_w), (l.pad_h, l.pad_w), codebook=data["codebook"])["y"]
        post = oracle.epilogue(acc, relu=True, pool=pool)
        rq = np.full(l.D, 120.0 / max(1.0, float(post.max())), dtype=np.float32)
        x_next_ref = oracle.epilogue(acc, relu=True, pool=pool, requant_scale=rq)
        plan = G.make_plan(l, data)
        plan.set_epilogue(relu=True, pool=pool, requant_scale=rq)
        try:
            plan.set_tuning(B.sc_tuning_t(), variant=B.SC_VARIANT_DENSE)
        except B.SparseConvError:
            plan.set_tuning(B.sc_tuning_t(), variant=B.SC_VARIANT_GATHER)
        inf = plan.info()
        y = torch.empty((l.N, l.D, inf.out_P, inf.out_Q), dtype=torch.int8, device="cuda")
        ws = torch.empty(max(plan.workspace_size(l.N), 16), dtype=torch.uint8, device="cuda")
        plan.forward(x_gpu.data_ptr(), y.data_ptr(), l.N, ws.data_ptr(), ws.numel(), torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        got = y.cpu().numpy()
        print("case chain", dtype, k, l.name, "variant", plan.get_tuning().variant, "pool", pool, got.shape, flush=True)
        assert np.array_equal(got, x_next_ref), (k, l.name, np.count_nonzero(got != x_next_ref))
        assert np.count_nonzero(got) > 0
        x_ref, x_gpu = x_next_ref, y
        plan.destroy()


@pytest.mark.parametrize("dtype", ["f32", "f16", "i8"])
def test_chunk_buffer_ring_of_the_producer_consumer_kernel(dtype):
    """tuning.buffers = 3 .. 5: a producer wave per chunk in flight, one barrier per phase; with tile
    widths whose rows are copied as whole instructions plus a partly filled one (not a power of two,
    not a multiple of an instruction), ragged last tiles, a last chunk with fewer channels, more
    workgroup units than workgroups, uneven rows, and the packed forms."""
    for l in (wl.Layer("ring_a", 72, 50, 20, 28, 1, 1, 1, 1, 0, 0, N=5, sparsity=0.8, dtype=dtype, seed=71),
              wl.Layer("ring_b", 40, 24, 28, 28, 1, 1, 1, 1, 0, 0, N=3, sparsity=0.9, dtype=dtype, seed=72)):
        data = wl.prepare(l, ragged=True)
        ref = G.oracle_out(l, data)
        plan = G.make_plan(l, data)
        words16 = 16 // {"f32": 4, "f16": 2, "i8": 1}[dtype]
        cases = [{"buffers": 3, "tile_q": 128, "chunk_c": 16}, {"buffers": 3, "tile_q": 392, "chunk_c": 24},
                 {"buffers": 4, "tile_q": 448, "chunk_c": 8, "tile_d": 16}, {"buffers": 5, "tile_q": 192, "chunk_c": 7},
                 {"buffers": 3, "producers": 2, "tile_q": 272, "chunk_c": 32, "wg_threads": 512, "tile_d": 24},
                 {"buffers": 0, "producers": 2, "tile_q": 448, "chunk_c": 16},      # the partial-row copies with two buffers
                 {"buffers": 0, "producers": 1, "tile_q": 400, "chunk_c": 24}]
        if dtype != "f32":
            cases += [{"buffers": 3, "tile_q": 384, "chunk_c": 16, "pack": 1}]
        if dtype != "i8":
            cases += [{"buffers": 3, "tile_q": 512, "chunk_c": 16, "pack": 2}, {"buffers": 4, "tile_q": 384 // words16 * words16, "chunk_c": 9, "pack": 2}]
        for extra in cases:
            kw = dict(variant=B.SC_VARIANT_SLAB, wsrc=1, pipeline=1, wg_threads=1024)
            kw.update(extra)
            kw["tile_q"] = -(-kw["tile_q"] // words16) * words16          # rows and tiles are whole 16-byte words
            plan.set_tuning(B.sc_tuning_t(), **kw)
            t = plan.get_tuning().as_dict()
            assert t["buffers"] == extra["buffers"] and (not t["buffers"] or t["producers"] == t["buffers"] - 1)
            print("case", l.name, dtype, t, flush=True)
            G.check(l, G.run_gpu(plan, data["x"]), ref, f"{l.name} {t}")
        # refused: without channel chunks, outside the producer/consumer form, producers that do not match
        for bad in ({"pipeline": 1, "buffers": 3}, {"pipeline": 2, "buffers": 3, "chunk_c": 16},
                    {"pipeline": 0, "buffers": 3, "chunk_c": 16}, {"pipeline": 1, "buffers": 3, "producers": 1, "chunk_c": 16},
                    {"pipeline": 1, "buffers": 6, "chunk_c": 16}, {"pipeline": 1, "buffers": 1, "chunk_c": 16}):
            with pytest.raises(B.SparseConvError):
                plan.set_tuning(B.sc_tuning_t(), variant=B.SC_VARIANT_SLAB, wsrc=1, wg_threads=1024, **bad)
        plan.destroy()


@pytest.mark.parametrize("dtype", ["f32", "f16", "i8"])
def test_sample_groups_along_the_lanes_with_interleaved_samples(dtype):
    """tuning.pack = 3 with tuning.sub_batch = 2 .. 8 on small planes: a workgroup takes that many groups
    of 4 (8 for f16) samples and numbers its lanes over (group, position).  Batches that end inside a
    word and inside a group, planes of 2 x 2 .. 5 x 3 with and without padding, stride 2, several
    chunks with a short last one, output-channel blocks that leave waves without rows; and the refusals."""
    cases = ((wl.Layer("sg2x2", 40, 24, 2, 2, 3, 3, 1, 1, 1, 1, N=37, sparsity=0.8, dtype=dtype, seed=81),
              [dict(tile_p=2, sub_batch=8, chunk_c=16, tile_d=8, wg_threads=256), dict(tile_p=2, sub_batch=4, chunk_c=40, wg_threads=512),
               dict(tile_p=1, sub_batch=2, chunk_c=7, tile_d=5, wg_threads=1024), dict(tile_p=2, sub_batch=3, chunk_c=24, tile_d=4, wg_threads=128)]),
             (wl.Layer("sg4x4", 24, 20, 4, 4, 3, 3, 1, 1, 1, 1, N=21, sparsity=0.7, dtype=dtype, seed=82),
              [dict(tile_p=4, sub_batch=2, chunk_c=8, tile_d=16, wg_threads=1024), dict(tile_p=2, sub_batch=5, chunk_c=24, wg_threads=256),
               dict(tile_p=1, sub_batch=8, chunk_c=5, tile_d=7, wg_threads=512)]),
             (wl.Layer("sg5x3s2", 16, 12, 9, 6, 3, 2, 2, 2, 1, 0, N=19, sparsity=0.6, dtype=dtype, seed=83),
              [dict(tile_p=5, sub_batch=2, chunk_c=6, wg_threads=256), dict(tile_p=2, sub_batch=4, chunk_c=16, tile_d=4, wg_threads=512)]),
             (wl.Layer("sg1x1", 32, 16, 3, 3, 1, 1, 1, 1, 0, 0, N=9, sparsity=0.5, dtype=dtype, seed=84),
              []))
    for l, tunings in cases:
        data = wl.prepare(l, ragged=True)
        ref = G.oracle_out(l, data)
        plan = G.make_plan(l, data)
        for extra in tunings:
            plan.set_tuning(B.sc_tuning_t(), variant=B.SC_VARIANT_SLAB, wsrc=1, pack=3, **extra)
            t = plan.get_tuning().as_dict()
            assert t["pack"] == 3 and t["sub_batch"] == extra["sub_batch"]
            print("case", l.name, dtype, t, flush=True)
            G.check(l, G.run_gpu(plan, data["x"]), ref, f"{l.name} {t}")
        # refused: groups that do not fit a wave, more than one slot per lane, too many groups
        for bad in (dict(tile_p=l.P, sub_batch=64 // max(l.P * (l.Q + (l.S - 1) // l.stride_w), 1) + 1, chunk_c=8),
                    dict(tile_p=1, sub_batch=9, chunk_c=8)):
            if bad["sub_batch"] > 1:
                with pytest.raises(B.SparseConvError):
                    plan.set_tuning(B.sc_tuning_t(), variant=B.SC_VARIANT_SLAB, wsrc=1, pack=3, **bad)
        plan.destroy()


@pytest.mark.parametrize("dtype", ["f32", "i8"])
def test_channel_chunks_dealt_to_several_workgroups(dtype):
    """tuning.split_n = 2 .. 16 on the chunked one-shot slab kernel: the chunks of a tile go to that many
    workgroups, which add their partial sums into y (cleared first) with atomic adds.  Splits that do
    not divide the number of chunks, a short last chunk, every staging form of that kernel (table, row
    runs, plain copy, interleaved samples with and without sample groups, several samples per
    workgroup, lane-distributed weights); y poisoned before every launch; int8 sums stay exact."""
    cases = ((wl.Layer("ks3x3", 40, 24, 9, 7, 3, 3, 1, 1, 1, 1, N=6, sparsity=0.7, dtype=dtype, seed=91),
              [dict(chunk_c=8, split_n=2, tile_p=3), dict(chunk_c=6, split_n=7, tile_p=9, tile_d=8),
               dict(chunk_c=4, split_n=10, tile_p=2, pack=3), dict(chunk_c=8, split_n=5, tile_p=1, pack=3, sub_batch=2, tile_d=16),
               dict(chunk_c=7, split_n=3, tile_p=4, sub_batch=2), dict(chunk_c=5, split_n=4, tile_p=3, wsrc=3)]),
             (wl.Layer("ks1x1", 96, 50, 7, 7, 1, 1, 1, 1, 0, 0, N=5, sparsity=0.8, dtype=dtype, seed=92),
              [dict(chunk_c=16, split_n=6, tile_q=49, wg_threads=1024), dict(chunk_c=32, split_n=3, tile_q=49, tile_d=16, sub_batch=2),
               dict(chunk_c=20, split_n=2, tile_q=32, wg_threads=512)]),
             (wl.Layer("ks3x3s2", 32, 20, 14, 14, 3, 3, 2, 2, 1, 1, N=5, sparsity=0.6, dtype=dtype, seed=93),
              [dict(chunk_c=8, split_n=4, tile_p=7), dict(chunk_c=4, split_n=8, tile_p=7, pack=3, tile_d=8)]))
    for l, tunings in cases:
        data = wl.prepare(l, ragged=True)
        ref = G.oracle_out(l, data)
        plan = G.make_plan(l, data)
        for extra in tunings:
            kw = dict(variant=B.SC_VARIANT_SLAB, wsrc=1, wg_threads=256)
            kw.update(extra)
            plan.set_tuning(B.sc_tuning_t(), **kw)
            t = plan.get_tuning().as_dict()
            assert t["split_n"] == extra["split_n"] and t["chunk_c"] == extra["chunk_c"]
            print("case", l.name, dtype, t, flush=True)
            for _ in range(2):                         # twice: the second launch finds y full of the first result
                G.check(l, G.run_gpu(plan, data["x"]), ref, f"{l.name} {t}")
        # refused: more workgroups than chunks, outside the chunked one-shot form, more than 16
        for bad in (dict(chunk_c=l.C, split_n=2), dict(chunk_c=8, split_n=17), dict(chunk_c=0, split_n=2)):
            with pytest.raises(B.SparseConvError):
                plan.set_tuning(B.sc_tuning_t(), variant=B.SC_VARIANT_SLAB, wsrc=1, wg_threads=256, **bad)
        plan.destroy()
    # 16-bit outputs cannot be added atomically with one rounding: refused
    l = wl.Layer("ksf16", 32, 16, 6, 6, 3, 3, 1, 1, 1, 1, N=2, sparsity=0.5, dtype="f16", seed=94)
    plan = G.make_plan(l, wl.prepare(l))
    with pytest.raises(B.SparseConvError):
        plan.set_tuning(B.sc_tuning_t(), variant=B.SC_VARIANT_SLAB, wsrc=1, chunk_c=8, split_n=2)
    plan.destroy()


def test_forward_captured_in_a_hip_graph_replays_correctly():
    """The forward path records kernels only (no memset, no allocation), so a caller may capture it:
    a gather-kernel shape with its padding pre-pass, a split-K shape with its clear kernel, and the
    matrix-core tile, each captured once and replayed three times with eager launches and
    synchronisations in between; every replay is checked against the oracle on poisoned outputs."""
    import torch
    cases = (("f32", dict(variant=B.SC_VARIANT_GATHER, sub_batch=2)),
             ("f32", dict(variant=B.SC_VARIANT_SLAB, wsrc=1, pack=3, chunk_c=8, split_n=3, tile_p=3, wg_threads=256)),
             ("i8", dict(variant=B.SC_VARIANT_SLAB, wsrc=1, chunk_c=8, split_n=2, tile_p=3, wg_threads=256)),
             ("f16", dict(variant=B.SC_VARIANT_DENSE, wg_threads=512)),
             ("i8", dict(variant=B.SC_VARIANT_DENSE, pipeline=1, producers=4, tile_p=3)))
    for dtype, tuning in cases:
        l = wl.Layer("graph", 40, 24, 9, 7, 3, 3, 1, 1, 1, 1, N=6, sparsity=0.7, dtype=dtype, seed=101)
        data = wl.prepare(l)
        ref = G.oracle_out(l, data)
        plan = G.make_plan(l, data)
        plan.set_tuning(B.sc_tuning_t(), **tuning)
        x = G.to_device(np.ascontiguousarray(data["x"]))
        inf = plan.info()
        y = torch.empty((l.N, l.D, inf.P, inf.Q), dtype=B.torch_out_dtype(plan.dtype), device="cuda")
        ws = torch.empty(max(plan.workspace_size(l.N), 16), dtype=torch.uint8, device="cuda")
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        g = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            plan.forward(x.data_ptr(), y.data_ptr(), l.N, ws.data_ptr(), ws.numel(), side.cuda_stream)   # warm-up outside capture
            side.synchronize()
            with torch.cuda.graph(g, stream=side):
                plan.forward(x.data_ptr(), y.data_ptr(), l.N, ws.data_ptr(), ws.numel(), side.cuda_stream)
        torch.cuda.synchronize()
        for rep in range(3):
            y.view(torch.uint8).fill_(0x7f)                  # eager work between the replays
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            print("case graph", dtype, tuning, "replay", rep, flush=True)
            G.check(l, G.to_host(y), ref, f"graph replay {rep} {dtype} {tuning}")
        del g
        plan.destroy()


def test_interleaved_samples_staged_by_rows():
    """tuning.stage_rows = 1 (fp32, pack = 3): rows of 16- and 8-byte loads, strides of one and two, tiles
    at the top and bottom edge of the plane, several chunks with a short last one, sample groups,
    split-K, batches that end inside a word; refused where rows are no whole 8-byte loads, where the
    tile is narrower than the plane, for other types and without interleaved samples."""
    cases = ((wl.Layer("rows16", 40, 24, 9, 8, 3, 3, 1, 1, 1, 1, N=7, sparsity=0.7, dtype="f32", seed=111),
              [dict(tile_p=3, chunk_c=8), dict(tile_p=9, chunk_c=16, tile_d=8), dict(tile_p=1, chunk_c=7, wg_threads=768),
               dict(tile_p=2, chunk_c=8, split_n=3), dict(tile_p=4, chunk_c=12, sub_batch=1)]),
             (wl.Layer("rows8", 24, 20, 6, 6, 3, 3, 1, 1, 1, 1, N=21, sparsity=0.6, dtype="f32", seed=112),
              [dict(tile_p=2, chunk_c=8, sub_batch=3), dict(tile_p=6, chunk_c=24), dict(tile_p=3, chunk_c=5, split_n=4, tile_d=16)]),
             (wl.Layer("rows_s2", 32, 20, 14, 12, 3, 3, 2, 2, 1, 1, N=5, sparsity=0.6, dtype="f32", seed=113),
              [dict(tile_p=7, chunk_c=8), dict(tile_p=2, chunk_c=4, tile_d=8), dict(tile_p=3, chunk_c=16, split_n=2)]),
             (wl.Layer("rows_5x5", 16, 12, 10, 12, 5, 5, 1, 1, 2, 2, N=3, sparsity=0.8, dtype="f32", seed=114),
              [dict(tile_p=4, chunk_c=8)]))
    for l, tunings in cases:
        data = wl.prepare(l, ragged=True)
        ref = G.oracle_out(l, data)
        plan = G.make_plan(l, data)
        for extra in tunings:
            kw = dict(variant=B.SC_VARIANT_SLAB, wsrc=1, pack=3, stage_rows=1, wg_threads=256)
            kw.update(extra)
            plan.set_tuning(B.sc_tuning_t(), **kw)
            t = plan.get_tuning().as_dict()
            assert t["stage_rows"] == 1 and t["pack"] == 3
            print("case", l.name, t, flush=True)
            G.check(l, G.run_gpu(plan, data["x"]), ref, f"{l.name} {t}")
        with pytest.raises(B.SparseConvError):          # without interleaved samples
            plan.set_tuning(B.sc_tuning_t(), variant=B.SC_VARIANT_SLAB, wsrc=1, stage_rows=1, chunk_c=8, tile_p=2)
        with pytest.raises(B.SparseConvError):          # GATHER
            plan.set_tuning(B.sc_tuning_t(), variant=B.SC_VARIANT_GATHER, stage_rows=1)
        plan.destroy()
    for l in (wl.Layer("rows_odd", 16, 12, 9, 7, 3, 3, 1, 1, 1, 1, N=3, sparsity=0.5, dtype="f32", seed=115),     # rows of 28 bytes
              wl.Layer("rows_f16", 16, 12, 8, 8, 3, 3, 1, 1, 1, 1, N=9, sparsity=0.5, dtype="f16", seed=116)):
        plan = G.make_plan(l, wl.prepare(l))
        with pytest.raises(B.SparseConvError):
            plan.set_tuning(B.sc_tuning_t(), variant=B.SC_VARIANT_SLAB, wsrc=1, pack=3, stage_rows=1, chunk_c=8, tile_p=2)
        plan.destroy()


def test_random_candidates_on_seeded_random_layers():
    """Eighteen seeded layers of random geometry (filters 1x1 .. 5x5, strides, paddings, planes of 2 .. 20,
    3 .. 130 channels, batches 1 .. 9, every type, unified and ragged tables), and on each about forty
    of the autotuner's candidates drawn at random: each gives the oracle's result."""
    for seed in range(18):
        rng = np.random.default_rng(1000 + seed)
        dtype = ["f32", "f16", "i8", "cb4", "cb4h", "f32"][seed % 6]
        R, S = [(1, 1), (3, 3), (1, 3), (5, 5), (2, 2), (3, 1)][int(rng.integers(6))]
        sh, sw = (int(rng.integers(1, 3)), int(rng.integers(1, 3))) if R * S > 1 else (1, 1)
        ph, pw = int(rng.integers(0, R // 2 + 1)), int(rng.integers(0, S // 2 + 1))
        H, W = int(rng.integers(max(R, 2), 21)), int(rng.integers(max(S, 2), 21))
        C, D, N = int(rng.integers(3, 131)), int(rng.integers(3, 91)), int(rng.integers(1, 10))
        sp = float(rng.uniform(0.3, 0.95))
        l = wl.Layer(f"rand{seed}", C, D, H, W, R, S, sh, sw, ph, pw, N=N, sparsity=sp, dtype=dtype, seed=500 + seed)
        data = wl.prepare(l, ragged=bool(seed & 1))
        ref = G.oracle_out(l, data)
        plan = G.make_plan(l, data)
        nc = plan.num_candidates()
        pick = sorted(set(int(i) for i in rng.integers(0, nc, size=44)))
        print(f"case rand{seed}: {dtype} C{C} D{D} {H}x{W} {R}x{S} s{sh},{sw} p{ph},{pw} N{N} sp{sp:.2f}: {nc} candidates, {len(pick)} drawn", flush=True)
        for i in pick:
            t = plan.candidate(i)
            plan.set_tuning(t)
            G.check(l, G.run_gpu(plan, data["x"]), ref, f"{l.name} candidate {i} { {k: v for k, v in t.as_dict().items() if v} }")
        plan.destroy()


@pytest.mark.parametrize("dtype", ["f16", "i8", "cb4", "cb4h"])
def test_dense_variant_on_pointwise_layers_in_their_natural_layout(dtype):
    """tuning.stage_rows = 1 on the matrix-core tile (pointwise layers): the tile is copied to LDS as
    [channel][position] and read with the transposing LDS reads.  Planes whose runs are whole 16-,
    8-, 4-, 2-byte loads and odd ones, several chunks with a last one that is not full, channels
    that do not fill a block, tiles of rows and whole planes of several samples, batches that do
    not fill the last group, four and eight waves; refused for filters with taps and with the
    pipelined form."""
    shapes = [("pw16", 150, 70, 8, 8, 7, 0.7), ("pw28", 64, 40, 28, 28, 3, 0.5), ("pw14", 200, 37, 14, 14, 5, 0.8),
              ("pw7", 96, 48, 7, 7, 19, 0.9), ("pw5x6", 40, 130, 5, 6, 9, 0.6), ("pw_one_block", 24, 40, 9, 8, 3, 0.5)]
    cb = 64 if dtype in ("i8", "cb4") else 32
    for name, C, D, H, W, N, sp in shapes:
        l = wl.Layer(name, C, D, H, W, 1, 1, 1, 1, 0, 0, N=N, sparsity=sp, dtype=dtype, seed=888)
        data = wl.prepare(l)
        ref = G.oracle_out(l, data)
        plan = G.make_plan(l, data)
        ran = 0
        for extra in ({}, {"tile_d": 16}, {"tile_d": 32, "tile_p": 1}, {"tile_d": 64, "tile_p": 2, "chunk_c": cb},
                      {"tile_d": 128, "wg_per_cu": 1}, {"tile_d": 64, "tile_p": 1000, "sub_batch": 4, "chunk_c": 2 * cb},
                      {"tile_d": 128, "waves_m": 2, "tile_p": 2}, {"tile_d": 64, "waves_m": 1, "tile_p": 3},
                      {"tile_d": 32, "waves_m": 2, "tile_p": 1000, "sub_batch": 3},
                      {"tile_d": 32, "tile_p": 1000, "sub_batch": 16, "chunk_c": 128, "wg_per_cu": 1},
                      {"tile_d": 16, "split_n": 2}, {"tile_d": 32, "tile_p": 2, "split_n": 3}, {"tile_d": 16, "tile_p": 1, "split_n": 16}):
            for threads in (256, 512):
                try:
                    plan.set_tuning(B.sc_tuning_t(), variant=B.SC_VARIANT_DENSE, wg_threads=threads, stage_rows=1, **extra)
                except B.SparseConvError as e:
                    assert e.status == 4
                    continue
                t = plan.get_tuning()
                assert t.variant == B.SC_VARIANT_DENSE and t.stage_rows == 1 and t.wg_threads == threads
                print("case dense natural", name, dtype, t.as_dict(), flush=True)
                G.check(l, G.run_gpu(plan, data["x"]), ref, f"{name} dense natural {extra} {threads}")
                ran += 1
        assert ran >= 6, (name, ran)
        # pipelined: the chunks are copied by direct-to-LDS loads (runs and planes of whole 16-byte words, one
        # sample per workgroup); refused otherwise
        piped = 0
        for extra in ({}, {"tile_p": 1, "chunk_c": cb, "producers": 1}, {"tile_p": 2, "tile_d": 32, "producers": 4},
                      {"tile_p": 4, "tile_d": 64, "waves_m": 1, "chunk_c": 3 * cb}, {"tile_p": 1000, "tile_d": 128, "chunk_c": cb}):
            for threads in (256, 512):
                try:
                    plan.set_tuning(B.sc_tuning_t(), variant=B.SC_VARIANT_DENSE, wg_threads=threads, stage_rows=1, pipeline=1, **extra)
                except B.SparseConvError as e:
                    assert e.status == 4
                    continue
                t = plan.get_tuning()
                assert t.stage_rows == 1 and t.pipeline == 1 and t.sub_batch == 1
                print("case dense natural pipelined", name, dtype, t.as_dict(), flush=True)
                G.check(l, G.run_gpu(plan, data["x"]), ref, f"{name} dense natural pipelined {extra} {threads}")
                piped += 1
        whole_words = (H * W * (1 if dtype in ("i8", "cb4") else 2)) % 16 == 0
        assert (piped >= 2) == whole_words, (name, piped)
        plan.destroy()
    l = wl.Layer("taps", 32, 16, 8, 8, 3, 3, 1, 1, 1, 1, N=2, sparsity=0.5, dtype=dtype, seed=889)
    plan = G.make_plan(l, wl.prepare(l))
    with pytest.raises(B.SparseConvError):
        plan.set_tuning(B.sc_tuning_t(), variant=B.SC_VARIANT_DENSE, stage_rows=1)
    plan.destroy()


def test_natural_layout_candidates_on_seeded_random_pointwise_layers():
    """Twelve seeded pointwise layers (planes of whole 16-byte words and odd ones, 3 .. 300 channels, batches
    1 .. 11, the four 16- and 8-bit types) and on each up to thirty of the autotuner's natural-layout
    candidates of the matrix-core tile (register copy and direct-to-LDS copy) drawn at random."""
    ran = 0
    for seed in range(12):
        rng = np.random.default_rng(7000 + seed)
        dtype = ["f16", "i8", "cb4h", "cb4"][seed % 4]
        H, W = int(rng.integers(1, 9)) * 4, int(rng.integers(1, 9)) * 4
        if seed % 3 == 0:
            H, W = int(rng.integers(2, 30)), int(rng.integers(2, 30))
        C, D, N = int(rng.integers(3, 300)), int(rng.integers(3, 200)), int(rng.integers(1, 12))
        sp = float(rng.uniform(0.3, 0.95))
        l = wl.Layer(f"rnat{seed}", C, D, H, W, 1, 1, 1, 1, 0, 0, N=N, sparsity=sp, dtype=dtype, seed=900 + seed)
        data = wl.prepare(l, ragged=bool(seed & 1))
        ref = G.oracle_out(l, data)
        plan = G.make_plan(l, data)
        nat = [i for i in range(plan.num_candidates())
               if plan.candidate(i).stage_rows and plan.candidate(i).variant == B.SC_VARIANT_DENSE]
        pick = [nat[int(i)] for i in sorted(set(rng.integers(0, len(nat), size=30)))] if nat else []
        print(f"case rnat{seed}: {dtype} C{C} D{D} {H}x{W} N{N} sp{sp:.2f}: {len(nat)} natural-layout candidates, {len(pick)} drawn", flush=True)
        for i in pick:
            t = plan.candidate(i)
            plan.set_tuning(t)
            G.check(l, G.run_gpu(plan, data["x"]), ref, f"{l.name} candidate {i} { {k: v for k, v in t.as_dict().items() if v} }")
            ran += 1
        plan.destroy()
    assert ran >= 150, ran
