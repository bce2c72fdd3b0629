"""Host logic of the synthetic workload generator (no GPU)."""
import numpy as np

from paper_2112_15445_amd import workloads as wl


def test_config1_is_58_of_576():
    (l,) = wl.config1()
    assert (l.K, l.n, l.N, l.P, l.Q) == (576, 58, 1, 32, 32)
    rowptr, colidx, vals = wl.draw_weights_csr(l)
    assert np.all(np.diff(rowptr) == 58) and vals.dtype == np.float32
    for d in range(l.D):
        row = colidx[rowptr[d]:rowptr[d + 1]]
        assert np.all(np.diff(row) > 0) and row.min() >= 0 and row.max() < l.K
    assert 0.04 < vals.std() < 0.06
    x = wl.draw_input(l)
    assert x.shape == (1, 64, 32, 32) and x.min() >= -1 and x.max() < 1


def test_config_shapes_and_counts():
    assert [l.n for l in wl.config2()] == [8, 115, 86, 173, 115, 230, 230, 184, 369, 369, 230, 230, 230]
    assert [l.n for l in wl.config5()[:13]] == [3, 58, 58, 115, 115, 230, 230, 230] + [461] * 5
    assert len(wl.config3()) == 30 and len(wl.config4()) == 75 and len(wl.config5()) == 26
    by = {l.name: l for l in wl.config3()}
    assert by["s56_reduce1x1_sp90"].n == 26 and by["s56_expand1x1_sp90"].n == 6
    assert by["s28_conv3x3_s2_sp90"].P == 28 and by["s28_conv3x3_s2_sp90"].H == 56
    assert by["s7_conv3x3_sp80"].n == 922
    h = wl.headline_layer()
    assert abs(h.algorithmic_bytes() - 128.46e6) < 0.05e6 and h.useful_macs == 166985728
    assert len({l.seed for l in wl.config2()}) == 13


def test_draws_are_seeded():
    l = wl.config2()[4]
    a = wl.draw_weights_csr(l)
    b = wl.draw_weights_csr(l)
    assert all(np.array_equal(u, v) for u, v in zip(a, b))
    assert np.array_equal(wl.draw_input(l, 2), wl.draw_input(l, 2))


def test_ragged_draw_has_unified_maximum():
    l = wl.config1()[0]
    rowptr, colidx, _ = wl.draw_weights_csr(l, ragged=True)
    lens = np.diff(rowptr)
    assert lens.max() == l.n and lens.min() < l.n


def test_quantisers():
    l = wl.config5()[1]
    p = wl.prepare(l, N=1)
    assert p["values"].dtype == np.int8 and p["x"].dtype == np.int8 and p["scales"].shape == (l.D,)
    assert np.abs(p["values"].astype(int)).max() == 127 and np.abs(p["x"].astype(int)).max() == 127
    pc = wl.prepare(wl.config5()[14], N=1)
    assert pc["values"].dtype == np.uint8 and pc["values"].max() < 16
    cent, cb, sc = wl.codebook16()
    assert np.all(np.diff(cent) > 0) and cb[0] == -127 and cb[15] == 127 and np.all(cb == -cb[::-1])
    # nearest-centroid assignment, ties to the lower index
    mid = 0.5 * (cent[3] + cent[4])
    assert wl.assign_codebook(np.array([cent[5], mid]), cent).tolist() in ([5, 3], [5, 4])
    assert wl.assign_codebook(np.array([0.0]), cent).tolist() == [7]


def test_one_dimensional_workload_shapes():
    ls = wl.config6()
    assert len(ls) == 12 and {l.dtype for l in ls} == {"f32", "f16"}
    l = ls[0]
    assert (l.C, l.D, l.H, l.W, l.R, l.S, l.N) == (300, 64, 1, 64, 1, 2, 128)
    assert (l.P, l.Q) == (1, 63) and l.K == 600
    assert [x.n for x in ls[:6]] == [138, 102, 75, 207, 153, 113]      # 77 / 83 / 87.5 % of 600 and 900
