"""Pins for the CPU oracle: everything here checks the oracle against something other than itself
(a library routine, a closed form, brute force in Python, an invariant of the method, or a value
the paper fixes).  No GPU, no HIP library."""
import os

import numpy as np
import pytest
import scipy.sparse as sp
import torch

import oracle
from paper_2112_15445_amd import workloads as wl


def _rand_layer(rng, integer=False, C=None, D=None):
    C = C or int(rng.integers(1, 5))
    D = D or int(rng.integers(1, 5))
    R, S = int(rng.integers(1, 4)), int(rng.integers(1, 4))
    stride = (int(rng.integers(1, 3)), int(rng.integers(1, 3)))
    pad = (int(rng.integers(0, 3)), int(rng.integers(0, 3)))
    H = int(rng.integers(max(1, R - 2 * pad[0]), 8))
    W = int(rng.integers(max(1, S - 2 * pad[1]), 8))
    N = int(rng.integers(1, 3))
    if integer:
        x = rng.integers(-127, 128, size=(N, C, H, W)).astype(np.int8)
        w = rng.integers(-127, 128, size=(D, C, R, S)).astype(np.int8)
    else:
        x = rng.uniform(-1, 1, size=(N, C, H, W)).astype(np.float32)
        w = rng.normal(0, 0.05, size=(D, C, R, S)).astype(np.float32)
    return x, w, stride, pad


def _prune(rng, w, keep_frac):
    D = w.shape[0]
    K = w[0].size
    flat = w.reshape(D, K)
    rowptr = [0]
    cols, vals = [], []
    for d in range(D):
        k = int(rng.integers(0, K + 1)) if keep_frac is None else max(0, int(round(keep_frac * K)))
        sel = np.sort(rng.choice(K, size=k, replace=False))
        cols.extend(sel.tolist())
        vals.extend(flat[d, sel].tolist())
        rowptr.append(len(cols))
    return (np.array(rowptr, np.int32), np.array(cols, np.int32),
            np.array(vals, dtype=w.dtype))


# ------------------------------------------------------------------ dense definition vs library
@pytest.mark.parametrize("seed", range(25))
def test_dense_matches_torch_conv2d_float64(seed):
    rng = np.random.default_rng(seed)
    x, w, stride, pad = _rand_layer(rng)
    y = oracle.dense_conv(x, w, stride, pad)
    t = torch.nn.functional.conv2d(torch.from_numpy(x).double(), torch.from_numpy(w).double(),
                                   stride=stride, padding=pad).numpy()
    assert y.shape == t.shape
    np.testing.assert_allclose(y, t, rtol=0, atol=1e-13)


@pytest.mark.parametrize("seed", range(10))
def test_dense_int_matches_torch_in_exact_double(seed):
    rng = np.random.default_rng(100 + seed)
    x, w, stride, pad = _rand_layer(rng, integer=True)
    y = oracle.dense_conv(x, w, stride, pad)
    assert y.dtype == np.int32
    t = torch.nn.functional.conv2d(torch.from_numpy(x).double(), torch.from_numpy(w).double(),
                                   stride=stride, padding=pad).numpy()
    assert np.array_equal(y, t.astype(np.int64))


def test_dense_midsize_matches_torch():
    rng = np.random.default_rng(7)
    x = rng.uniform(-1, 1, size=(2, 16, 14, 13)).astype(np.float32)
    w = rng.normal(0, 0.05, size=(8, 16, 3, 3)).astype(np.float32)
    for stride, pad in (((1, 1), (1, 1)), ((2, 2), (1, 1)), ((2, 1), (0, 2))):
        y = oracle.dense_conv(x, w, stride, pad)
        t = torch.nn.functional.conv2d(torch.from_numpy(x).double(), torch.from_numpy(w).double(),
                                       stride=stride, padding=pad).numpy()
        np.testing.assert_allclose(y, t, rtol=0, atol=1e-13)


# ------------------------------------------------------------------ sparse method == dense result
@pytest.mark.parametrize("seed", range(40))
def test_sparse_equals_dense_on_tiny_layers(seed):
    rng = np.random.default_rng(1000 + seed)
    integer = seed % 2 == 1
    x, w, stride, pad = _rand_layer(rng, integer=integer)
    rowptr, colidx, vals = _prune(rng, w, None)          # ragged rows, any count incl. 0 and K
    D, C, R, S = w.shape
    wd = oracle.dense_from_csr(rowptr, colidx, vals, D, C, R, S)
    yd = oracle.dense_conv(x, wd.astype(w.dtype) if integer else wd, stride, pad)
    ys = oracle.sparse_conv(x, rowptr, colidx, vals, R, S, stride, pad)
    if integer:
        assert np.array_equal(ys, yd)
    else:
        np.testing.assert_allclose(ys, yd, rtol=0, atol=1e-13)


@pytest.mark.parametrize("integer", [False, True])
def test_zero_sparsity_is_dense_convolution(integer):
    rng = np.random.default_rng(5)
    x, w, stride, pad = _rand_layer(rng, integer=integer, C=3, D=4)
    rowptr, colidx, vals = _prune(rng, w, 1.0)            # keep every position: n = K
    D, C, R, S = w.shape
    st = oracle.sparse_conv_steps(x, rowptr, colidx, vals, R, S, stride, pad)
    assert st["n"] == C * R * S
    yd = oracle.dense_conv(x, w, stride, pad)
    if integer:
        assert np.array_equal(st["y"], yd)
    else:
        np.testing.assert_allclose(st["y"], yd, rtol=0, atol=1e-12)


def test_superposition_of_disjoint_supports():
    rng = np.random.default_rng(11)
    x, w, stride, pad = _rand_layer(rng, C=4, D=3)
    D, C, R, S = w.shape
    K = C * R * S
    mask = rng.random((D, K)) < 0.5

    def csr(m):
        rp, ci, va = [0], [], []
        for d in range(D):
            sel = np.nonzero(m[d])[0]
            ci.extend(sel.tolist())
            va.extend(w.reshape(D, K)[d, sel].tolist())
            rp.append(len(ci))
        return np.array(rp, np.int32), np.array(ci, np.int32), np.array(va, np.float32)

    ya = oracle.sparse_conv(x, *csr(mask), R, S, stride, pad)
    yb = oracle.sparse_conv(x, *csr(~mask), R, S, stride, pad)
    yall = oracle.sparse_conv(x, *csr(np.ones_like(mask)), R, S, stride, pad)
    np.testing.assert_allclose(ya + yb, yall, rtol=0, atol=1e-13)


# ------------------------------------------------------------------ the paper's worked example
def test_paper_figure_two_tap_filter(golden_dir):
    taps = {}
    for line in open(os.path.join(golden_dir, "paper_figure_two_taps.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, r, s, a, b = line.split()
        taps[name] = (int(r), int(s), int(a), int(b))
    rng = np.random.default_rng(3)
    H, W, pad = 6, 7, 1
    Wp = W + 2 * pad
    x = rng.uniform(-1, 1, size=(1, 1, H, W)).astype(np.float32)
    w1, w2 = np.float32(0.3), np.float32(-0.7)
    r1, s1, a1, b1 = taps["w1"]
    r2, s2, a2, b2 = taps["w2"]
    rowptr = np.array([0, 2], np.int32)
    colidx = np.array([r1 * 3 + s1, r2 * 3 + s2], np.int32)
    vals = np.array([w1, w2], np.float32)
    st = oracle.sparse_conv_steps(x, rowptr, colidx, vals, 3, 3, (1, 1), (pad, pad))
    # the pre-computed offsets the figure implies
    assert st["lam"].tolist() == [[a1 + b1 * Wp, a2 + b2 * Wp]] == [[2, 2 * Wp]]
    xp = np.pad(x[0, 0].astype(np.float64), pad)
    P, Q = H, W
    expect = np.empty((P, Q))
    for p in range(P):
        for q in range(Q):
            expect[p, q] = float(w1) * xp[p, q + 2] + float(w2) * xp[p + 2, q]
    np.testing.assert_allclose(st["y"][0, 0], expect, rtol=0, atol=1e-15)


def test_paper_padded_input_extents(golden_dir):
    for line in open(os.path.join(golden_dir, "paper_padded_extents.txt")):
        if line.startswith("#") or not line.strip():
            continue
        C, H, W, pad, Hp, Wp = map(int, line.split())
        # a single-channel slice is enough to pin the padded geometry; keep it small
        x = np.ones((1, 1, H, W), np.float32)
        st = oracle.sparse_conv_steps(x, np.array([0, 1], np.int32), np.array([8], np.int32),
                                      np.array([1.0], np.float32), 3, 3, (1, 1), (pad, pad))
        assert st["xp"].shape == (1, 1, Hp, Wp)
        assert st["y"].shape == (1, 1, H, W)
        # last tap (r=2, s=2) sits two padded rows and two columns from the origin
        assert st["lam"][0, 0] == 2 * Wp + 2
        l = wl.Layer("t", C, 1, H, W)
        assert (l.Hp, l.Wp) == (Hp, Wp)


def test_mac_count_reduced_by_sparsity_ratio(golden_dir):
    for line in open(os.path.join(golden_dir, "paper_vgg16_table_layers.txt")):
        if line.startswith("#") or not line.strip():
            continue
        C, H, W, D, s = line.split()
        l = wl.Layer("t", int(C), int(D), int(H), int(W), N=128, sparsity=float(s) / 100)
        dense = l.N * l.D * l.P * l.Q * l.K
        achieved = 1 - l.n / l.K
        assert l.useful_macs == l.N * l.D * l.P * l.Q * l.n
        assert abs(l.useful_macs - (1 - achieved) * dense) < 1e-6 * dense
        assert abs(achieved - float(s) / 100) <= 0.5 / l.K + 1e-12


# ------------------------------------------------------------------ unified non-zero count
def test_unified_nnz_invariants_and_padding_is_neutral():
    rng = np.random.default_rng(21)
    x, w, stride, pad = _rand_layer(rng, C=4, D=6)
    D, C, R, S = w.shape
    rowptr, colidx, vals = _prune(rng, w, None)
    st = oracle.sparse_conv_steps(x, rowptr, colidx, vals, R, S, stride, pad)
    n = int(np.max(np.diff(rowptr)))
    assert st["n"] == n and st["theta"].shape == (D, n) and st["lam"].shape == (D, n)
    for d in range(D):
        ln = rowptr[d + 1] - rowptr[d]
        assert np.array_equal(st["col"][d, :ln], colidx[rowptr[d]:rowptr[d + 1]])
        assert np.all(st["theta"][d, ln:] == 0)                 # fillers are explicit zeros
        assert np.all(st["col"][d, ln:] == (colidx[rowptr[d + 1] - 1] if ln else 0))
    # feeding the already-unified arrays back must give the same result (padding is neutral)
    rp2 = np.arange(D + 1, dtype=np.int32) * n
    y2 = oracle.sparse_conv(x, rp2, st["col"].ravel(), st["theta"].ravel().astype(np.float32),
                            R, S, stride, pad)
    np.testing.assert_array_equal(y2, st["y"])


def test_entry_order_within_row_is_irrelevant_for_integers():
    rng = np.random.default_rng(22)
    x, w, stride, pad = _rand_layer(rng, integer=True, C=4, D=3)
    D, C, R, S = w.shape
    rowptr, colidx, vals = _prune(rng, w, 0.6)
    y = oracle.sparse_conv(x, rowptr, colidx, vals, R, S, stride, pad)
    ci, va = colidx.copy(), vals.copy()
    for d in range(D):
        perm = rng.permutation(rowptr[d + 1] - rowptr[d]) + rowptr[d]
        ci[rowptr[d]:rowptr[d + 1]] = colidx[perm]
        va[rowptr[d]:rowptr[d + 1]] = vals[perm]
    assert np.array_equal(oracle.sparse_conv(x, rowptr, ci, va, R, S, stride, pad), y)


def test_duplicate_columns_add_up():
    x = np.arange(16, dtype=np.float32).reshape(1, 1, 4, 4)
    rowptr = np.array([0, 3], np.int32)
    colidx = np.array([0, 0, 3], np.int32)                      # 2x2 filter, tap 0 twice
    vals = np.array([1.0, 2.0, 0.5], np.float32)
    y = oracle.sparse_conv(x, rowptr, colidx, vals, 2, 2)
    xe = x[0, 0].astype(np.float64)
    np.testing.assert_allclose(y[0, 0], 3.0 * xe[:-1, :-1] + 0.5 * xe[1:, 1:], atol=1e-15)


# ------------------------------------------------------------------ stretch
def test_stretch_round_trip_and_bounds():
    rng = np.random.default_rng(31)
    for _ in range(20):
        x, w, stride, pad = _rand_layer(rng)
        D, C, R, S = w.shape
        N, _, H, W = x.shape
        rowptr, colidx, vals = _prune(rng, w, 1.0)
        st = oracle.sparse_conv_steps(x, rowptr, colidx, vals, R, S, stride, pad)
        Hp, Wp = H + 2 * pad[0], W + 2 * pad[1]
        lam, col = st["lam"], st["col"]
        c, rem = lam // (Hp * Wp), lam % (Hp * Wp)
        r, s = rem // Wp, rem % Wp
        assert np.array_equal((c * R + r) * S + s, col)
        assert np.all((r < R) & (s < S) & (c < C))
        P, Q = st["y"].shape[2:]
        assert (P - 1) * stride[0] * Wp + (Q - 1) * stride[1] + lam.max() < C * Hp * Wp


# ------------------------------------------------------------------ 1x1 special case: CSR SpMM
@pytest.mark.parametrize("seed", range(4))
def test_pointwise_conv_is_csr_spmm(seed):
    rng = np.random.default_rng(40 + seed)
    N, C, D, H, W = 2, 12, 7, 5, 6
    x = rng.uniform(-1, 1, size=(N, C, H, W)).astype(np.float32)
    w = rng.normal(0, 0.05, size=(D, C, 1, 1)).astype(np.float32)
    rowptr, colidx, vals = _prune(rng, w, 0.3)
    A = sp.csr_matrix((vals.astype(np.float64), colidx, rowptr), shape=(D, C))
    y = oracle.sparse_conv(x, rowptr, colidx, vals, 1, 1)
    for b in range(N):
        ref = A @ x[b].reshape(C, H * W).astype(np.float64)
        np.testing.assert_allclose(y[b].reshape(D, H * W), ref, rtol=0, atol=1e-14)


# ------------------------------------------------------------------ integer and codebook paths
def _brute_sparse(x, rowptr, colidx, vals, R, S, stride, pad):
    """Pure-Python statement of the definition on the *unpadded* input (tiny cases only)."""
    N, C, H, W = x.shape
    D = len(rowptr) - 1
    P = (H + 2 * pad[0] - R) // stride[0] + 1
    Q = (W + 2 * pad[1] - S) // stride[1] + 1
    y = np.zeros((N, D, P, Q), dtype=object)
    for b in range(N):
        for d in range(D):
            for k in range(rowptr[d], rowptr[d + 1]):
                c, r, s = colidx[k] // (R * S), (colidx[k] // S) % R, colidx[k] % S
                for p in range(P):
                    for q in range(Q):
                        ih, iw = p * stride[0] + r - pad[0], q * stride[1] + s - pad[1]
                        if 0 <= ih < H and 0 <= iw < W:
                            y[b, d, p, q] += int(vals[k]) * int(x[b, c, ih, iw])
    return y.astype(np.int64)


@pytest.mark.parametrize("seed", range(6))
def test_int8_path_matches_python_brute_force(seed):
    rng = np.random.default_rng(50 + seed)
    x, w, stride, pad = _rand_layer(rng, integer=True)
    D, C, R, S = w.shape
    rowptr, colidx, vals = _prune(rng, w, 0.4)
    y = oracle.sparse_conv(x, rowptr, colidx, vals, R, S, stride, pad)
    assert y.dtype == np.int32
    assert np.array_equal(y, _brute_sparse(x, rowptr, colidx, vals, R, S, stride, pad))


def test_codebook_path_equals_int8_path_after_host_decode():
    rng = np.random.default_rng(60)
    x, w, stride, pad = _rand_layer(rng, integer=True, C=4, D=5)
    D, C, R, S = w.shape
    rowptr, colidx, _ = _prune(rng, w, 0.5)
    idx = rng.integers(0, 16, size=colidx.shape[0]).astype(np.uint8)
    cb = np.sort(rng.integers(-127, 128, size=16)).astype(np.int8)
    y_cb = oracle.sparse_conv(x, rowptr, colidx, idx, R, S, stride, pad, codebook=cb)
    y_i8 = oracle.sparse_conv(x, rowptr, colidx, cb[idx], R, S, stride, pad)
    assert np.array_equal(y_cb, y_i8)
    assert np.array_equal(y_cb, _brute_sparse(x, rowptr, colidx, cb[idx], R, S, stride, pad))


def test_sixteen_bit_codebook_path_equals_the_half_path_after_host_decode():
    """4-bit indices into 16 fp16 centroids with fp16 activations (the 4b/16b configuration): the
    same result as the fp16 path run on the decoded weights, and as the dense definition (torch
    float64 conv2d on the decoded dense tensor), rounded once to fp16."""
    rng = np.random.default_rng(61)
    x, w, stride, pad = _rand_layer(rng, C=5, D=4)
    x16 = x.astype(np.float16)
    D, C, R, S = w.shape
    rowptr, colidx, _ = _prune(rng, w, 0.5)
    idx = rng.integers(0, 16, size=colidx.shape[0]).astype(np.uint8)
    cb = np.sort(rng.normal(0, 0.05, size=16)).astype(np.float16)
    y_cb = oracle.sparse_conv(x16, rowptr, colidx, idx, R, S, stride, pad, codebook=cb, out_dtype=np.float16)
    y_h = oracle.sparse_conv(x16, rowptr, colidx, cb[idx], R, S, stride, pad, out_dtype=np.float16)
    assert y_cb.dtype == np.float16 and np.array_equal(y_cb, y_h)
    wd = oracle.dense_from_csr(rowptr, colidx, cb[idx].astype(np.float64), D, C, R, S)
    t = torch.nn.functional.conv2d(torch.from_numpy(x16.astype(np.float64)), torch.from_numpy(wd),
                                   stride=stride, padding=pad).numpy()
    assert np.array_equal(y_cb, t.astype(np.float16))


def test_fp16_operands_single_rounding():
    rng = np.random.default_rng(70)
    x, w, stride, pad = _rand_layer(rng, C=4, D=3)
    x16, w16 = x.astype(np.float16), w.astype(np.float16)
    D, C, R, S = w.shape
    rowptr, colidx, vals = _prune(rng, w16, 0.5)
    y = oracle.sparse_conv(x16, rowptr, colidx, vals, R, S, stride, pad, out_dtype=np.float16)
    assert y.dtype == np.float16
    wd = oracle.dense_from_csr(rowptr, colidx, vals.astype(np.float64), D, C, R, S)
    t = torch.nn.functional.conv2d(torch.from_numpy(x16.astype(np.float64)), torch.from_numpy(wd),
                                   stride=stride, padding=pad).numpy()
    assert np.array_equal(y, t.astype(np.float16))


# ------------------------------------------------------------------ the linear fixed-point quantiser
def test_pow2_quantiser_worked_examples():
    """Values fixed by the paper's formulas (section "Quantisation"): int_bits = ceil(log2 max|x|),
    frac_bits = total_bits - int_bits - 1, sigma = 2^-frac_bits, code = round(x / sigma)."""
    # max 0.75 -> int_bits 0, frac_bits 7, sigma 1/128
    c, f = oracle.quantise_pow2(np.array([0.3, -0.75, 0.1, 0.0]), 8)
    assert f == 7 and c.tolist() == [38, -96, 13, 0]
    # max 3.0 -> int_bits 2, frac_bits 5, sigma 1/32
    c, f = oracle.quantise_pow2(np.array([3.0, -1.0, 0.015625, 2.984375]), 8)
    assert f == 5 and c.tolist() == [96, -32, 0, 96]          # 0.5 and 95.5 are ties: to even
    # max 0.05 -> int_bits ceil(-4.32) = -4, frac_bits 11: small tensors gain resolution
    c, f = oracle.quantise_pow2(np.array([0.05, -0.025]), 8)
    assert f == 11 and c.tolist() == [102, -51]
    # a maximum that is an exact power of two needs one more bit than the formula grants: saturates
    c, f = oracle.quantise_pow2(np.array([1.0, -1.0, 0.5]), 8)
    assert f == 7 and c.tolist() == [127, -128, 64]
    # fewer bits, and the all-zero tensor
    c, f = oracle.quantise_pow2(np.array([0.9, -0.3]), 4)
    assert f == 3 and c.tolist() == [7, -2]
    c, f = oracle.quantise_pow2(np.zeros(3), 8)
    assert f == 7 and c.tolist() == [0, 0, 0]
    # saturation threshold: the maximum is scaled first (1.3 * 0.75 = 0.975 -> int_bits 0) and the data clipped to it
    c, f = oracle.quantise_pow2(np.array([1.3, -0.2]), 8, saturate_at=0.75)
    assert f == 7 and c.tolist() == [125, -26]                # 0.975 * 128 = 124.8, -25.6


@pytest.mark.parametrize("seed", range(4))
def test_pow2_quantiser_properties(seed):
    rng = np.random.default_rng(90 + seed)
    x = (rng.normal(0, 10.0 ** rng.integers(-3, 3), size=500)).astype(np.float32)
    for bits in (8, 6, 3):
        c, f = oracle.quantise_pow2(x, bits)
        sigma = 2.0 ** -f
        m = float(np.max(np.abs(x)))
        assert 2.0 ** (bits - 1 - f) >= m > 2.0 ** (bits - 2 - f)          # int_bits = ceil(log2 max)
        q = sigma * c.astype(np.float64)
        unsat = np.abs(x.astype(np.float64)) <= sigma * (2 ** (bits - 1) - 1)
        assert np.all(np.abs(q[unsat] - x[unsat]) <= sigma / 2)             # nearest grid point
        assert np.all(np.diff(c[np.argsort(x, kind="stable")].astype(int)) >= 0)   # monotone
        c2, f2 = oracle.quantise_pow2(q, bits)                              # the grid is a fixed point
        if int(np.max(np.abs(c.astype(int)))) > 2 ** (bits - 2):           # ... while the maximum keeps its octave
            assert f2 == f and np.array_equal(c2, c)


# ------------------------------------------------------------------ the pins have teeth
def test_planted_mistakes_are_caught():
    """Re-run step 4 of the oracle with deliberately wrong step-2 / step-3 results and check that
    the dense definition exposes each of them (non-square shapes so transpositions matter)."""
    import ctypes
    from oracle import oracle as om
    lib = om._load()
    rng = np.random.default_rng(80)
    N, C, H, W, D, R, S = 1, 3, 6, 9, 4, 3, 2
    stride, pad = (2, 1), (1, 2)
    x = rng.uniform(-1, 1, size=(N, C, H, W)).astype(np.float32)
    w = rng.normal(0, 0.05, size=(D, C, R, S)).astype(np.float32)
    rowptr, colidx, vals = _prune(rng, w, 0.5)
    st = oracle.sparse_conv_steps(x, rowptr, colidx, vals, R, S, stride, pad)
    yd = oracle.dense_conv(x, oracle.dense_from_csr(rowptr, colidx, vals, D, C, R, S), stride, pad)
    np.testing.assert_allclose(st["y"], yd, atol=1e-13)
    Hp, Wp = H + 2 * pad[0], W + 2 * pad[1]
    P, Q = st["y"].shape[2:]
    col = st["col"].astype(np.int64)
    c, r, s = col // (R * S), (col // S) % R, col % S

    def run(lam, theta=None, sh=stride[0], sw=stride[1], wp=Wp):
        lam = np.ascontiguousarray(lam, np.int64)
        th = np.ascontiguousarray(st["theta"] if theta is None else theta, np.float64)
        y = np.empty((N, D, P, Q))
        lib.oracle_gather_mac_f64(om._p(st["xp"]), om._p(th), om._p(lam), om._p(y), N,
                                  C * Hp * Wp, D, st["n"], P, Q, sh, sw, wp)
        return y

    good = (c * Hp + r) * Wp + s
    np.testing.assert_allclose(run(good), yd, atol=1e-13)
    wrong = {
        "row pitch without padding": (c * Hp + r) * W + s,
        "plane pitch without padding": (c * H + r) * Wp + s,
        "r and s transposed": (c * Hp + s) * Wp + r,
        "channel dropped": r * Wp + s,
    }
    for name, lam in wrong.items():
        lam = np.minimum(lam, good.max())                     # stay in bounds
        assert np.abs(run(lam) - yd).max() > 1e-6, name
    assert np.abs(run(good, sh=stride[1], sw=stride[0]) - yd)[..., :min(P, Q), :min(P, Q)].max() > 1e-6
    th = st["theta"].copy()
    th[:, -1] = 0
    assert np.abs(run(good, theta=th) - yd).max() > 1e-6, "dropped term"
    assert np.abs(run(good, theta=-st["theta"]) - yd).max() > 1e-6, "sign"


# ------------------------------------------------------------------------------------------------
# epilogue of a VGG-shaped layer: ReLU, 2 x 2 max-pool, requantisation
# ------------------------------------------------------------------------------------------------
def test_epilogue_relu_and_pool_against_torch():
    import torch
    rng = np.random.default_rng(5)
    for shape in ((2, 3, 6, 8), (1, 4, 7, 5), (3, 2, 2, 2), (2, 2, 1, 9)):
        y = rng.normal(size=shape)
        t = torch.from_numpy(y)
        assert np.array_equal(oracle.epilogue(y, relu=True), torch.relu(t).numpy())
        if shape[2] >= 2 and shape[3] >= 2:
            ref = torch.nn.functional.max_pool2d(t, 2).numpy()
            assert np.array_equal(oracle.epilogue(y, pool=2), ref)
            ref = torch.nn.functional.max_pool2d(torch.relu(t), 2).numpy()
            assert np.array_equal(oracle.epilogue(y, relu=True, pool=2), ref)
        else:
            assert oracle.epilogue(y, pool=2).shape == (shape[0], shape[1], shape[2] // 2, shape[3] // 2)
    yi = rng.integers(-500, 500, size=(2, 3, 4, 6)).astype(np.int32)
    ref = torch.nn.functional.max_pool2d(torch.relu(torch.from_numpy(yi.astype(np.float64))), 2).numpy()
    got = oracle.epilogue(yi, relu=True, pool=2)
    assert got.dtype == np.int32 and np.array_equal(got, ref.astype(np.int32))


def test_epilogue_pool_hand_values_and_dropped_odd_edges():
    y = np.arange(15, dtype=np.float64).reshape(1, 1, 3, 5)      # rows 0..2, columns 0..4
    out = oracle.epilogue(y, pool=2)
    assert out.shape == (1, 1, 1, 2)                              # third row and fifth column dropped
    assert out.tolist() == [[[[6.0, 8.0]]]]                      # max(0,1,5,6), max(2,3,7,8)
    y = np.array([[[[-3.0, -1.0], [-2.0, -5.0]]]])
    assert oracle.epilogue(y, pool=2).item() == -1.0
    assert oracle.epilogue(y, relu=True, pool=2).item() == 0.0    # ReLU first, then the window maximum


def test_epilogue_requantisation_hand_values():
    acc = np.array([10, 14, -10, -14, 1000, -1000, 0, 3], dtype=np.int32).reshape(1, 1, 1, 8)
    q = oracle.epilogue(acc, requant_scale=np.array([0.25], np.float32))
    # 2.5 -> 2 and 3.5 -> 4 (ties to even), symmetric for negatives, saturation at +-127, 0.75 -> 1
    assert q.dtype == np.int8 and q.reshape(-1).tolist() == [2, 4, -2, -4, 127, -127, 0, 1]
    # per-channel scales, applied after ReLU and pooling
    acc = np.array([[[[7, -9], [3, 5]]], [[[7, -9], [3, 5]]]], dtype=np.int32).reshape(1, 2, 2, 2)
    q = oracle.epilogue(acc, relu=True, pool=2, requant_scale=np.array([1.0, 0.5], np.float32))
    assert q.reshape(-1).tolist() == [7, 4]                       # 7 * 1 and 7 * 0.5 = 3.5 -> 4


def test_epilogue_requantisation_is_single_precision_arithmetic():
    """The code is rint(float32(acc) * float32(scale)) with every step rounded to single precision:
    against the same three steps done one scalar at a time, and different from the double-precision
    evaluation on an accumulator that single precision cannot hold exactly."""
    rng = np.random.default_rng(11)
    acc = rng.integers(-2 ** 26, 2 ** 26, size=(1, 3, 2, 50)).astype(np.int32)
    sc = (rng.random(3) * 1e-5 + 1e-6).astype(np.float32)
    q = oracle.epilogue(acc, requant_scale=sc)
    for d in range(3):
        for i, a in enumerate(acc[0, d].reshape(-1)):
            v = np.float32(np.float32(a) * sc[d])
            e = int(max(-127, min(127, np.rint(v))))
            assert q[0, d].reshape(-1)[i] == e
    big = np.array([2 ** 24 + 1], dtype=np.int32).reshape(1, 1, 1, 1)     # float32 rounds it to 2^24
    assert oracle.epilogue(big, requant_scale=np.array([2.0 ** -18], np.float32)).item() == 64
    assert np.float32(big.item()) == np.float32(2 ** 24)


def test_epilogue_relu_commutes_with_pool_and_positive_scale():
    rng = np.random.default_rng(12)
    y = rng.normal(size=(2, 3, 6, 6))
    a = oracle.epilogue(oracle.epilogue(y, relu=True), pool=2)
    b = oracle.epilogue(oracle.epilogue(y, pool=2), relu=True)
    assert np.array_equal(a, b)
