"""Host-only checks of the C ABI: the library loads, exports every function the header declares,
and every argument error is reported before any GPU work (no GPU needed, no compute calls)."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2112_15445_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "sparse_conv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sparse_conv_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared_functions()
    assert len(names) >= 14
    lib = ctypes.CDLL(B.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(B.EXPORTS) == names          # the binding wraps exactly the declared set


def test_status_strings():
    L = B.lib()
    seen = {L.sparse_conv_status_string(i).decode() for i in range(9)}
    assert len(seen) == 9 and "ok" in seen
    assert L.sparse_conv_status_string(99).decode() == "unknown status"


def test_struct_layouts_match_the_header(tmp_path):
    """Sizes and a few offsets of the binding's ctypes structures against what a C compiler makes
    of include/sparse_conv.h."""
    import subprocess
    src = tmp_path / "sizes.c"
    src.write_text(
        '#include <stdio.h>\n#include <stddef.h>\n#include "sparse_conv.h"\n'
        'int main(void) { printf("%zu %zu %zu %zu %zu %zu %zu\\n", sizeof(sc_layer_t), sizeof(sc_tuning_t), '
        'sizeof(sc_plan_info_t), offsetof(sc_plan_info_t, tuning), offsetof(sc_tuning_t, ragged), offsetof(sc_tuning_t, pack), '
        'offsetof(sc_plan_info_t, weight_bytes)); return 0; }\n')
    exe = tmp_path / "sizes"
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    subprocess.check_call(["gcc", "-I", os.path.join(root, "include"), str(src), "-o", str(exe)])
    c = [int(v) for v in subprocess.check_output([str(exe)]).split()]
    assert c == [ctypes.sizeof(B.sc_layer_t), ctypes.sizeof(B.sc_tuning_t), ctypes.sizeof(B.sc_plan_info_t),
                 B.sc_plan_info_t.tuning.offset, B.sc_tuning_t.ragged.offset, B.sc_tuning_t.pack.offset,
                 B.sc_plan_info_t.weight_bytes.offset]
    assert ctypes.sizeof(B.sc_layer_t) == 40 and ctypes.sizeof(B.sc_tuning_t) == 17 * 4


def _expect(status, fn, *a, **k):
    with pytest.raises(B.SparseConvError) as e:
        fn(*a, **k)
    assert e.value.status == status, e.value


GOOD = dict(rowptr=np.array([0, 1, 2], np.int32), colidx=np.array([0, 35], np.int32),
            values=np.array([1.0, 2.0], np.float32))


def _layer(**kw):
    d = dict(C=4, D=2, H=5, W=5, R=3, S=3, stride=(1, 1), pad=(1, 1))
    d.update(kw)
    return B.make_layer(**d)


def test_create_rejects_bad_arguments_on_the_host():
    mk = B.Plan.create_csr
    _expect(1, mk, _layer(), B.SC_F32, None, GOOD["colidx"], GOOD["values"])                    # null rowptr
    _expect(1, mk, _layer(), B.SC_F32, GOOD["rowptr"], None, GOOD["values"])                    # null colidx
    _expect(2, mk, _layer(C=0), B.SC_F32, **GOOD)                                               # bad dim
    _expect(2, mk, _layer(stride=(0, 1)), B.SC_F32, **GOOD)
    _expect(2, mk, _layer(H=1, W=1, pad=(0, 0)), B.SC_F32, **GOOD)                              # empty output
    _expect(3, mk, _layer(), B.SC_F32, np.array([1, 1, 2], np.int32), GOOD["colidx"], GOOD["values"])
    _expect(3, mk, _layer(), B.SC_F32, np.array([0, 2, 1], np.int32), GOOD["colidx"], GOOD["values"])
    _expect(3, mk, _layer(), B.SC_F32, GOOD["rowptr"], np.array([0, 36], np.int32), GOOD["values"])
    _expect(3, mk, _layer(), B.SC_F32, GOOD["rowptr"], np.array([-1, 3], np.int32), GOOD["values"])
    _expect(4, mk, _layer(), 7, **GOOD)                                                         # dtype
    _expect(4, mk, _layer(), B.SC_I8, GOOD["rowptr"], GOOD["colidx"], np.array([1, 2], np.int8))  # no scales
    _expect(4, mk, _layer(), B.SC_CB4_I8, GOOD["rowptr"], GOOD["colidx"], np.array([1, 2], np.uint8),
            scales=np.ones(2, np.float32))                                                      # no codebook
    _expect(3, mk, _layer(), B.SC_CB4_I8, GOOD["rowptr"], GOOD["colidx"], np.array([1, 16], np.uint8),
            scales=np.ones(2, np.float32), codebook=np.zeros(16, np.int8))                      # index > 15
    _expect(4, mk, _layer(), B.SC_CB4_F16, GOOD["rowptr"], GOOD["colidx"], np.array([1, 2], np.uint8))  # no codebook
    _expect(3, mk, _layer(), B.SC_CB4_F16, GOOD["rowptr"], GOOD["colidx"], np.array([1, 16], np.uint8),
            codebook=np.zeros(16, np.float16))                                                  # index > 15
    _expect(4, mk, _layer(), 5, GOOD["rowptr"], GOOD["colidx"], GOOD["values"])                 # unknown dtype
    _expect(5, mk, _layer(C=70000, H=200, W=200), B.SC_F32, **GOOD)                             # >= 2^31 elements
    _expect(2, B.Plan.create_ell, _layer(), B.SC_F32, -1, GOOD["colidx"], GOOD["values"])
    _expect(1, B.Plan.create_ell, _layer(), B.SC_F32, 1, None, GOOD["values"])


def test_null_plan_arguments():
    L = B.lib()
    assert L.sparse_conv_plan_info(None, None) == 1
    assert L.sparse_conv_forward(None, None, None, 1, None, 0, None) == 1
    assert L.sparse_conv_plan_set_tuning(None, None, None) == 1
    assert L.sparse_conv_workspace_size(None, 1, None) == 1
    assert L.sparse_conv_plan_num_candidates(None, None) == 1
    L.sparse_conv_plan_destroy(None)          # allowed


def test_product_path_has_no_cpu_fallback():
    """The binding never imports the oracle, and a missing library is an import error."""
    src = open(os.path.join(ROOT, "paper_2112_15445_amd", "binding.py")).read()
    assert "oracle" not in src.replace("never imports the oracle", "")
    for root, _, files in os.walk(os.path.join(ROOT, "paper_2112_15445_amd")):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                body = open(os.path.join(root, f)).read()
                assert "import oracle" not in body and "from oracle" not in body, f


def test_pow2_quantiser_helper_matches_the_oracle_bit_for_bit():
    """sparse_conv_quantize_pow2 (host code of the library) against the oracle's statement of the
    same formulas: identical codes and frac_bits over magnitudes, bit widths and saturation levels."""
    import oracle
    rng = np.random.default_rng(7)
    for scale in (1e-3, 0.05, 1.0, 37.0, 1024.0):
        x = rng.normal(0, scale, size=4000).astype(np.float32)
        x[:8] = [0.0, scale, -scale, 0.5 * scale, 1.5 * scale, -2.5 * scale, 2.0 ** -20, -0.0]
        for bits in (8, 5, 2):
            for sat in (1.0, 0.99, 0.5):
                c, f = B.quantize_pow2(x, bits, sat)
                co, fo = oracle.quantise_pow2(x, bits, sat)
                assert f == fo and np.array_equal(c, co), (scale, bits, sat)
    for x in (np.array([1.0, -1.0, 0.5], np.float32), np.array([4.0], np.float32), np.zeros(5, np.float32),
              np.zeros(0, np.float32)):
        c, f = B.quantize_pow2(x, 8)
        co, fo = oracle.quantise_pow2(x, 8)
        assert f == fo and np.array_equal(c, co)
    fb = ctypes.c_int32()
    L = B.lib()
    one = np.ones(1, np.float32)
    out = np.zeros(1, np.int8)
    p = lambda a: ctypes.c_void_p(a.ctypes.data)
    assert L.sparse_conv_quantize_pow2(None, 1, 8, 1.0, p(out), ctypes.byref(fb)) == 1
    assert L.sparse_conv_quantize_pow2(p(one), 1, 8, 1.0, p(out), None) == 1
    assert L.sparse_conv_quantize_pow2(p(one), 1, 9, 1.0, p(out), ctypes.byref(fb)) == 4
    assert L.sparse_conv_quantize_pow2(p(one), 1, 8, 0.0, p(out), ctypes.byref(fb)) == 4
    bad = np.array([np.inf], np.float32)
    assert L.sparse_conv_quantize_pow2(p(bad), 1, 8, 1.0, p(out), ctypes.byref(fb)) == 5
