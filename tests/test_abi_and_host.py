"""CPU-side checks: the built library exports every symbol the header declares,
argument validation works without a GPU, and the speed accounting reproduces
the paper's printed table rows."""
import ctypes as C
import os
import re

import pytest

from paper_2507_23777_amd import metrics, xsm

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "xsm.h")).read()
    return sorted(set(re.findall(r"XSM_API\s+[\w\s\*]+?\b(xsm_\w+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared()
    assert len(names) >= 14 and set(names) == set(xsm.API)
    L = xsm.lib()
    for n in names:
        assert hasattr(L, n), n


def test_create_validates_configuration():
    L = xsm.lib()
    import synth_inputs as si
    h = C.c_void_p()
    good = xsm.make_config(si.get_config("c0"))
    assert L.xsm_create(C.byref(good), C.byref(h)) == 0
    assert L.xsm_weights_bytes(h) > 0 and L.xsm_kv_bytes(h) > 0 and L.xsm_workspace_bytes(h) > 0
    import numpy as np
    w = si.make_weights(si.get_config("c0"))
    assert L.xsm_canonical_weight_elems(h) == si.pack_canonical(si.get_config("c0"), w).size
    # unbound context refuses work, with a message
    vp, bt = xsm.xsm_verify_params(), xsm.xsm_batch()
    assert L.xsm_spec_step(h, C.byref(bt), C.byref(vp), None) == -3
    assert b"bound" in L.xsm_last_error(h)
    assert L.xsm_bind(h, None, None, None) == -1
    L.xsm_destroy(h)
    for field, val in [("head_dim", 48), ("n_draft", 16), ("d_model", 100), ("dtype", 3), ("max_batch", 0)]:
        bad = xsm.make_config(si.get_config("c0"))
        setattr(bad, field, val)
        assert L.xsm_create(C.byref(bad), C.byref(h)) == -1, field
        assert len(L.xsm_last_error(None)) > 0


def test_speedup_formula_reproduces_printed_tables(golden_dir):
    rows = [l.split() for l in open(os.path.join(golden_dir, "speedup_tables.txt"))
            if l.strip() and not l.startswith("#")]
    base = float(rows[0][2])
    assert rows[0][0] == "A"
    for name, scr, lat, printed in rows:
        s = metrics.speedup(float(scr), float(lat), base)
        # printed inputs are themselves rounded, so allow one unit of the last printed digit
        assert abs(s - float(printed)) < 0.0101, name
    assert metrics.step_compression_ratio([1, 2, 5, 1, 1]) == 2.0
    with pytest.raises(ValueError):
        metrics.step_compression_ratio([])
