"""The oracle reproduces its own committed fixture (drift guard); fixture is oracle-written only."""
import importlib.util
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))


def _load_maker():
    spec = importlib.util.spec_from_file_location("make_oracle_golden", os.path.join(HERE, "golden", "make_oracle_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_oracle_matches_committed_fixture():
    mk = _load_maker()
    rows = [l.split() for l in open(os.path.join(HERE, "golden", "oracle_c1_head.txt")) if not l.startswith("#")]
    assert len(rows) == 32
    for fb in ("adam_denom", "sgdm"):
        st = mk.compute(fb)
        for r in (r for r in rows if r[0] == fb):
            i = int(r[1])
            assert float(st.theta[i]) == float.fromhex(r[2])
            assert float(st.m[i]) == float.fromhex(r[3])
            assert float(st.v[i]) == float.fromhex(r[4])
    # the two readings really differ on this workload
    a = [r for r in rows if r[0] == "adam_denom"]
    b = [r for r in rows if r[0] == "sgdm"]
    assert any(x[2] != y[2] for x, y in zip(a, b))


def test_oracle_full_features_matches_committed_fixture():
    """Every optional phase at once, fp32 and bfloat16 first moment: guards the research-mode code against drift."""
    mk = _load_maker()
    rows = [l.split() for l in open(os.path.join(HERE, "golden", "oracle_full_features.txt")) if not l.startswith("#")]
    assert len(rows) >= 30
    for md in ("f32", "bf16_m"):
        sts = mk.compute_full(md)
        for r in (r for r in rows if r[0] == md):
            st, i = sts[int(r[1])], int(r[2])
            assert float(st.theta[i]) == float.fromhex(r[3])
            assert float(st.m[i]) == float.fromhex(r[4])
            assert float(st.v[i]) == float.fromhex(r[5])
    a = [r for r in rows if r[0] == "f32"]
    b = [r for r in rows if r[0] == "bf16_m"]
    assert any(x[3] != y[3] for x, y in zip(a, b)) and any(x[4] != y[4] for x, y in zip(a, b))
