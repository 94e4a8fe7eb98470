"""The oracle still reproduces the values stored by tests/golden/make_golden.py."""
import importlib.util
import os

import numpy as np

from oracle import flurka_oracle as fo
from paper_2306_15799_amd import inputs

HERE = os.path.dirname(os.path.abspath(__file__))


def _load_maker():
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(HERE, "golden", "make_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_oracle_reproduces_stored_small_cases():
    mk = _load_maker()
    stored = {}
    with open(os.path.join(HERE, "golden", "oracle_small_cases.txt")) as f:
        for line in f:
            if line.startswith("#"):
                continue
            case, key, *vals = line.split()
            stored[(case, key)] = np.array([float(v) for v in vals])
    assert len(stored) == 12
    for name, w in mk.CASES:
        t = inputs.make_inputs(w, seed=3)
        out = fo.flurka_attention(t["Q"], t["K"], t["V"], t["E"], t["F"], t["omega"], w.phi)
        g = fo.flurka_attention_bwd(t["Q"], t["K"], t["V"], t["E"], t["F"], t["omega"], t["dOut"], w.phi)
        rec = {"out": out[:, :, mk.ROWS], "dQ": g[0][:, :, mk.ROWS], "dK": g[1][:, :, mk.ROWS],
               "dV": g[2][:, :, mk.ROWS], "dE": g[3][:, mk.ROWS], "dF": g[4][:, mk.ROWS]}
        for key, val in rec.items():
            ref = stored[(name, key)]
            assert np.allclose(np.ravel(val), ref, rtol=1e-10, atol=1e-13), (name, key)
