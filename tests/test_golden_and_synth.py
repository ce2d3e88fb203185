"""Drift detector for the oracle and sanity of the synthetic workloads (CPU only)."""
import importlib.util
import json
import os

import numpy as np
import pytest

from paper_2108_04167_amd import synth

HERE = os.path.dirname(os.path.abspath(__file__))


def test_oracle_has_not_drifted_from_its_frozen_tiny_case():
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(HERE, "golden", "make_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    now = mod.build()
    with open(os.path.join(HERE, "golden", "tiny_admm.json")) as f:
        ref = json.load(f)
    assert now["perm_head"] == ref["perm_head"]
    assert now["ranks"] == ref["ranks"]
    assert now["n_margin"] == ref["n_margin"]
    assert np.allclose(now["z_head"], ref["z_head"], rtol=1e-9, atol=1e-12)
    assert now["x_norm"] == pytest.approx(ref["x_norm"], rel=1e-9)
    assert now["bias"] == pytest.approx(ref["bias"], rel=1e-8, abs=1e-10)


@pytest.mark.parametrize("cfg,n,r", [(1, 512, 8), (2, 512, 22), (3, 512, 54), (4, 512, 18), (5, 512, 90)])
def test_workloads_have_the_stated_shapes(cfg, n, r):
    w = synth.make_workload(cfg, n=n)
    assert w.F.shape == (n, r) and w.F.dtype == np.float64 and w.F.flags.c_contiguous
    assert set(np.unique(w.y)) <= {-1.0, 1.0} and set(np.unique(w.y_test)) <= {-1.0, 1.0}
    assert 0.2 < (w.y > 0).mean() < 0.8
    assert w.F_test.shape[1] == r and w.F_test.shape[0] == w.y_test.size
    w2 = synth.make_workload(cfg, n=n)
    assert np.array_equal(w.F, w2.F) and np.array_equal(w.y, w2.y)
    assert np.array_equal(w.omega(), w2.omega()) and w.omega().shape == (n, w.s)


def test_workload_specifics():
    w2 = synth.make_workload(2, n=4096)
    assert np.allclose(w2.F.mean(axis=0), 0, atol=1e-12) and np.allclose(w2.F.std(axis=0), 1, atol=1e-12)
    w3 = synth.make_workload(3, n=4096)
    assert set(np.unique(w3.F[:, 10:])) <= {0.0, 1.0}
    assert 0.08 < w3.F[:, 10:].mean() < 0.12
    w4 = synth.make_workload(4, n=1024)
    assert w4.F.min() >= -1 and w4.F.max() <= 1
    w5 = synth.make_workload(5, n=256)
    assert w5.C_grid == (0.1, 1.0, 10.0, 100.0) and w5.beta_grid == (0.5, 1.0, 2.0)
    full = {1: (2048, 64, 128), 2: (65536, 128, 256)}
    for c, (n, leaf, s) in full.items():
        w = synth.make_workload(c)
        assert (w.n, w.leaf, w.s) == (n, leaf, s)
