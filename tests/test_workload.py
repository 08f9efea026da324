"""The seeded input generators: determinism, shapes, the stated statistics."""
import importlib.util
import json
import os

import numpy as np

from oracle import logits as lg
from paper_2510_24211_amd import workload as wl

HERE = os.path.dirname(os.path.abspath(__file__))


def test_bf16_rounding_nearest_even():
    x = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 2.0 ** -7, 1.0 + 3 * 2.0 ** -8, -0.0], dtype=np.float32)
    b = wl.f32_to_bf16_bits(x)
    back = lg.bf16_bits_to_f64(b)
    assert list(back[:4]) == [1.0, 1.0, 1.0 + 2.0 ** -7, 1.0 + 2.0 ** -6]   # ties to even
    assert b[4] == 0x8000


def test_weight_is_deterministic_and_scaled():
    w = wl.scaled(wl.WORKLOADS["C1"], V=5000, d=64)
    W = wl.lm_head_weight(w)
    assert W.shape == (5000, 64) and W.dtype == np.uint16
    assert np.array_equal(W, wl.lm_head_weight(w))
    assert np.array_equal(W[:4096], wl.lm_head_weight(wl.scaled(w, V=4096)))
    vals = lg.bf16_bits_to_f64(W)
    assert abs(vals.std() - 0.02) < 5e-4 and abs(vals.mean()) < 5e-4


def test_hidden_table_drift_and_cfg_rows():
    w = wl.scaled(wl.WORKLOADS["C2"], N=128, d=256, V=512, v_lo=4, v_hi=260)
    t = wl.HiddenTable(w)
    full = t.full(drop_cache=False)
    assert full.shape == (1, 2, 128, w.age_cap + 1, 256)
    assert np.array_equal(full[0, 1, 70, 3], t.row(0, 1, 70, 3))
    assert np.array_equal(t.row(0, 0, 5, 99), t.row(0, 0, 5, w.age_cap))      # clean beyond the cap
    v = lg.bf16_bits_to_f64(full)
    clean = v[0, :, :, w.age_cap]
    assert abs(clean.std() - 1.0) < 0.02
    for a in (0, 1, 4):
        dev = (v[0, 0, :, a] - clean[0]).std()
        assert abs(dev - 0.3 * 0.6 ** a) < 0.15 * 0.3 * 0.6 ** a + 3e-3
    corr = np.corrcoef(clean[0].ravel(), clean[1].ravel())[0, 1]
    assert abs(corr - 0.9) < 0.02
    h = t.window([100], [[0] * 32])
    assert h.shape == (1, 2, 32, 256) and np.all(h[0, :, 28:] == 0)          # past the end


def test_video_frame_recursion():
    w = wl.scaled(wl.WORKLOADS["C4"], N=8 * 16, d=512, V=256, B=1)
    t = wl.HiddenTable(w)
    v = lg.bf16_bits_to_f64(t.full())[0, 0, :, w.age_cap].reshape(8, 16, 512)
    for f in range(1, 8):
        c = np.corrcoef(v[f].ravel(), v[f - 1].ravel())[0, 1]
        assert abs(c - 0.9) < 0.03
    assert abs(v[7].std() - 1.0) < 0.05


def test_c0_golden_regression():
    spec = importlib.util.spec_from_file_location("make_c0", os.path.join(HERE, "golden", "make_c0_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    want = json.load(open(os.path.join(HERE, "golden", "c0_golden.json")))
    assert mod.run() == want
