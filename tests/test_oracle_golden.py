"""Golden fixtures of the oracle: hand-worked optimizer rows (from the formulas of Algorithm 1, steps 5-6, and the
row-wise AdaGrad definition of Section 3.2) and a stored mini case that guards against drift."""
import json
import os

import numpy as np
import torch

import workloads as W

GOLD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def test_hand_worked_rows_of_algorithm_1(oracle_mod):
    n = 0
    for line in open(os.path.join(GOLD, "algorithm1_worked_rows.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        scal, g, w0, v_new, w_new = [np.array(p.split(), dtype=np.float64) for p in line.split("|")]
        eta, eps, c, v_old = scal
        for dtype in (np.float32, np.float16):
            tab = np.stack([np.zeros_like(w0), w0, np.ones_like(w0)]).astype(dtype)
            v = np.array([v_old], dtype=np.float32)
            oracle_mod.adagrad_row(tab, 1, v, g, eta, eps, c)
            assert v[0] == np.float32(v_new[0])
            np.testing.assert_allclose(tab[1].astype(np.float64), w_new, rtol=0, atol=2e-3 if dtype == np.float16 else 1e-7)
            assert np.all(tab[0] == 0) and np.all(tab[2] == 1)
        # the same rows through the whole backward: one bag holding the row once, upstream gradient = g
        tab = np.stack([w0, w0]).astype(np.float32)
        state = np.array([7.0, v_old], dtype=np.float32)
        oracle_mod.backward_rowwise_adagrad([tab], state, g.astype(np.float32)[None, :], np.array([1]), np.array([0, 1]), 1,
                                            "sum", eta, eps, c)
        np.testing.assert_allclose(tab[1], w_new, rtol=0, atol=1e-7)
        assert state[1] == np.float32(v_new[0]) and state[0] == 7.0 and np.array_equal(tab[0], w0.astype(np.float32))
        n += 1
    assert n == 5


def test_stored_mini_case_is_reproduced(oracle_mod):
    doc = json.load(open(os.path.join(GOLD, "c1_mini_oracle.json")))
    c = doc["config"]
    cfg = W.config(c["name"], B=c["B"], rows_scale=c["rows_scale"], c=c["c"])
    assert cfg.rows == c["rows"] and cfg.D == c["D"]
    tab = W.weight_rows(cfg, 0, torch.arange(cfg.rows[0])).numpy()
    idx, off = (x.numpy() for x in W.make_batch(cfg, 0))
    assert idx.tolist() == doc["indices"] and off.tolist() == doc["offsets"]         # the generator did not drift
    gout = W.make_grad_out(cfg, 0).numpy()
    out = oracle_mod.forward([tab], idx, off, cfg.B, cfg.pooling)
    assert out.tobytes().hex() == doc["out_hex"]
    state = np.zeros(cfg.rows[0], dtype=np.float32)
    res = oracle_mod.backward_rowwise_adagrad([tab], state, gout, idx, off, cfg.B, cfg.pooling, cfg.lr, cfg.eps, cfg.c)
    assert tab.tobytes().hex() == doc["weights_after_hex"] and state.tobytes().hex() == doc["state_after_hex"]
    assert res.order.tolist() == doc["order"] and res.unique_rows.tolist() == doc["unique_rows"]
    assert res.seg_start.tolist() == doc["seg_start"]
