"""The input generator: deterministic, well-formed, and shaped like the stated distributions."""
import numpy as np
import torch

import workloads as W


def test_batches_are_well_formed_and_deterministic():
    for name, kw in (("C1", {}), ("C2", dict(T=5, B=128, rows_scale=0.01)), ("C3", dict(T=6, B=64, rows_scale=1e-3)),
                     ("C4", dict(T=4, B=64, rows_scale=1e-3)), ("C5", dict(T=32, B=64, rows_scale=1e-3))):
        cfg = W.config(name, **kw)
        idx, off = W.make_batch(cfg, 0)
        idx2, off2 = W.make_batch(cfg, 0)
        assert torch.equal(idx, idx2) and torch.equal(off, off2)
        idx3, _ = W.make_batch(cfg, 1)
        assert idx3.numel() != idx.numel() or not torch.equal(idx, idx3)
        assert off.numel() == cfg.T * cfg.B + 1 and off[0] == 0 and off[-1] == idx.numel()
        L = off[1:] - off[:-1]
        assert int(L.min()) >= 1
        for t in range(cfg.T):
            seg = idx[off[t * cfg.B]:off[(t + 1) * cfg.B]]
            assert int(seg.min()) >= 0 and int(seg.max()) < cfg.rows[t]


def test_length_and_id_distributions():
    cfg = W.config("C2", T=2, B=4096)
    idx, off = W.make_batch(cfg, 0)
    L = (off[1:] - off[:-1]).double()
    assert abs(L.mean().item() - 11.0) < 0.3 and abs(L.var().item() - 10.0) < 1.0        # Poisson(10)+1
    cfg5 = W.config("C5", T=16, B=8192, rows_scale=1e-3)
    _, off5 = W.make_batch(cfg5, 0)
    L5 = off5[1:] - off5[:-1]
    assert int(L5.max()) <= 500 and 10.0 < L5.double().mean().item() < 14.5               # lognormal(2,1) capped
    # bounded Zipf: the hottest row of a table carries about 1/H_{R,s} of its lookups
    cfg3 = W.config("C3", T=1, B=4096, rows_scale=1e-2)
    i3, _ = W.make_batch(cfg3, 0)
    R = cfg3.rows[0]
    top = torch.bincount(i3, minlength=R).max().item() / i3.numel()
    H = float((torch.arange(1, R + 1, dtype=torch.float64) ** -1.2).sum())
    assert abs(top - 1.0 / H) < 0.02
    c1 = W.config("C1")
    i1, o1 = W.make_batch(c1, 0)
    assert i1.numel() == 512 * 20 and torch.all(o1[1:] - o1[:-1] == 20)


def test_procedural_weights_are_uniform_and_row_addressable():
    cfg = W.config("C2", T=3, B=8, rows_scale=1e-2)
    flat = torch.empty(cfg.total_elems, dtype=torch.float32)
    W.fill_weights(cfg, flat, chunk_elems=1000)
    woff = cfg.w_offsets()
    for t in range(cfg.T):
        rows = torch.tensor([0, cfg.rows[t] // 2, cfg.rows[t] - 1])
        got = W.weight_rows(cfg, t, rows)
        for k, r in enumerate(rows.tolist()):
            assert torch.equal(got[k], flat[woff[t] + r * cfg.D[t]: woff[t] + (r + 1) * cfg.D[t]])
    assert flat.min() >= -0.01 and flat.max() < 0.01
    assert abs(flat.mean().item()) < 2e-4 and abs(flat.std().item() - 0.01 / np.sqrt(3)) < 2e-4
    # tables differ, seeds differ
    assert not torch.equal(W.weight_rows(cfg, 0, torch.arange(4)), W.weight_rows(cfg, 1, torch.arange(4)))
    cfg_b = W.config("C2", T=3, B=8, rows_scale=1e-2, seed=1)
    assert not torch.equal(W.weight_rows(cfg, 0, torch.arange(4)), W.weight_rows(cfg_b, 0, torch.arange(4)))


def test_named_configs_have_the_stated_shapes():
    c2, c3, c4, c5 = (W.config(n) for n in ("C2", "C3", "C4", "C5"))
    assert c2.T == 26 and min(c2.rows) >= 1000 and max(c2.rows) <= 1_000_000 and set(c2.D) == {64}
    assert c3.T == 128 and set(c3.D) == {64, 128, 256} and min(c3.rows) >= 10_000 and max(c3.rows) <= 10_000_000
    assert c4.T == 256 and abs(c4.total_rows - 4e8) < 1e6 and c4.weight_dtype == "f16" and set(c4.D) == {128, 256}
    assert 170e9 < c4.weight_bytes + 4 * c4.total_rows < 190e9
    assert c5.T == 128 and c5.rows.count(50_000_000) == 8 and c5.rows.count(100_000) == 120 and c5.pooling == "mean"
    assert c5.rows[:8] == [50_000_000] * 8
    c5i = W.config("C5I")                       # same tables, the big ones no longer next to one another
    assert sorted(c5i.rows) == sorted(c5.rows) and sum(c5i.D) == sum(c5.D) and c5i.pooling == "mean"
    big = [i for i, r in enumerate(c5i.rows) if r == 50_000_000]
    assert len(big) == 8 and min(np.diff(big)) == 16 and all(c5i.D[i] == 128 for i in big)
