"""Edge cases of the HIP path against the oracle: empty and ragged inputs, degenerate shapes, the extremes
of the segment-length classes, unusual widths, the error path, determinism and graph replay."""
import numpy as np
import pytest
import torch

import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def H():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import gpu_harness
    return gpu_harness


def make_cfg(rows, D, dtype="f32", B=8, pooling="sum", c=1.0, lr=0.05, eps=1e-8):
    cfg = W.Config("edge", list(rows), list(D), dtype, B, pooling, ("fixed", 1), ("uniform",))
    cfg.c, cfg.lr, cfg.eps = c, lr, eps
    return cfg


def run_custom(H, cfg, lens, ids, seed=0, state_kind="hash", steps=1):
    """lens: T*B bag lengths; ids: concatenated table-local ids."""
    from paper_2508_03854_amd import TBE
    off = torch.zeros(len(lens) + 1, dtype=torch.int64)
    off[1:] = torch.cumsum(torch.as_tensor(lens, dtype=torch.int64), 0)
    idx = torch.as_tensor(ids, dtype=torch.int64)
    assert off[-1] == idx.numel()
    g = torch.Generator().manual_seed(seed)
    tabs = H.host_tables(cfg)
    flat = H.flat_from_tables(tabs)
    state_np = (W.state_rows(cfg, torch.arange(cfg.total_rows)).numpy() if state_kind == "hash"
                else np.zeros(cfg.total_rows, dtype=np.float32))
    state = torch.from_numpy(state_np.copy()).cuda()
    tbe = TBE(cfg.rows, cfg.D, cfg.weight_dtype)
    ws = tbe.alloc_workspace(cfg.B, max(1, idx.numel()))
    reps = []
    for s in range(steps):
        gout = torch.randn(cfg.B, cfg.sum_D, generator=g, dtype=torch.float32)
        reps.append(H.check_step(cfg, tbe, flat, state, tabs, state_np, idx, off, gout, ws, same_inputs=(s == 0)))
    tbe.close()
    return reps


def test_empty_bags_everywhere_and_long_runs_of_empty_bags(H):
    rng = np.random.default_rng(0)
    cfg = make_cfg([50, 7, 300], [64, 32, 128], B=3000, pooling="mean")
    lens = rng.integers(0, 3, size=3 * 3000)
    lens[100:2900] = 0                      # 2800 empty bags in a row inside table 0
    lens[3000:6000] = 0                     # table 1 has no lookups at all
    lens[0] = 0
    lens[-1] = 0
    ids = np.concatenate([rng.integers(0, cfg.rows[t], size=int(lens[t * 3000:(t + 1) * 3000].sum())) for t in range(3)])
    rep = run_custom(H, cfg, lens, ids)
    assert rep[0]["U"] > 0


def test_no_lookups_at_all(H):
    from paper_2508_03854_amd import TBE
    cfg = make_cfg([10, 20], [16, 8], B=5)
    tabs = H.host_tables(cfg)
    flat = H.flat_from_tables(tabs)
    before = flat.clone()
    state = torch.ones(30, device="cuda")
    tbe = TBE(cfg.rows, cfg.D, "f32")
    off = torch.zeros(2 * 5 + 1, dtype=torch.int64, device="cuda")
    idx = torch.zeros(0, dtype=torch.int64, device="cuda")
    out = tbe.forward(flat, idx, off, 5, "sum")
    assert torch.count_nonzero(out) == 0
    ws = tbe.alloc_workspace(5, 1)
    tbe.backward_rowwise_adagrad(torch.randn(5, 24, device="cuda"), idx, off, 5, flat, state, ws, lr=0.1, eps=1e-8)
    torch.cuda.synchronize()
    assert torch.equal(flat, before) and torch.equal(state, torch.ones(30, device="cuda"))


def test_batch_of_one_single_table_single_row(H):
    cfg = make_cfg([1], [4], B=1)
    run_custom(H, cfg, [5], [0, 0, 0, 0, 0])                  # one row hit five times in one bag
    cfg = make_cfg([3], [8], B=1, dtype="f16", pooling="mean")
    run_custom(H, cfg, [2], [2, 0])                           # max id = rows-1


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("pooling", ["sum", "mean"])
def test_segment_length_classes(H, dtype, pooling):
    # rows hit exactly 1, 2, 63, 64, 65, 511, 512, 513, 1025 and 5000 times: every boundary of the short / medium /
    # long classes of the segment kernels; B is large so the hits of one row spread over many bags
    rng = np.random.default_rng(1)
    counts = [1, 2, 63, 64, 65, 511, 512, 513, 1025, 5000, 1, 1, 3, 64, 64]
    B = 700
    cfg = make_cfg([len(counts) + 5, 40], [64, 256], dtype=dtype, B=B, pooling=pooling, c=4.0)
    ids0 = np.concatenate([np.full(n, r) for r, n in enumerate(counts)])
    rng.shuffle(ids0)
    lens0 = rng.multinomial(len(ids0), np.ones(B) / B)
    ids1 = rng.integers(0, 40, size=3 * B)
    lens1 = np.full(B, 3)
    rep = run_custom(H, cfg, np.concatenate([lens0, lens1]), np.concatenate([ids0, ids1]), steps=2)
    assert rep[0]["max_seg"] == 5000


def test_one_row_takes_a_hundred_thousand_lookups(H):
    rng = np.random.default_rng(2)
    B, n = 2048, 120_000
    cfg = make_cfg([10], [128], B=B)
    ids = np.where(rng.random(n) < 0.9, 3, rng.integers(0, 10, size=n))
    lens = rng.multinomial(n, np.ones(B) / B)
    rep = run_custom(H, cfg, lens, ids, state_kind="zeros")
    assert rep[0]["max_seg"] > 100_000


@pytest.mark.parametrize("dtype,Ds", [("f32", [4, 12, 20, 36, 96, 100, 160, 260, 384, 512, 1024]),
                                      ("f16", [8, 24, 40, 96, 136, 264, 520, 1024])])
def test_unusual_widths(H, dtype, Ds):
    # widths that are not powers of two, narrower than a float4 group, and wider than one 64-lane pass
    rng = np.random.default_rng(3)
    B = 64
    rows = [30 + 3 * i for i in range(len(Ds))]
    cfg = make_cfg(rows, Ds, dtype=dtype, B=B, pooling="mean", c=2.0)
    lens = rng.integers(0, 9, size=len(Ds) * B)
    ids = np.concatenate([rng.integers(0, rows[t], size=int(lens[t * B:(t + 1) * B].sum())) for t in range(len(Ds))])
    # make one row of the widest table long enough for the chunked path
    run_custom(H, cfg, lens, ids)
    cfg2 = make_cfg([5], [Ds[-1]], dtype=dtype, B=600)
    run_custom(H, cfg2, np.full(600, 3), rng.integers(0, 2, size=1800))


def test_invalid_ids_are_reported_and_harmless():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2508_03854_amd import TBE
    import oracle
    rows, D, B = [10, 6], [8, 16], 4
    tbe = TBE(rows, D, "f32")
    g = torch.Generator().manual_seed(0)
    flat_cpu = torch.randn(10 * 8 + 6 * 16, generator=g)
    flat = flat_cpu.cuda()
    lens = [2, 1, 0, 3, 1, 1, 2, 1]
    good = torch.tensor([1, 9, 4, 0, 3, 3, 5, 0, 2, 1, 5], dtype=torch.int64)
    bad = good.clone()
    bad[1] = 10                      # == rows[0]
    bad[3] = -1
    bad[8] = 6                       # == rows[1]
    off = torch.zeros(9, dtype=torch.int64)
    off[1:] = torch.cumsum(torch.tensor(lens), 0)
    out = tbe.forward(flat, bad.cuda(), off.cuda(), B, "sum")
    assert tbe.poll_index_error() and not tbe.poll_index_error()          # reported once, then cleared
    # the forward skips invalid ids: same as the oracle on the bags with those lookups removed
    keep = torch.ones(11, dtype=torch.bool)
    keep[[1, 3, 8]] = False
    lens2 = [1, 1, 0, 2, 1, 1, 1, 1]
    off2 = np.concatenate([[0], np.cumsum(lens2)])
    tabs = [flat_cpu[:80].view(10, 8).numpy().copy(), flat_cpu[80:].view(6, 16).numpy().copy()]
    ref = oracle.forward(tabs, good[keep].numpy(), off2, B, "sum")
    np.testing.assert_allclose(out.cpu().numpy(), ref, rtol=1e-6, atol=1e-6)
    # the backward gives invalid ids to no row: same as the oracle without them
    state = torch.zeros(16, device="cuda")
    gout = torch.randn(B, 24, generator=g)
    ws = tbe.alloc_workspace(B, 11)
    tbe.backward_rowwise_adagrad(gout.cuda(), bad.cuda(), off.cuda(), B, flat, state, ws, lr=0.1, eps=1e-8)
    assert tbe.poll_index_error()
    st = np.zeros(16, dtype=np.float32)
    oracle.backward_rowwise_adagrad(tabs, st, gout.numpy(), good[keep].numpy(), off2, B, "sum", 0.1, 1e-8, 1.0)
    np.testing.assert_allclose(flat.cpu().numpy(), np.concatenate([t.reshape(-1) for t in tabs]), rtol=1e-5, atol=1e-6)
    np.testing.assert_allclose(state.cpu().numpy(), st, rtol=1e-5)
    dbg = tbe.debug_sorted(ws, B, 11)
    valid_keys = {1, 4, 3} | {10 + 5, 10 + 0, 10 + 1}                     # table 0: ids 1,4,3,3; table 1: ids 5,0,1,5
    assert dbg["num_unique"] == len(valid_keys) + 1
    assert set(dbg["unique_rows"][:-1].tolist()) == valid_keys
    assert int(dbg["unique_rows"][-1]) == 16                              # the trailing pseudo-row of invalid ids


def test_argument_checks_return_status_codes():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2508_03854_amd import TBE, TbeError
    from paper_2508_03854_amd import binding as Bn
    tbe = TBE([10], [8], "f32")
    flat = torch.zeros(80, device="cuda")
    state = torch.zeros(10, device="cuda")
    idx = torch.zeros(4, dtype=torch.int64, device="cuda")
    off = torch.tensor([0, 2, 4], dtype=torch.int64, device="cuda")
    gout = torch.zeros(2, 8, device="cuda")
    ws = tbe.alloc_workspace(2, 4)
    for kw, code in ((dict(lr=float("nan"), eps=1e-8), Bn.EINVAL), (dict(lr=0.1, eps=-1.0), Bn.EINVAL),
                     (dict(lr=0.1, eps=1e-8, momentum_scale=0.0), Bn.EINVAL),
                     (dict(lr=0.1, eps=1e-8, momentum_scale=-2.0), Bn.EINVAL)):
        with pytest.raises(TbeError) as e:
            tbe.backward_rowwise_adagrad(gout, idx, off, 2, flat, state, ws, **kw)
        assert e.value.status == code
    with pytest.raises(TbeError) as e:
        tbe.backward_rowwise_adagrad(gout, idx, off, 2, flat, state, ws[:256], lr=0.1, eps=1e-8)
    assert e.value.status == Bn.EWORKSPACE
    with pytest.raises(TbeError) as e:
        TBE([10], [6], "f32")
    assert e.value.status == Bn.ESHAPE
    torch.cuda.synchronize()
    assert torch.count_nonzero(flat) == 0 and torch.count_nonzero(state) == 0     # nothing was launched


def test_two_runs_agree_bit_for_bit_and_graph_replay_matches_eager():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2508_03854_amd import TBE
    cfg = W.config("C3", T=6, B=512, rows_scale=2e-3, c=2.0)
    idx, off = (x.cuda() for x in W.make_batch(cfg, 0))
    gout = W.make_grad_out(cfg, 0).cuda()
    tbe = TBE(cfg.rows, cfg.D, cfg.weight_dtype)
    ws = tbe.alloc_workspace(cfg.B, idx.numel())

    def fresh():
        flat = torch.empty(cfg.total_elems, device="cuda")
        W.fill_weights(cfg, flat)
        return flat, torch.zeros(cfg.total_rows, device="cuda")

    def eager(flat, state, n):
        outs = []
        for _ in range(n):
            outs.append(tbe.forward(flat, idx, off, cfg.B, cfg.pooling).clone())
            tbe.backward_rowwise_adagrad(gout, idx, off, cfg.B, flat, state, ws, pooling=cfg.pooling, lr=cfg.lr,
                                         eps=cfg.eps, momentum_scale=cfg.c)
        torch.cuda.synchronize()
        return outs

    f1, s1 = fresh()
    o1 = eager(f1, s1, 3)
    f2, s2 = fresh()
    o2 = eager(f2, s2, 3)
    assert torch.equal(f1, f2) and torch.equal(s1, s2) and all(torch.equal(a, b) for a, b in zip(o1, o2))

    # the two hot calls record no memset and allocate nothing: capture one step, replay it three times with eager
    # work and synchronisation in between, and compare every replay with the eager sequence
    f3, s3 = fresh()
    out3 = torch.empty(cfg.B, cfg.sum_D, device="cuda")
    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    f_warm, s_warm = fresh()
    with torch.cuda.stream(stream):                      # warm-up on the side stream, on scratch copies
        tbe.forward(f_warm, idx, off, cfg.B, cfg.pooling, out=out3, stream=stream)
        tbe.backward_rowwise_adagrad(gout, idx, off, cfg.B, f_warm, s_warm, ws, pooling=cfg.pooling, lr=cfg.lr,
                                     eps=cfg.eps, momentum_scale=cfg.c, stream=stream)
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=stream):
        cur = torch.cuda.current_stream()
        tbe.forward(f3, idx, off, cfg.B, cfg.pooling, out=out3, stream=cur)
        tbe.backward_rowwise_adagrad(gout, idx, off, cfg.B, f3, s3, ws, pooling=cfg.pooling, lr=cfg.lr, eps=cfg.eps,
                                     momentum_scale=cfg.c, stream=cur)
    for k in range(3):
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out3, o1[k]), f"replay {k}: forward differs from eager"
        _ = (out3 * 2).sum().item()                      # unrelated eager work between replays
    assert torch.equal(f3, f1) and torch.equal(s3, s1)
    tbe.close()


def test_checkpoint_resume_is_bit_identical():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2508_03854_amd import TBE
    cfg = W.config("C2", T=4, B=256, rows_scale=0.02, c=4.0)
    tbe = TBE(cfg.rows, cfg.D, cfg.weight_dtype)
    batches = [tuple(x.cuda() for x in W.make_batch(cfg, s)) for s in range(2)]
    gouts = [W.make_grad_out(cfg, s).cuda() for s in range(2)]
    ws = tbe.alloc_workspace(cfg.B, max(b[0].numel() for b in batches))
    res = []
    for copy_between in (False, True):
        flat = torch.empty(cfg.total_elems, device="cuda")
        W.fill_weights(cfg, flat)
        state = torch.zeros(cfg.total_rows, device="cuda")
        for s in range(2):
            tbe.backward_rowwise_adagrad(gouts[s], batches[s][0], batches[s][1], cfg.B, flat, state, ws, lr=cfg.lr,
                                         eps=cfg.eps, momentum_scale=cfg.c)
            if copy_between:                                  # "checkpoint": the caller's two buffers are all the state
                flat = flat.cpu().cuda()
                state = state.cpu().cuda()
        res.append((flat.clone(), state.clone()))
    assert torch.equal(res[0][0], res[1][0]) and torch.equal(res[0][1], res[1][1])


def test_hand_worked_rows_of_algorithm_1_on_the_gpu():
    # the fixture's rows (worked by hand from Algorithm 1, steps 5-6), padded with zero columns to the minimum width 4
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import os
    from paper_2508_03854_amd import TBE
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "algorithm1_worked_rows.txt")
    n = 0
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        scal, g, w0, v_new, w_new = [np.array(p.split(), dtype=np.float64) for p in line.split("|")]
        eta, eps, c, v_old = scal
        pad = lambda x: np.concatenate([x, np.zeros(4 - len(x))]) if len(x) < 4 else x
        g, w0, w_new = pad(g), pad(w0), pad(w_new)
        for dtype, tdt in (("f32", torch.float32),):
            tbe = TBE([3], [4], dtype)
            flat = torch.tensor(np.stack([w0, w0, w0]).reshape(-1), dtype=tdt, device="cuda")
            state = torch.tensor([7.0, float(v_old), 7.0], device="cuda")
            idx = torch.tensor([1], dtype=torch.int64, device="cuda")
            off = torch.tensor([0, 1], dtype=torch.int64, device="cuda")
            gout = torch.tensor(g[None, :], dtype=torch.float32, device="cuda")
            ws = tbe.alloc_workspace(1, 1)
            tbe.backward_rowwise_adagrad(gout, idx, off, 1, flat, state, ws, lr=float(eta), eps=float(eps),
                                         momentum_scale=float(c))
            torch.cuda.synchronize()
            got = flat.cpu().numpy().reshape(3, 4)
            np.testing.assert_allclose(got[1], w_new, rtol=1e-6, atol=1e-7)
            assert np.array_equal(got[0], w0.astype(np.float32)) and np.array_equal(got[2], w0.astype(np.float32))
            assert state.cpu().tolist() == [7.0, float(v_new[0]), 7.0]
            tbe.close()
        n += 1
    assert n == 5


def test_ids_repeated_inside_bags_sort_payload_per_segment(H):
    # several lookups share (row, bag): the pooled sort carries the bag, so such lookups are interchangeable - what
    # is unique is the multiset of bags per segment, and with the stable order even the sequence: both are compared
    import oracle
    from paper_2508_03854_amd import TBE
    rng = np.random.default_rng(21)
    cfg = make_cfg([6, 9], [8, 16], B=40, pooling="mean", c=1.0)
    lens = rng.integers(0, 30, size=2 * 40)
    off = torch.zeros(81, dtype=torch.int64)
    off[1:] = torch.cumsum(torch.as_tensor(lens, dtype=torch.int64), 0)
    ids = np.concatenate([rng.integers(0, cfg.rows[t], size=int(lens[t * 40:(t + 1) * 40].sum())) for t in range(2)])
    idx = torch.as_tensor(ids, dtype=torch.int64)
    keys, bag_of = oracle.linearize(cfg.rows, ids, off.numpy(), 40)
    pairs = set(zip(keys.tolist(), bag_of.tolist()))
    assert len(pairs) < len(ids) // 2                      # most (row, bag) pairs occur more than once
    tabs = H.host_tables(cfg)
    flat = H.flat_from_tables(tabs)
    state_np = np.zeros(cfg.total_rows, dtype=np.float32)
    state = torch.zeros(cfg.total_rows, device="cuda")
    tbe = TBE(cfg.rows, cfg.D, cfg.weight_dtype)
    ws = tbe.alloc_workspace(cfg.B, idx.numel())
    gout = torch.randn(cfg.B, cfg.sum_D, generator=torch.Generator().manual_seed(3))
    H.check_step(cfg, tbe, flat, state, tabs, state_np, idx, off, gout, ws)     # exact sequence, floats, untouched rows
    dbg = tbe.debug_sorted(ws, cfg.B, idx.numel())
    ks_ref, order = oracle.stable_sort(keys)
    uq, seg = oracle.run_lengths(ks_ref)
    vs = dbg["vals_sorted"].numpy()
    for u in range(len(uq)):
        got = np.sort(vs[seg[u]:seg[u + 1]])
        want = np.sort(bag_of[order[seg[u]:seg[u + 1]]])
        assert np.array_equal(got, want), f"segment {u}: bags differ as a multiset"
    tbe.close()


def test_zero_gradient_rows_at_zero_moment_with_eps_zero():
    # rows that appear in the batch with a zero gradient, moment 0, eps = 0: both sides leave them as they are (the
    # oracle's rule for step 6 at v = 0, g = 0); their neighbours with a nonzero gradient step by lr*sqrt(c)*g/||g||
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import oracle
    from paper_2508_03854_amd import TBE
    for dtype, tdt in (("f32", torch.float32), ("f16", torch.float16)):
        D = 8
        w0 = (np.arange(5 * D, dtype=np.float32).reshape(5, D) - 17.0) / 64.0
        tab = w0.astype(np.float16 if dtype == "f16" else np.float32)
        tbe = TBE([5], [D], dtype)
        flat = torch.tensor(tab.reshape(-1), dtype=tdt, device="cuda")
        state = torch.zeros(5, device="cuda")
        # bags: {0}, {1, 1}, {3}, {4}; gradient rows: zero, zero, nonzero, the negative of itself twice -> cancels for row 1
        idx = torch.tensor([0, 1, 1, 3, 4], dtype=torch.int64)
        off = torch.tensor([0, 1, 2, 3, 4, 5], dtype=torch.int64)
        g = np.zeros((5, D), dtype=np.float32)
        g[1] = 1.5
        g[2] = -1.5                       # row 1 is hit by bags 1 and 2: the two gradients cancel exactly
        g[3] = np.array([3, 0, -4, 0, 0, 0, 0, 0], dtype=np.float32)
        ws = tbe.alloc_workspace(5, 5)
        tbe.backward_rowwise_adagrad(torch.tensor(g, device="cuda"), idx.cuda(), off.cuda(), 5, flat, state, ws, lr=0.5,
                                     eps=0.0, momentum_scale=4.0)
        torch.cuda.synchronize()
        assert not tbe.poll_index_error()
        ref, v = [tab.copy()], np.zeros(5, dtype=np.float32)
        oracle.backward_rowwise_adagrad(ref, v, g, idx.numpy(), off.numpy(), 5, "sum", 0.5, 0.0, 4.0, want_indices=False)
        got = flat.cpu().numpy().reshape(5, D)
        bits = np.uint16 if dtype == "f16" else np.uint32
        for r in (0, 1, 2, 4):            # zero gradient (rows 0, 1, 4) or not in the batch (row 2): bits kept
            assert np.array_equal(got[r].view(bits), tab[r].view(bits)), (dtype, r)
            assert np.array_equal(ref[0][r].view(bits), tab[r].view(bits)), (dtype, r)
        assert np.isfinite(got).all() and np.isfinite(ref[0]).all()
        np.testing.assert_allclose(got[3].astype(np.float64), ref[0][3].astype(np.float64),
                                   rtol=1e-2 if dtype == "f16" else 1e-6, atol=1e-7)
        np.testing.assert_allclose(got[3].astype(np.float64) - tab[3].astype(np.float64), -0.5 * 2.0 * g[3] / 5.0,
                                   atol=2e-3 if dtype == "f16" else 1e-6)
        assert state.cpu().tolist() == [0.0, 0.0, 0.0, 25.0, 0.0] and v.tolist() == [0.0, 0.0, 0.0, 25.0, 0.0]
        tbe.close()


# ---- tables sorted segment by segment on their local ids (fewer key bits than the linearised key needs) ----------
def test_segmented_sort_shapes(H):
    # 3 x 250 rows: local ids need 8 bits (one radix pass), linearised keys 10 bits (two): the per-table path
    rng = np.random.default_rng(7)
    cfg = make_cfg([250, 250, 250], [8, 16, 8], B=700, pooling="sum", c=2.0)
    lens = rng.integers(0, 6, size=3 * 700)
    lens[700:1400] = 0                                    # the middle table sees no id at all
    ids = np.concatenate([rng.integers(0, 250, size=int(lens[t * 700:(t + 1) * 700].sum())) for t in range(3)])
    reps = run_custom(H, cfg, lens, ids, steps=2)
    assert reps[0]["U"] > 300
    # many small tables, some of them empty, ragged sizes that do not line up with any tile
    T = 37
    cfg = make_cfg([200 + 3 * t for t in range(T)], [8] * T, B=129, pooling="mean")
    lens = rng.integers(0, 4, size=T * 129)
    for t in (0, 5, 6, 36):
        lens[t * 129:(t + 1) * 129] = 0
    ids = np.concatenate([rng.integers(0, 200 + 3 * t, size=int(lens[t * 129:(t + 1) * 129].sum())) for t in range(T)])
    run_custom(H, cfg, lens, ids)
    # one table holds almost everything (many chunks), the others a handful of lookups
    cfg = make_cfg([255, 255, 255, 255], [8, 8, 8, 8], B=50000, pooling="sum")
    lens = np.zeros(4 * 50000, dtype=np.int64)
    lens[50000:100000] = rng.integers(8, 12, size=50000)
    lens[[3, 150001, 199999]] = 2
    ids = np.concatenate([rng.integers(0, 255, size=int(lens[t * 50000:(t + 1) * 50000].sum())) for t in range(4)])
    reps = run_custom(H, cfg, lens, ids)
    assert reps[0]["max_seg"] > 1000


def test_segmented_sort_invalid_ids_and_malformed_offsets():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2508_03854_amd import TBE
    import oracle
    rows, D, B = [250, 250, 250], [8, 8, 8], 4
    tbe = TBE(rows, D, "f32")
    g = torch.Generator().manual_seed(0)
    flat_cpu = torch.randn(750 * 8, generator=g)
    flat = flat_cpu.cuda()
    lens = [2, 1, 0, 3, 1, 1, 2, 1, 0, 2, 2, 1]
    good = torch.tensor([1, 249, 4, 0, 3, 3, 5, 0, 2, 1, 5, 7, 7, 100, 249, 3], dtype=torch.int64)
    bad = good.clone()
    bad[1] = 250                     # == rows[0]
    bad[8] = -3
    bad[14] = 100000
    off = torch.zeros(13, dtype=torch.int64)
    off[1:] = torch.cumsum(torch.tensor(lens), 0)
    state = torch.zeros(750, device="cuda")
    gout = torch.randn(B, 24, generator=g)
    ws = tbe.alloc_workspace(B, 16)
    tbe.backward_rowwise_adagrad(gout.cuda(), bad.cuda(), off.cuda(), B, flat, state, ws, lr=0.1, eps=1e-8)
    assert tbe.poll_index_error()
    keep = torch.ones(16, dtype=torch.bool)
    keep[[1, 8, 14]] = False
    lens2 = [1, 1, 0, 3, 1, 1, 1, 1, 0, 2, 1, 1]
    off2 = np.concatenate([[0], np.cumsum(lens2)])
    tabs = [flat_cpu[t * 2000:(t + 1) * 2000].view(250, 8).numpy().copy() for t in range(3)]
    st = np.zeros(750, dtype=np.float32)
    res = oracle.backward_rowwise_adagrad(tabs, st, gout.numpy(), good[keep].numpy(), off2, B, "sum", 0.1, 1e-8, 1.0)
    np.testing.assert_allclose(flat.cpu().numpy(), np.concatenate([t.reshape(-1) for t in tabs]), rtol=1e-5, atol=1e-6)
    np.testing.assert_allclose(state.cpu().numpy(), st, rtol=1e-5)
    dbg = tbe.debug_sorted(ws, B, 16)
    uq = dbg["unique_rows"].numpy()
    assert sorted(uq[uq < 750].tolist()) == res.unique_rows.tolist()      # the valid rows, each once
    assert (uq == 750).sum() == 3                                         # one pseudo-row per table that saw an invalid id
    # offsets that are not ascending: nothing may fault, the call returns, results are unspecified
    wrong = off.clone()
    wrong[4], wrong[8] = 14, 3
    flat2 = flat_cpu.cuda()
    tbe.backward_rowwise_adagrad(gout.cuda(), good.cuda(), wrong.cuda(), B, flat2, state, ws, lr=0.1, eps=1e-8)
    torch.cuda.synchronize()
    assert torch.isfinite(flat2).all()
    tbe.poll_index_error()
    tbe.close()


# ---- the hottest rows of a bag-sliced table: reduced by streaming the table's gradient block once ---------------
@pytest.mark.parametrize("dtype,pooling", [("f32", "sum"), ("f16", "mean")])
def test_dense_rows_path(H, dtype, pooling):
    rng = np.random.default_rng(11)
    B = 32768                                   # B * D * 4 = 8 MB per table: sliced over the XCDs
    cfg = make_cfg([6, 5000, 40], [64, 64, 128], dtype=dtype, B=B, pooling=pooling, c=2.0)
    lens = np.concatenate([rng.integers(2, 7, size=B),       # table 0: six rows, all of them hit ~20000 times
                           rng.integers(0, 41, size=B),      # table 1: 24 hot rows (more than one pass takes) + a tail
                           rng.integers(0, 3, size=B)])      # table 2: 40 rows with ~800 hits: long, but not dense
    n0, n1, n2 = (int(lens[t * B:(t + 1) * B].sum()) for t in range(3))
    hot = rng.integers(0, 24, size=n1)
    tail = rng.integers(24, 5000, size=n1)
    ids1 = np.where(rng.random(n1) < 0.9, hot * 7 % 5000, tail)     # hot rows scattered over the key range
    ids = np.concatenate([rng.integers(0, 6, size=n0), ids1, rng.integers(0, 40, size=n2)])
    reps = run_custom(H, cfg, lens, ids, steps=2)
    assert reps[0]["max_seg"] > 20000


def test_apply_twice_on_one_prepared_workspace_is_two_steps():
    # the row-update pass clears its own counters and tickets: run again on the same sorted batch it is one more
    # step on that batch, equal to two one-call backwards bit for bit (hot rows, dense rows and tickets included)
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2508_03854_amd import TBE
    cfg = W.config("C3", T=8, B=16384, rows_scale=0.02, c=2.0)
    idx, off = (x.cuda() for x in W.make_batch(cfg, 0))
    gout = W.make_grad_out(cfg, 0).cuda()
    tbe = TBE(cfg.rows, cfg.D, cfg.weight_dtype)
    ws = tbe.alloc_workspace(cfg.B, idx.numel())
    res = []
    for split in (False, True):
        flat = torch.empty(cfg.total_elems, device="cuda")
        W.fill_weights(cfg, flat)
        state = torch.zeros(cfg.total_rows, device="cuda")
        if split:
            tbe.backward_prepare(idx, off, cfg.B, ws)
            for _ in range(2):
                tbe.backward_apply_rowwise_adagrad(gout, off, cfg.B, idx.numel(), flat, state, ws, pooling=cfg.pooling,
                                                   lr=cfg.lr, eps=cfg.eps, momentum_scale=cfg.c)
        else:
            for _ in range(2):
                tbe.backward_rowwise_adagrad(gout, idx, off, cfg.B, flat, state, ws, pooling=cfg.pooling, lr=cfg.lr,
                                             eps=cfg.eps, momentum_scale=cfg.c)
        torch.cuda.synchronize()
        res.append((flat, state))
    assert torch.equal(res[0][0].view(torch.int32), res[1][0].view(torch.int32))
    assert torch.equal(res[0][1].view(torch.int32), res[1][1].view(torch.int32))
    tbe.close()


@pytest.mark.parametrize("dtype,pooling", [("f32", "sum"), ("f16", "mean")])
def test_more_hot_rows_than_the_partial_sum_area_holds(H, dtype, pooling):
    # thousands of rows just above the hot-row threshold in a bag-sliced table need more partial-sum slots than the
    # workspace keeps (it is sized for skewed batches): slots go out in row order, the rows left without are reduced
    # by the kernel that applies their step - same results, and the same bits on every run
    from paper_2508_03854_amd import TBE
    rng = np.random.default_rng(31)
    B = 32768                                   # B * D * 4 = 8 MB: every XCD owns an eighth of the bags
    R = 3600
    cfg = make_cfg([R, 50], [64, 64], dtype=dtype, B=B, pooling=pooling, c=1.0, lr=0.01)
    lens = np.concatenate([rng.integers(55, 64, size=B), rng.integers(0, 3, size=B)])
    n0, n1 = int(lens[:B].sum()), int(lens[B:].sum())
    ids = np.concatenate([rng.integers(0, R, size=n0), rng.integers(0, 50, size=n1)])     # ~540 lookups per row
    assert n0 / R > 515
    tbe = TBE(cfg.rows, cfg.D, dtype)
    slots_needed = 8 * R
    assert slots_needed > (n0 + n1) // 192 + 4096            # the area is too small for them
    tbe.close()
    reps = run_custom(H, cfg, lens, ids, steps=1)
    assert 512 < reps[0]["max_seg"] < 1000
    # determinism
    off = torch.zeros(2 * B + 1, dtype=torch.int64)
    off[1:] = torch.cumsum(torch.as_tensor(lens, dtype=torch.int64), 0)
    idx = torch.as_tensor(ids, dtype=torch.int64)
    gout = torch.randn(B, cfg.sum_D, generator=torch.Generator().manual_seed(2)).cuda()
    tabs = H.host_tables(cfg)
    res = []
    tbe = TBE(cfg.rows, cfg.D, dtype)
    ws = tbe.alloc_workspace(B, idx.numel())
    for _ in range(3):
        flat = H.flat_from_tables(tabs)
        state = torch.zeros(cfg.total_rows, device="cuda")
        tbe.backward_rowwise_adagrad(gout, idx.cuda(), off.cuda(), B, flat, state, ws, pooling=pooling, lr=0.01, eps=1e-8)
        torch.cuda.synchronize()
        res.append((flat, state))
    bits = torch.int32 if dtype == "f32" else torch.int16
    for k in (1, 2):
        assert torch.equal(res[0][0].view(bits), res[k][0].view(bits)) and torch.equal(res[0][1], res[k][1])
    tbe.close()


def test_sliced_ticketed_and_dense_paths_are_deterministic():
    # a batch large enough for the bag-sliced hot rows, their tickets and the dense rows, on small tables: the
    # order in which work is handed out varies from run to run, the bits of the result must not
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2508_03854_amd import TBE
    cfg = W.config("C3", T=16, B=16384, rows_scale=0.02, c=2.0)
    idx, off = (x.cuda() for x in W.make_batch(cfg, 0))
    tbe = TBE(cfg.rows, cfg.D, cfg.weight_dtype)
    ws = tbe.alloc_workspace(cfg.B, idx.numel())
    results = []
    for io in (torch.float32, torch.bfloat16):
        gout = W.make_grad_out(cfg, 0).cuda().to(io)
        runs = []
        for _ in range(3):
            flat = torch.empty(cfg.total_elems, device="cuda")
            W.fill_weights(cfg, flat)
            state = torch.zeros(cfg.total_rows, device="cuda")
            for _step in range(2):
                tbe.backward_rowwise_adagrad_ex(gout, idx, off, cfg.B, flat, state, ws, pooling=cfg.pooling, lr=cfg.lr,
                                                eps=cfg.eps, momentum_scale=cfg.c)
            torch.cuda.synchronize()
            runs.append((flat, state))
        for f, s in runs[1:]:
            assert torch.equal(f.view(torch.int32), runs[0][0].view(torch.int32))
            assert torch.equal(s.view(torch.int32), runs[0][1].view(torch.int32))
        results.append(runs[0])
    dbg = tbe.debug_sorted(ws, cfg.B, idx.numel())
    seg = dbg["seg_start"].numpy()
    assert np.diff(seg).max() > cfg.B // 8            # some row is long enough for the dense path
    tbe.close()


@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_wide_rows_with_bag_sliced_hot_rows(H, dtype):
    # 1024 columns (the wide-row kernels) and a batch large enough for the bag-sliced hot-row path at that width
    rng = np.random.default_rng(13)
    B = 8192                                     # B * 1024 * 4 = 32 MB per table: 64 sub-slices
    cfg = make_cfg([7, 300], [1024, 520 if dtype == "f16" else 516], dtype=dtype, B=B, pooling="mean", c=2.0)
    lens = rng.integers(0, 6, size=2 * B)
    n0, n1 = int(lens[:B].sum()), int(lens[B:].sum())
    ids = np.concatenate([rng.integers(0, 7, size=n0), rng.integers(0, 300, size=n1)])
    reps = run_custom(H, cfg, lens, ids)
    assert reps[0]["max_seg"] > 2000


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("pooling", ["sum", "mean"])
def test_tables_of_every_width_class_in_one_handle(H, dtype, pooling):
    # One handle with rows of 4 to 1024 columns: every forward class, both row-update kernels (each must take the
    # rows of its own width class and leave the others alone), hot rows in narrow and in wide tables, and a batch
    # large enough that the 256-column table's hottest rows take the streamed hot-row path.
    rng = np.random.default_rng(29)
    B = 8192
    v = 8 if dtype == "f16" else 4
    rows = [5, 400, 9, 1000, 3, 60, 700, 11]
    D = [1024, 4 * v, 64, 512 + v, 256, 2 * v, 768, 128]
    cfg = make_cfg(rows, D, dtype=dtype, B=B, pooling=pooling, c=4.0)
    T = len(rows)
    lens = rng.integers(0, 6, size=T * B)
    ids = np.concatenate([rng.integers(0, rows[t], size=int(lens[t * B:(t + 1) * B].sum())) for t in range(T)])
    reps = run_custom(H, cfg, lens, ids)
    assert reps[0]["max_seg"] > 4096              # rows of table 4 (256 columns) above the hot-row threshold


@pytest.mark.parametrize("name,kw,idt", [("C3", dict(T=6, B=512, rows_scale=2e-3), torch.int64),
                                         ("C5", dict(T=16, B=1024, rows_scale=1e-3), torch.int32),
                                         ("C4", dict(T=4, B=4096, rows_scale=1e-3), torch.int64)])
def test_prepare_then_apply_equals_the_one_call_backward(name, kw, idt):
    # the sort of the ids on a second stream, concurrent with the forward, then the row updates on the first one:
    # bit for bit what the one-call backward gives (which the other tests hold against the oracle)
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2508_03854_amd import TBE
    cfg = W.config(name, c=2.0, **kw)
    idx, off = (x.cuda().to(idt) for x in W.make_batch(cfg, 0))
    tbe = TBE(cfg.rows, cfg.D, cfg.weight_dtype)
    ws = tbe.alloc_workspace(cfg.B, idx.numel())
    kwargs = dict(pooling=cfg.pooling, lr=cfg.lr, eps=cfg.eps, momentum_scale=cfg.c)

    def fresh():
        flat = torch.empty(cfg.total_elems, dtype=cfg.torch_weight_dtype, device="cuda")
        W.fill_weights(cfg, flat)
        state = torch.empty(cfg.total_rows, device="cuda")
        W.fill_state(cfg, state, "hash")
        return flat, state

    f1, s1 = fresh()
    f2, s2 = fresh()
    main, side = torch.cuda.current_stream(), torch.cuda.Stream()
    out = torch.empty(cfg.B, cfg.sum_D, device="cuda")
    for step in range(2):
        gout = W.make_grad_out(cfg, step).cuda()
        tbe.backward_rowwise_adagrad_ex(gout, idx, off, cfg.B, f1, s1, ws, **kwargs)
        one = tbe.debug_sorted(ws, cfg.B, idx.numel())
        side.wait_stream(main)
        tbe.backward_prepare(idx, off, cfg.B, ws, stream=side)
        tbe.forward_ex(f2, idx, off, cfg.B, cfg.pooling, out=out)
        main.wait_stream(side)
        tbe.backward_apply_rowwise_adagrad(gout, off, cfg.B, idx.numel(), f2, s2, ws, **kwargs)
        two = tbe.debug_sorted(ws, cfg.B, idx.numel())
        torch.cuda.synchronize()
        assert not tbe.poll_index_error()
        for key in ("keys_sorted", "vals_sorted", "unique_rows", "seg_start"):
            assert torch.equal(torch.as_tensor(one[key]), torch.as_tensor(two[key])), key
        assert torch.equal(f1, f2) and torch.equal(s1, s2), f"step {step}: the two-call backward differs"
    # the same for the plain SGD step
    g1, g2 = f1.clone(), f1.clone()
    gout = W.make_grad_out(cfg, 7).cuda()
    tbe.backward_sgd(gout, idx, off, cfg.B, g1, ws, pooling=cfg.pooling, lr=cfg.lr)
    tbe.backward_prepare(idx, off, cfg.B, ws)
    tbe.backward_apply_sgd(gout, off, cfg.B, idx.numel(), g2, ws, pooling=cfg.pooling, lr=cfg.lr)
    torch.cuda.synchronize()
    assert torch.equal(g1, g2) and not torch.equal(g1, f1)
    # argument checks of the split calls
    from paper_2508_03854_amd.binding import TbeError
    with pytest.raises(TbeError):
        tbe.backward_prepare(idx, off, cfg.B, ws[:1024])
    with pytest.raises(TbeError):
        tbe.backward_apply_rowwise_adagrad(gout, off, cfg.B, idx.numel(), f2, s2, ws[:1024], **kwargs)
    tbe.close()


@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_bag_lengths_around_the_long_bag_bounds(H, dtype):
    # narrow rows take one bag per lane group unless the bag is long (more than 32 / 48 / 64 ids by lanes per row), in
    # which case a whole wavefront walks it: lengths on both sides of every bound, in every narrow-row class,
    # next to empty and short bags in the same wavefront
    rng = np.random.default_rng(41)
    v = 8 if dtype == "f16" else 4
    D = [v, 2 * v, 4 * v, 8 * v, 16 * v, 32 * v]          # 1 .. 32 lanes per row
    rows = [11, 60, 500, 37, 900, 64]
    B = 150
    cfg = make_cfg(rows, D, dtype=dtype, B=B, pooling="mean", c=2.0)
    special = [0, 1, 31, 32, 33, 47, 48, 49, 63, 64, 65, 66, 130, 500]
    lens = rng.integers(0, 9, size=len(D) * B)
    for t in range(len(D)):
        where = rng.choice(B, size=len(special), replace=False)
        lens[t * B + where] = special
    ids = np.concatenate([rng.integers(0, rows[t], size=int(lens[t * B:(t + 1) * B].sum())) for t in range(len(D))])
    run_custom(H, cfg, lens, ids)
