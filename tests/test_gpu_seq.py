"""GPU parity of the non-pooled lookup and its backward (tbe_lookup_seq, tbe_backward_seq_rowwise_adagrad) against
the CPU oracle: the workloads' ids read as sequences (table t owns one run of positions)."""
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


def run_seq(H, cfg, io="f32", idt=torch.int64, steps=2):
    import oracle
    from paper_2508_03854_amd import TBE
    tabs = H.host_tables(cfg)
    flat = H.flat_from_tables(tabs)
    state_np = W.state_rows(cfg, torch.arange(cfg.total_rows)).numpy()
    state = torch.from_numpy(state_np.copy()).cuda()
    tbe = TBE(cfg.rows, cfg.D, cfg.weight_dtype)
    iv = np.uint32 if cfg.weight_dtype == "f32" else np.uint16
    io_t = H._IO_TORCH[io]
    out_rep = []
    for step in range(steps):
        idx, off = W.make_batch(cfg, step)
        idx, toff, total = W.as_sequence(cfg, idx, off)
        nnz = idx.numel()
        # ---- lookup: a copy with at most one rounding, so bit-exact on the first step
        out_ref = oracle.lookup_seq(tabs, idx.numpy(), toff.numpy(), out_dtype=io)
        out = torch.full((total + 64,), 7.0, dtype=io_t, device="cuda")        # 64 guard elements behind the output
        tbe.lookup_seq(flat, idx.to(idt).cuda(), toff.to(idt).cuda(), out)
        assert not tbe.poll_index_error()
        got = H.io_to_numpy(out.cpu(), io)
        guard = H.io_to_numpy(torch.full((64,), 7.0, dtype=io_t), io)
        assert np.array_equal(got[total:].view(guard.dtype), guard), "wrote behind the output"
        bits = np.uint32 if io == "f32" else np.uint16
        if step == 0 or cfg.weight_dtype == "f32":
            same = np.array_equal(got[:total].view(bits), out_ref.view(bits))
            if step == 0:
                assert same, "lookup differs from the oracle"
        # ---- backward
        gseq = W.make_grad_seq(cfg, total, step).to(io_t)
        prev_w = flat.clone()
        prev_v = state.clone()
        U = oracle.backward_seq(tabs, state_np, H.io_to_numpy(gseq, io), idx.numpy(), toff.numpy(), cfg.lr, cfg.eps, cfg.c,
                                grad_dtype=io)
        ws = tbe.alloc_workspace(1, max(1, nnz))
        tbe.backward_seq_rowwise_adagrad(gseq.cuda(), idx.to(idt).cuda(), toff.to(idt).cuda(), flat, state, ws,
                                         lr=cfg.lr, eps=cfg.eps, momentum_scale=cfg.c)
        assert not tbe.poll_index_error()
        dbg = tbe.debug_sorted(ws, 1, nnz)
        assert dbg["num_unique"] == U
        # integer by-products: the stable sort of (row key, position)
        base = np.asarray(cfg.row_base())
        keys = np.concatenate([idx.numpy()[toff[t]:toff[t + 1]] + base[t] for t in range(cfg.T)])
        ks_ref, order = oracle.stable_sort(keys)              # the oracle's sort (pinned against the library's on the CPU)
        assert np.array_equal(dbg["keys_sorted"].numpy(), ks_ref)
        assert np.array_equal(dbg["vals_sorted"].numpy(), order)
        uq_ref, seg_ref = oracle.run_lengths(ks_ref)
        assert np.array_equal(dbg["unique_rows"].numpy(), uq_ref) and np.array_equal(dbg["seg_start"].numpy(), seg_ref)
        touched = np.zeros(cfg.total_rows, dtype=bool)
        touched[dbg["unique_rows"].numpy()] = True
        assert touched.sum() == U
        gpu_tabs = H.split_flat(flat.cpu().numpy(), cfg)
        prev_tabs = H.split_flat(prev_w.cpu().numpy(), cfg)
        rtol = H.RTOL_F32 if cfg.weight_dtype == "f32" else H.RTOL_F16
        werr = 0.0
        for t in range(cfg.T):
            m = touched[base[t]:base[t + 1]]
            assert np.array_equal(gpu_tabs[t][~m].view(iv), prev_tabs[t][~m].view(iv)), f"untouched rows of table {t} changed"
            if m.any():
                werr = max(werr, H.assert_close(gpu_tabs[t][m], tabs[t][m], rtol, cfg.w_scale, f"weights of table {t}"))
                if cfg.weight_dtype == "f16" and step == 0:
                    assert H.half_ulp_distance(gpu_tabs[t][m], tabs[t][m]).max() <= 1
        sv = state.cpu().numpy()
        assert np.array_equal(sv[~touched].view(np.uint32), prev_v.cpu().numpy()[~touched].view(np.uint32))
        verr = H.assert_close(sv[touched], state_np[touched], H.RTOL_F32, 1e-6, "moments")
        out_rep.append({"nnz": nnz, "U": U, "w_max_err": werr, "v_max_err": verr})
    tbe.close()
    return out_rep


@pytest.mark.parametrize("name,kw,io,idt", [
    ("C1", dict(), "f32", torch.int64),                                     # one table, uniform ids
    ("C2", dict(), "f32", torch.int32),                                     # 26 tables, Zipf head: rows with thousands of hits
    ("C3", dict(T=12, B=512, rows_scale=2e-3), "bf16", torch.int64),        # D in {64,128,256}
    ("C4", dict(T=8, B=256, rows_scale=1e-3), "f16", torch.int32),          # fp16 tables
    ("C5", dict(T=32, B=1024, rows_scale=1e-3), "f32", torch.int64),        # D = 128 and 32, very hot rows
])
def test_sequence_lookup_and_backward_match_oracle(H, name, kw, io, idt):
    cfg = W.config(name, c=2.0, pooling="sum", **kw)
    reps = run_seq(H, cfg, io, idt)
    print(name, io, reps, flush=True)
    assert reps[0]["U"] > 0


def test_sequence_edge_cases(H):
    import oracle
    from paper_2508_03854_amd import TBE, binding as P
    rows, D = [50, 7, 300], [8, 64, 16]
    tbe = TBE(rows, D, "f32")
    rng = np.random.default_rng(1)
    tabs = [rng.standard_normal((r, d)).astype(np.float32) for r, d in zip(rows, D)]
    flat = torch.from_numpy(np.concatenate([a.reshape(-1) for a in tabs])).cuda()
    # empty middle table, a run shorter than a wavefront, and a table boundary inside one wavefront's 64 positions
    ns = [70, 0, 3]
    toff = torch.tensor(np.concatenate([[0], np.cumsum(ns)]), dtype=torch.int64)
    idx = torch.tensor(np.concatenate([rng.integers(0, r, size=n) for r, n in zip(rows, ns)]), dtype=torch.int64)
    total = sum(n * d for n, d in zip(ns, D))
    out = torch.zeros(total, device="cuda")
    tbe.lookup_seq(flat, idx.cuda(), toff.cuda(), out)
    ref = oracle.lookup_seq(tabs, idx.numpy(), toff.numpy())
    assert np.array_equal(out.cpu().numpy().view(np.uint32), ref.view(np.uint32))
    # no lookups at all
    e_idx = torch.zeros(0, dtype=torch.int64, device="cuda")
    e_off = torch.zeros(4, dtype=torch.int64, device="cuda")
    tbe.lookup_seq(flat, e_idx, e_off, torch.zeros(0, device="cuda"))
    state = torch.zeros(sum(rows), device="cuda")
    ws = tbe.alloc_workspace(1, 1)
    before = flat.clone()
    tbe.backward_seq_rowwise_adagrad(torch.zeros(0, device="cuda"), e_idx, e_off, flat, state, ws, lr=0.1, eps=1e-8)
    assert torch.equal(flat, before)
    # an id outside its table: zero row, error flag; the backward skips it
    bad = idx.clone()
    bad[5] = 50
    out.fill_(3.0)
    tbe.lookup_seq(flat, bad.cuda(), toff.cuda(), out)
    assert tbe.poll_index_error()
    o = out.cpu().numpy()
    assert np.all(o[5 * 8:6 * 8] == 0.0)
    good = np.ones(total, bool)
    good[5 * 8:6 * 8] = False
    assert np.array_equal(o[good].view(np.uint32), ref[good].view(np.uint32))
    # offsets that do not ascend from 0 to nnz: flagged, nothing written outside the buffer, nothing updated
    wrong = torch.tensor([0, 80, 60, 73], dtype=torch.int64)
    guard = torch.full((total + 4096,), 5.0, device="cuda")
    st = P.load_library().tbe_lookup_seq(tbe._h, flat.data_ptr(), idx.cuda().data_ptr(), wrong.cuda().data_ptr(), P.I64, 73,
                                         guard.data_ptr(), P.IO_F32, total, torch.cuda.current_stream().cuda_stream)
    assert st == P.OK
    torch.cuda.synchronize()
    assert float(guard[total:].min()) == 5.0 and float(guard[total:].max()) == 5.0
    tbe.poll_index_error()
    ws = tbe.alloc_workspace(1, 73)
    before = flat.clone()
    g = torch.randn(total, device="cuda")
    tbe.backward_seq_rowwise_adagrad(g, idx.cuda(), wrong.cuda(), flat, state, ws, lr=0.1, eps=1e-8)
    assert tbe.poll_index_error()
    assert torch.equal(flat, before) and float(state.abs().max()) == 0.0
    tbe.close()


@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_sequence_tables_of_every_width_class(H, dtype):
    # rows of 8 to 1024 columns in one handle: both row-update kernels in the non-pooled layout, with rows that take
    # hundreds of lookups in a narrow and in a wide table
    v = 8 if dtype == "f16" else 4
    cfg = W.Config("seqmix", [40, 300, 9, 1000, 6], [1024, 2 * v, 512 + v, 64, 256], dtype, 512, "sum",
                   ("poisson1", 6.0), ("zipf", 1.1))
    cfg.c = 2.0
    reps = run_seq(H, cfg, "f32", torch.int64)
    print("seqmix", dtype, reps, flush=True)
    assert reps[0]["U"] > 300
