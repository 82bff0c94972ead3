"""The largest batch the ABI's 32-bit positions are meant to carry: more than 2^31 lookups in one call (the limit is
2^32 - 2^16).  Tables are small so that the lookups, not the weights, fill the memory.  The oracle checks sampled bags
and sampled rows one by one; the integer by-products are compared, table by table, with the library's stable sort."""
import numpy as np
import pytest
import torch

import workloads as W

pytestmark = pytest.mark.gpu


def _close(got, ref, rtol, scale, what):
    got, ref = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    err = np.abs(got - ref)
    tol = rtol * np.abs(ref) + rtol * scale
    assert (err <= tol).all(), f"{what}: max err {err.max():.3e} (tol {tol[np.argmax(err - tol)]:.3e})"


def test_more_than_two_to_the_31_lookups():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import gc
    gc.collect()
    torch.cuda.empty_cache()
    free, _ = torch.cuda.mem_get_info()
    if free < 240e9:
        pytest.skip("needs 240 GB of free HBM")
    import oracle
    from paper_2508_03854_amd import TBE
    dev = "cuda"
    T, B = 64, 1 << 21
    rows = [64, 1000, 50_000, 5_000_000] * (T // 4)
    D = [8, 4, 16, 4] * (T // 4)
    cfg = W.Config("MAX", rows, D, "f32", B, "sum", ("poisson1", 16.0), ("uniform",))
    cfg.c, cfg.lr = 2.0, 0.01
    doff, rbase, woff = cfg.D_offsets(), cfg.row_base(), cfg.w_offsets()
    rng = np.random.default_rng(0)

    flat = torch.empty(cfg.total_elems, dtype=torch.float32, device=dev)
    W.fill_weights(cfg, flat)
    state = torch.empty(cfg.total_rows, dtype=torch.float32, device=dev)
    W.fill_state(cfg, state, "hash")
    state0 = state.clone()
    idx, off = W.make_batch(cfg, 0, device=dev)
    gout = W.make_grad_out(cfg, 0, device=dev)
    nnz = idx.numel()
    assert (1 << 31) < nnz <= (1 << 32) - (1 << 16)
    tbe = TBE(cfg.rows, cfg.D, "f32")
    ws = tbe.alloc_workspace(B, nnz)
    print("nnz %d (2^31 + %d), workspace %.1f GB" % (nnz, nnz - (1 << 31), ws.numel() / 1e9), flush=True)

    def init_rows(t, ids):
        return W.weight_rows(cfg, t, torch.as_tensor(ids, dtype=torch.int64)).numpy()

    # ------------------------------------------------------------------ forward, sampled bags (also the last ones)
    out = tbe.forward(flat, idx, off, B, "sum")
    torch.cuda.synchronize()
    assert not tbe.poll_index_error()
    off_cpu = off.cpu().numpy()
    bags = set(rng.integers(0, T * B, size=100).tolist()) | {0, T * B - 1, T * B - 2, (T - 1) * B, (T // 2) * B}
    for bag in sorted(bags):
        t, b = divmod(bag, B)
        ids = idx[off_cpu[bag]:off_cpu[bag + 1]].cpu().numpy()
        uniq, inv = np.unique(ids, return_inverse=True)
        ref = oracle.forward_bag(np.ascontiguousarray(init_rows(t, uniq)), inv.astype(np.int64), 0, len(ids), "sum")
        _close(out[b, doff[t]:doff[t + 1]].cpu().numpy(), ref, 1e-5, cfg.w_scale, f"forward bag {bag}")
    print("forward: %d sampled bags ok" % len(bags), flush=True)
    del out

    # ------------------------------------------------------------------ backward
    tbe.backward_rowwise_adagrad(gout, idx, off, B, flat, state, ws, pooling="sum", lr=cfg.lr, eps=cfg.eps,
                                 momentum_scale=cfg.c)
    torch.cuda.synchronize()
    assert not tbe.poll_index_error()

    # integer by-products: table t owns positions [p0, p1) before and after the sort; inside them the sorted keys and
    # bag ids must be what the library's stable sort makes of the definition of the key
    import ctypes
    ptrs = [ctypes.c_void_p() for _ in range(5)]
    st = tbe._lib.tbe_debug_sorted(tbe._h, ws.data_ptr(), B, nnz, *[ctypes.byref(p) for p in ptrs])
    assert st == 0

    def u32_view(p, first, n):      # n values starting at element `first` of a uint32 array inside the workspace
        o = p.value - ws.data_ptr() + 4 * first
        return ws[o:o + 4 * n].view(torch.int32).to(torch.int64) & 0xFFFFFFFF

    U = int(u32_view(ptrs[4], 0, 1).item())
    uq = u32_view(ptrs[2], 0, U)
    ss = u32_view(ptrs[3], 0, U + 1)
    assert int(ss[0]) == 0 and int(ss[-1]) == nnz and bool((uq[1:] > uq[:-1]).all())
    u0 = 0
    for t in range(T):
        p0, p1 = int(off_cpu[t * B]), int(off_cpu[(t + 1) * B])
        keys = idx[p0:p1] + rbase[t]
        bag_of = torch.repeat_interleave(torch.arange(t * B, (t + 1) * B, device=dev), off[t * B + 1:(t + 1) * B + 1] - off[t * B:(t + 1) * B])
        want_k, order = torch.sort(keys, stable=True)
        assert bool((u32_view(ptrs[0], p0, p1 - p0) == want_k).all()), f"table {t}: sorted keys differ"
        assert bool((u32_view(ptrs[1], p0, p1 - p0) == bag_of[order]).all()), f"table {t}: sorted bag ids differ"
        head = torch.ones(p1 - p0, dtype=torch.bool, device=dev)
        head[1:] = want_k[1:] != want_k[:-1]
        hp = head.nonzero().squeeze(1)
        n_u = hp.numel()
        assert bool((uq[u0:u0 + n_u] == want_k[hp]).all()) and bool((ss[u0:u0 + n_u] == hp + p0).all()), f"table {t}: segments differ"
        u0 += n_u
        del keys, bag_of, want_k, order, head, hp
    assert u0 == U
    print("sort / dedup / segments ok for all %d tables: U=%d, longest segment %d" % (T, U, int((ss[1:] - ss[:-1]).max())), flush=True)

    # the moments that changed are exactly those of unique_rows
    changed = (state != state0).nonzero().squeeze(1)
    assert changed.numel() == U and bool((changed == uq).all())
    del changed

    # sampled rows of one table of every size class, and of the last table
    for t in (0, 1, 2, 3, T - 1):
        R, Dt = cfg.rows[t], cfg.D[t]
        p0, p1 = int(off_cpu[t * B]), int(off_cpu[(t + 1) * B])
        ids_t = idx[p0:p1]
        u_ids, cnt = torch.unique(ids_t, return_counts=True)
        picks = {int(u_ids[torch.argmax(cnt)]), int(u_ids[torch.argmin(cnt)]), int(u_ids[0]), int(u_ids[-1])}
        picks |= set(u_ids[torch.as_tensor(rng.integers(0, u_ids.numel(), size=4))].tolist())
        ids_np = ids_t.cpu().numpy()
        off_t = off_cpu[t * B:(t + 1) * B + 1] - off_cpu[t * B]
        g_block = np.ascontiguousarray(gout[:, doff[t]:doff[t + 1]].cpu().numpy())
        cur = flat[woff[t]:woff[t + 1]].view(R, Dt)
        for r in sorted(picks):
            g, hits = oracle.row_gradient_by_scan(0, r, Dt, 0, g_block, ids_np, off_t, B, "sum")
            assert hits == int(cnt[(u_ids == r).nonzero()[0, 0]])
            row = np.ascontiguousarray(init_rows(t, [r]))
            v = W.state_rows(cfg, torch.tensor([rbase[t] + r])).numpy().copy()
            oracle.adagrad_row(row, 0, v, g, cfg.lr, cfg.eps, cfg.c)
            _close(cur[r].cpu().numpy(), row[0], 1e-5, cfg.w_scale, f"table {t} row {r} ({hits} lookups) weights")
            _close(state[rbase[t] + r].item(), v[0], 1e-5, 1e-6, f"table {t} row {r} moment")
        # rows outside the batch keep their bits
        touched = torch.zeros(R, dtype=torch.bool, device=dev)
        touched[ids_t] = True
        init = W.weight_rows(cfg, t, torch.arange(R, device=dev))
        assert not bool(((cur != init).any(1) & ~touched).any()), f"table {t}: a row outside the batch changed"
        print("table %d (R=%d, D=%d): %d sampled rows ok" % (t, R, Dt, len(picks)), flush=True)
        del touched, init, ids_t, u_ids, cnt
    tbe.close()
