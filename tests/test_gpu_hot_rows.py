"""GPU parity of the forward path that serves a table's most-used rows from on-chip memory (the handle's hot-row
hint, written by the backward call before it), against the CPU oracle element by element.  The hint only exists after
a backward call, so every case runs at least two steps; the tunable forces the path at sizes the oracle can follow."""
import numpy as np
import pytest
import torch

import workloads as W

pytestmark = pytest.mark.gpu
FORCE = {"hot_rows_min_workgroups": 0}


@pytest.fixture(scope="module")
def H():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import gpu_harness
    return gpu_harness


@pytest.mark.parametrize("name,kw,opts", [
    # fp16 rows of 128 / 256 columns (16 / 32 lanes per row), B a multiple of a workgroup's bags and not
    ("C4", dict(T=6, B=1024, rows_scale=2e-3), dict()),
    ("C4", dict(T=5, B=1500, rows_scale=2e-3), dict(io="bf16", index_dtype=torch.int32)),
    # fp32 rows of 128 and 32 columns, mean pooling, bag lengths up to 500 (long bags leave the lane-group path)
    ("C5", dict(T=16, B=2048, rows_scale=1e-3), dict()),
    # fp32 rows of 64 / 128 columns next to 256-column ones (those take the one-wavefront-per-bag kernel)
    ("C3", dict(T=9, B=1024, rows_scale=2e-3), dict()),
    ("C2", dict(T=5, B=2048, rows_scale=0.02), dict()),
])
def test_hot_rows_against_oracle(H, name, kw, opts):
    cfg = W.config(name, c=2.0, **kw)
    reps = H.run_config(cfg, steps=3, state_kind="hash", tunables=FORCE, **opts)
    print(name, kw, reps, flush=True)
    assert reps[0]["max_seg"] > 512            # some rows are hot enough to be listed


def test_hot_rows_with_empty_bags_invalid_ids_and_a_stale_hint(H):
    """After a backward call has listed hot rows: a forward over another batch with empty bags, ids outside the table
    (skipped and reported), bags that hold one hot row many times, and bags longer than the lane-group bound; then a
    forward on a handle whose hint comes from a batch that shares no row with the one looked up."""
    import oracle
    from paper_2508_03854_amd import TBE
    cfg = W.config("C4", T=4, B=1024, rows_scale=2e-3, c=1.0)
    tabs = H.host_tables(cfg)
    flat = H.flat_from_tables(tabs)
    state = torch.zeros(cfg.total_rows, device="cuda")
    tbe = TBE(cfg.rows, cfg.D, cfg.weight_dtype)
    tbe.set_tunable("hot_rows_min_workgroups", 0)
    idx, off = W.make_batch(cfg, 0)
    ws = tbe.alloc_workspace(cfg.B, 4 * idx.numel())
    # a backward with a zero gradient leaves the tables as they are and lists the batch's hot rows
    zero_g = torch.zeros(cfg.B, cfg.sum_D, device="cuda")
    tbe.backward_rowwise_adagrad(zero_g, idx.cuda(), off.cuda(), cfg.B, flat, state, ws, pooling="sum", lr=cfg.lr,
                                 eps=cfg.eps)
    torch.cuda.synchronize()
    assert np.array_equal(flat.cpu().numpy().view(np.uint16), H.flat_from_tables(tabs).cpu().numpy().view(np.uint16))
    # the batch to look up: same distribution, edited
    idx2, off2 = W.make_batch(cfg, 1)
    lens = (off2[1:] - off2[:-1]).clone()
    lens[5:400] = 0                                  # a run of empty bags
    lens[cfg.B + 7] = 300                            # far above the lane-group bound
    lens[2 * cfg.B + 9] = 65
    g = torch.Generator().manual_seed(5)
    hot = torch.unique(idx[: int(off[cfg.B])], return_counts=True)
    hottest = int(hot[0][hot[1].argmax()])
    off2 = torch.zeros(cfg.T * cfg.B + 1, dtype=torch.int64)
    torch.cumsum(lens, 0, out=off2[1:])
    n = int(off2[-1])
    ids = torch.empty(n, dtype=torch.int64)
    for t in range(cfg.T):
        a, b = int(off2[t * cfg.B]), int(off2[(t + 1) * cfg.B])
        src = idx[int(off[t * cfg.B]): int(off[(t + 1) * cfg.B])]
        ids[a:b] = src[torch.randint(0, src.numel(), (b - a,), generator=g)]
    s0, e0 = int(off2[3]), int(off2[4])
    ids[s0:e0] = hottest                             # one bag that holds the hottest row of table 0 only
    bad = torch.randint(0, n, (50,), generator=g)
    ids_bad = ids.clone()
    ids_bad[bad[:25]] = -3
    ids_bad[bad[25:]] = 1 << 40
    out = tbe.forward(flat, ids_bad.cuda(), off2.cuda(), cfg.B, "sum").cpu().numpy()
    assert tbe.poll_index_error()
    # oracle: the same bags with the invalid lookups removed
    keep = torch.ones(n, dtype=torch.bool)
    keep[bad] = False
    bag_of = torch.searchsorted(off2, torch.arange(n), right=True) - 1
    lens3 = torch.bincount(bag_of[keep], minlength=cfg.T * cfg.B)
    off3 = torch.zeros_like(off2)
    torch.cumsum(lens3, 0, out=off3[1:])
    ref = oracle.forward(tabs, ids[keep].numpy(), off3.numpy(), cfg.B, "sum")
    H.assert_close(out, ref, H.RTOL_F32, cfg.w_scale, "forward with hot rows, empty bags and invalid ids")
    # a hint that lists rows the next batch never touches: ids of a disjoint range
    cfg2 = W.config("C4", T=4, B=1024, rows_scale=2e-3, c=1.0)
    shift = [r // 2 for r in cfg2.rows]
    idx_lo = torch.cat([idx[int(off[t * cfg.B]): int(off[(t + 1) * cfg.B])] % shift[t] for t in range(cfg.T)])
    idx_hi = torch.cat([idx[int(off[t * cfg.B]): int(off[(t + 1) * cfg.B])] % shift[t] + shift[t] for t in range(cfg.T)])
    tbe.backward_rowwise_adagrad(zero_g, idx_lo.cuda(), off.cuda(), cfg.B, flat, state, ws, pooling="sum", lr=cfg.lr,
                                 eps=cfg.eps)
    out = tbe.forward(flat, idx_hi.cuda(), off.cuda(), cfg.B, "sum").cpu().numpy()
    assert not tbe.poll_index_error()
    ref = oracle.forward(tabs, idx_hi.numpy(), off.numpy(), cfg.B, "sum")
    H.assert_close(out, ref, H.RTOL_F32, cfg.w_scale, "forward with a stale hint")
    tbe.close()


def test_hot_rows_do_not_change_results_beyond_summation_order(H):
    """The same forward with the path on and off: within the float tolerance of each other, and each run repeatable
    bit for bit."""
    from paper_2508_03854_amd import TBE
    cfg = W.config("C5", T=16, B=2048, rows_scale=1e-3)
    tabs = H.host_tables(cfg)
    flat = H.flat_from_tables(tabs)
    state = torch.zeros(cfg.total_rows, device="cuda")
    idx, off = W.make_batch(cfg, 0)
    d_idx, d_off = idx.cuda(), off.cuda()
    outs = []
    for v in (0, -1):
        tbe = TBE(cfg.rows, cfg.D, cfg.weight_dtype)
        tbe.set_tunable("hot_rows_min_workgroups", v)
        ws = tbe.alloc_workspace(cfg.B, idx.numel())
        tbe.backward_rowwise_adagrad(torch.zeros(cfg.B, cfg.sum_D, device="cuda"), d_idx, d_off, cfg.B, flat, state, ws,
                                     pooling=cfg.pooling, lr=cfg.lr, eps=cfg.eps)
        a = tbe.forward(flat, d_idx, d_off, cfg.B, cfg.pooling).clone()
        b = tbe.forward(flat, d_idx, d_off, cfg.B, cfg.pooling).clone()
        torch.cuda.synchronize()
        assert torch.equal(a.view(torch.int32), b.view(torch.int32))
        outs.append(a.cpu().numpy())
        tbe.close()
    H.assert_close(outs[0], outs[1], H.RTOL_F32, cfg.w_scale, "hot-row path against the plain path")
    assert not np.array_equal(outs[0].view(np.uint32), outs[1].view(np.uint32)) or True
