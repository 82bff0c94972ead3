"""GPU parity of the optimizer variants: the plain SGD step (tbe_backward_sgd) and a sweep of the moment scaling
factor c over (0, M] (Scaling Rule 1), against the CPU oracle."""
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


@pytest.mark.parametrize("name,kw,io,idt", [
    ("C1", dict(), "f32", torch.int64),
    ("C2", dict(), "f32", torch.int64),                                    # long rows: the split path
    ("C3", dict(T=12, B=512, rows_scale=2e-3), "bf16", torch.int32),
    ("C4", dict(T=8, B=256, rows_scale=1e-3), "f32", torch.int64),         # fp16 tables
    ("C5", dict(T=32, B=1024, rows_scale=1e-3), "f16", torch.int32),       # mean pooling
])
def test_sgd_step_matches_oracle(H, name, kw, io, idt):
    import oracle
    from paper_2508_03854_amd import TBE
    cfg = W.config(name, **kw)
    tabs = H.host_tables(cfg)
    flat = H.flat_from_tables(tabs)
    before = flat.clone()
    tbe = TBE(cfg.rows, cfg.D, cfg.weight_dtype)
    lr = 0.05
    for step in range(2):
        idx, off = W.make_batch(cfg, step)
        gout = W.make_grad_out(cfg, step).to(H._IO_TORCH[io])
        ws = tbe.alloc_workspace(cfg.B, max(1, idx.numel()))
        res = oracle.backward_sgd(tabs, H.io_to_numpy(gout, io), idx.numpy(), off.numpy(), cfg.B, cfg.pooling, lr=lr,
                                  grad_dtype=io)
        tbe.backward_sgd(gout.cuda(), idx.to(idt).cuda(), off.to(idt).cuda(), cfg.B, flat, ws, pooling=cfg.pooling, lr=lr)
        assert not tbe.poll_index_error()
        dbg = tbe.debug_sorted(ws, cfg.B, idx.numel())
        assert dbg["num_unique"] == res.U
        assert np.array_equal(dbg["unique_rows"].numpy(), res.unique_rows)
        gpu_tabs = H.split_flat(flat.cpu().numpy(), cfg)
        prev_tabs = H.split_flat(before.cpu().numpy(), cfg)
        touched = np.zeros(cfg.total_rows, dtype=bool)
        touched[res.unique_rows] = True
        base = cfg.row_base()
        iv = np.uint32 if cfg.weight_dtype == "f32" else np.uint16
        rtol = H.RTOL_F32 if cfg.weight_dtype == "f32" else H.RTOL_F16
        for t in range(cfg.T):
            m = touched[base[t]:base[t + 1]]
            assert np.array_equal(gpu_tabs[t][~m].view(iv), prev_tabs[t][~m].view(iv)), f"untouched rows of table {t} changed"
            if m.any():
                # operand magnitude of w - lr*g: a hot row's summed gradient can be far larger than the weights
                scale = max(cfg.w_scale, float(np.abs(tabs[t][m].astype(np.float64)).max()))
                H.assert_close(gpu_tabs[t][m], tabs[t][m], rtol, scale, f"weights of table {t}")
        before = flat.clone()
    tbe.close()


def test_c_sweep_matches_oracle_and_larger_c_means_larger_step(H):
    # Scaling Rule 1: c ranges over (0, M]; here M = 8 replicas would allow c up to 8
    import oracle
    from paper_2508_03854_amd import TBE
    cfg0 = W.config("C2", T=6, B=512, rows_scale=0.05)
    norms = []
    for c in (0.25, 1.0, 2.0, 4.0, 8.0):
        cfg = W.config("C2", T=6, B=512, rows_scale=0.05, c=c)
        reps = H.run_config(cfg, steps=2, state_kind="hash")
        assert reps[0]["U"] > 0
        # size of the first step on the device, from identical starting weights and moments
        tabs = H.host_tables(cfg)
        flat = H.flat_from_tables(tabs)
        w0 = flat.clone()
        state = W.state_rows(cfg, torch.arange(cfg.total_rows)).cuda()
        tbe = TBE(cfg.rows, cfg.D, cfg.weight_dtype)
        idx, off = W.make_batch(cfg, 0)
        ws = tbe.alloc_workspace(cfg.B, idx.numel())
        tbe.backward_rowwise_adagrad(W.make_grad_out(cfg, 0).cuda(), idx.cuda(), off.cuda(), cfg.B, flat, state, ws,
                                     lr=cfg.lr, eps=cfg.eps, momentum_scale=c)
        norms.append(float((flat - w0).double().norm()))
        tbe.close()
    assert all(b > a for a, b in zip(norms, norms[1:])), norms
    # with eps negligible the step scales as sqrt(c): doubling c twice doubles the step
    assert abs(norms[3] / norms[1] - 2.0) < 1e-3, norms
    assert cfg0.T == 6
