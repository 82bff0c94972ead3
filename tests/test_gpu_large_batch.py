"""GPU parity at batch sizes where a table's gradient block (B x D elements) is larger than one 4 MiB L2 cache, so
that the hot-row kernels take their bag-sliced form (every XCD reduces its eighth of the bags, dense rows are
streamed), against the CPU oracle element by element.  Small enough for the oracle: a few tables, scaled row counts."""
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


@pytest.mark.parametrize("name,kw,opts", [
    # fp16 tables, D in {128, 256}: B x 256 x 4 bytes = 4 MiB blocks
    ("C4", dict(T=4, B=4096, rows_scale=0.03), dict()),
    # B not a multiple of 8: the last XCD's share of the bags is shorter
    ("C4", dict(T=3, B=4099, rows_scale=0.02), dict()),
    # 16-bit gradients, int32 ids
    ("C4", dict(T=3, B=8192, rows_scale=0.03), dict(io="bf16", index_dtype=torch.int32)),
    ("C4", dict(T=3, B=8192, rows_scale=0.03), dict(io="f16")),
    # mean pooling, fp32 tables, D = 128 (4 MiB blocks) and D = 32, long-tailed bag lengths
    ("C5", dict(T=16, B=8192, rows_scale=2e-3), dict()),
    # fp32 tables of mixed widths 64 / 128 / 256
    ("C3", dict(T=6, B=8192, rows_scale=5e-3), dict()),
])
def test_large_batch_against_oracle(H, name, kw, opts):
    cfg = W.config(name, c=2.0, **kw)
    assert any(cfg.B * d * (2 if opts.get("io", "f32") != "f32" else 4) > (3 << 20) for d in cfg.D)
    reps = H.run_config(cfg, steps=2, state_kind="hash", **opts)
    print(name, kw, reps, flush=True)
    assert reps[0]["U"] > 1000


def test_large_batch_sgd_and_split_calls(H):
    """The same shapes through the plain SGD step, and through prepare + apply: bit-identical to the one-call form."""
    from paper_2508_03854_amd import TBE
    import oracle
    cfg = W.config("C4", T=3, B=4096, rows_scale=0.03)
    tabs = H.host_tables(cfg)
    idx, off = W.make_batch(cfg, 0)
    gout = W.make_grad_out(cfg, 0)
    tbe = TBE(cfg.rows, cfg.D, cfg.weight_dtype)
    ws = tbe.alloc_workspace(cfg.B, idx.numel())
    d_idx, d_off, d_go = idx.cuda(), off.cuda(), gout.cuda()
    # SGD against the oracle
    flat = H.flat_from_tables(tabs)
    tbe.backward_sgd(d_go, d_idx, d_off, cfg.B, flat, ws, pooling=cfg.pooling, lr=cfg.lr)
    ref = [t.copy() for t in tabs]
    oracle.backward_rowwise_adagrad(ref, None, gout.numpy(), idx.numpy(), off.numpy(), cfg.B, cfg.pooling, cfg.lr, 0.0,
                                    1.0, want_indices=False)
    got = H.split_flat(flat.cpu().numpy(), cfg)
    for t in range(cfg.T):
        H.assert_close(got[t], ref[t], H.RTOL_F16, cfg.w_scale, f"sgd weights of table {t}")
    # prepare + apply == one call, bit for bit
    st_np = W.state_rows(cfg, torch.arange(cfg.total_rows)).numpy()
    f1, s1 = H.flat_from_tables(tabs), torch.from_numpy(st_np.copy()).cuda()
    f2, s2 = H.flat_from_tables(tabs), torch.from_numpy(st_np.copy()).cuda()
    tbe.backward_rowwise_adagrad(d_go, d_idx, d_off, cfg.B, f1, s1, ws, pooling=cfg.pooling, lr=cfg.lr, eps=cfg.eps,
                                 momentum_scale=2.0)
    tbe.backward_prepare(d_idx, d_off, cfg.B, ws)
    tbe.backward_apply_rowwise_adagrad(d_go, d_off, cfg.B, idx.numel(), f2, s2, ws, pooling=cfg.pooling, lr=cfg.lr,
                                       eps=cfg.eps, momentum_scale=2.0)
    torch.cuda.synchronize()
    assert torch.equal(f1.view(torch.int16), f2.view(torch.int16))
    assert torch.equal(s1.view(torch.int32), s2.view(torch.int32))
    # and twice the same call: bit-identical (no dependence on scheduling)
    f3, s3 = H.flat_from_tables(tabs), torch.from_numpy(st_np.copy()).cuda()
    tbe.backward_rowwise_adagrad(d_go, d_idx, d_off, cfg.B, f3, s3, ws, pooling=cfg.pooling, lr=cfg.lr, eps=cfg.eps,
                                 momentum_scale=2.0)
    torch.cuda.synchronize()
    assert torch.equal(f1.view(torch.int16), f3.view(torch.int16))
    assert torch.equal(s1.view(torch.int32), s3.view(torch.int32))
    tbe.close()
