"""The backward entry point that allocates nothing (its scratch memory is a fixed array inside the library) against
the entry point that takes a caller's workspace: bit-identical tables and moments, on two calls in a row, the second
with a smaller batch; a batch beyond the array's size is refused."""
import ctypes

import pytest
import torch

import workloads as W

pytestmark = pytest.mark.gpu


def test_static_scratch_backward_equals_the_workspace_backward():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import gpu_harness as H
    from paper_2508_03854_amd import TBE, binding
    torch.cuda.set_device(0)
    for name, kw, kw2 in (("C2", dict(T=6, B=1024, rows_scale=0.05), dict(T=6, B=256, rows_scale=0.05)),
                          ("C4", dict(T=5, B=512, rows_scale=2e-3), dict(T=5, B=100, rows_scale=2e-3))):
        cfg = W.config(name, c=2.0, **kw)
        small = W.config(name, c=2.0, **kw2)         # same tables, smaller batch
        assert small.rows == cfg.rows and small.D == cfg.D
        tabs = H.host_tables(cfg)
        st_np = W.state_rows(cfg, torch.arange(cfg.total_rows)).numpy()
        tbe = TBE(cfg.rows, cfg.D, cfg.weight_dtype)
        f_ws, s_ws = H.flat_from_tables(tabs), torch.from_numpy(st_np.copy()).cuda()
        f_st, s_st = H.flat_from_tables(tabs), torch.from_numpy(st_np.copy()).cuda()
        for step, c in enumerate((cfg, small)):
            idx, off = W.make_batch(c, step)
            gout = W.make_grad_out(c, step).cuda()
            d_idx, d_off = idx.cuda(), off.cuda()
            need = tbe.workspace_bytes(c.B, idx.numel())
            assert need <= binding.STATIC_SCRATCH_BYTES
            ws = tbe.alloc_workspace(c.B, idx.numel())
            tbe.backward_rowwise_adagrad_ex(gout, d_idx, d_off, c.B, f_ws, s_ws, ws, pooling=c.pooling, lr=c.lr,
                                            eps=c.eps, momentum_scale=c.c)
            tbe.backward_rowwise_adagrad_static(gout, d_idx, d_off, c.B, f_st, s_st, pooling=c.pooling, lr=c.lr,
                                                eps=c.eps, momentum_scale=c.c)
            torch.cuda.synchronize()
            assert not tbe.poll_index_error()
            iv = torch.int32 if cfg.weight_dtype == "f32" else torch.int16
            assert torch.equal(f_ws.view(iv), f_st.view(iv)), f"{name} step {step}: tables differ"
            assert torch.equal(s_ws.view(torch.int32), s_st.view(torch.int32)), f"{name} step {step}: moments differ"
            assert not torch.equal(f_ws.view(iv), H.flat_from_tables(tabs).view(iv))     # the step did change rows
        tbe.close()
    # a batch whose scratch need exceeds the array: refused, nothing launched, tables untouched
    cfg = W.config("C2", T=6, B=1024, rows_scale=0.05)
    tbe = TBE(cfg.rows, cfg.D, cfg.weight_dtype)
    big_nnz = 4_000_000
    assert tbe.workspace_bytes(cfg.B, big_nnz) > binding.STATIC_SCRATCH_BYTES
    idx = torch.zeros(big_nnz, dtype=torch.int64, device="cuda")
    off = torch.zeros(cfg.T * cfg.B + 1, dtype=torch.int64, device="cuda")
    off[-1] = big_nnz
    flat = torch.zeros(cfg.total_elems, device="cuda")
    state = torch.zeros(cfg.total_rows, device="cuda")
    gout = torch.ones(cfg.B, cfg.sum_D, device="cuda")
    with pytest.raises(binding.TbeError) as e:
        tbe.backward_rowwise_adagrad_static(gout, idx, off, cfg.B, flat, state, lr=0.1, eps=1e-8)
    assert e.value.status == binding.EWORKSPACE
    torch.cuda.synchronize()
    assert float(flat.abs().sum()) == 0.0 and float(state.abs().sum()) == 0.0
    tbe.close()
