"""GPU parity of the extended entry points (tbe_forward_ex, tbe_backward_rowwise_adagrad_ex): int32 ids and
offsets, and binary16 / bfloat16 pooled output and upstream gradient, against the CPU oracle."""
import ctypes

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


def test_c1_int32_ids_are_bit_identical_to_int64(H):
    from paper_2508_03854_amd import TBE
    cfg = W.config("C1")
    reps = H.run_config(cfg, steps=2, index_dtype=torch.int32)
    print("C1 int32", reps, flush=True)
    # and the two id widths give the same bits on the device
    tabs = H.host_tables(cfg)
    idx, off = W.make_batch(cfg, 0)
    gout = W.make_grad_out(cfg, 0).cuda()
    tbe = TBE(cfg.rows, cfg.D, cfg.weight_dtype)
    ws = tbe.alloc_workspace(cfg.B, idx.numel())
    results = []
    for dt in (torch.int64, torch.int32):
        flat = H.flat_from_tables(tabs)
        state = torch.zeros(cfg.total_rows, device="cuda")
        out = tbe.forward_ex(flat, idx.to(dt).cuda(), off.to(dt).cuda(), cfg.B)
        tbe.backward_rowwise_adagrad_ex(gout, idx.to(dt).cuda(), off.to(dt).cuda(), cfg.B, flat, state, ws,
                                        lr=cfg.lr, eps=cfg.eps)
        results.append((out.cpu(), flat.cpu(), state.cpu()))
    for a, b in zip(*results):
        assert torch.equal(a.view(torch.int32), b.view(torch.int32))
    tbe.close()


@pytest.mark.parametrize("index_dtype,io", [(torch.int32, "bf16"), (torch.int64, "f16"), (torch.int32, "f16"),
                                             (torch.int64, "bf16")])
def test_c2_full_size_variants(H, index_dtype, io):
    # Zipf head: covers the short, whole-wave and split long-row paths with a 16-bit gradient
    cfg = W.config("C2")
    reps = H.run_config(cfg, steps=2, index_dtype=index_dtype, io=io)
    print("C2", index_dtype, io, reps, flush=True)
    assert reps[0]["max_seg"] > 1000


@pytest.mark.parametrize("name,kw,index_dtype,io", [
    ("C3", dict(T=12, B=512, rows_scale=2e-3), torch.int32, "bf16"),
    ("C4", dict(T=8, B=256, rows_scale=1e-3), torch.int32, "bf16"),      # fp16 tables, 16-bit activations: the usual mix
    ("C4", dict(T=8, B=256, rows_scale=1e-3), torch.int64, "f16"),
    ("C5", dict(T=32, B=1024, rows_scale=1e-3), torch.int32, "f16"),     # mean pooling, D=32 tables
])
def test_scaled_config_variants(H, name, kw, index_dtype, io):
    cfg = W.config(name, c=2.0, **kw)
    reps = H.run_config(cfg, steps=2, state_kind="hash", index_dtype=index_dtype, io=io)
    print(name, index_dtype, io, reps, flush=True)


def test_mixed_or_unknown_dtypes_are_rejected(H):
    from paper_2508_03854_amd import TBE, binding as P
    tbe = TBE([16], [8], "f32")
    flat = torch.zeros(16 * 8, device="cuda")
    idx = torch.zeros(4, dtype=torch.int32, device="cuda")
    off64 = torch.tensor([0, 4], dtype=torch.int64, device="cuda")
    with pytest.raises(TypeError):
        tbe.forward_ex(flat, idx, off64, 1)
    with pytest.raises(TypeError):
        tbe.forward_ex(flat, idx, off64.to(torch.int32), 1, out=torch.zeros(1, 8, dtype=torch.float64, device="cuda"))
    # unknown enum values straight through the C ABI: an error status, nothing launched
    L = P.load_library()
    out = torch.full((1, 8), 7.0, device="cuda")
    off = off64.to(torch.int32)
    st = L.tbe_forward_ex(tbe._h, flat.data_ptr(), None, idx.data_ptr(), off.data_ptr(), 5, 1, 4, 0, out.data_ptr(), 0,
                          torch.cuda.current_stream().cuda_stream)
    assert st == P.EDTYPE
    st = L.tbe_forward_ex(tbe._h, flat.data_ptr(), None, idx.data_ptr(), off.data_ptr(), 1, 1, 4, 0, out.data_ptr(), 9,
                          torch.cuda.current_stream().cuda_stream)
    assert st == P.EDTYPE
    ws = tbe.alloc_workspace(1, 4)
    state = torch.zeros(16, device="cuda")
    st = L.tbe_backward_rowwise_adagrad_ex(tbe._h, out.data_ptr(), 3, idx.data_ptr(), off.data_ptr(), 1, 1, 4, 0,
                                           ctypes.c_float(0.1), ctypes.c_float(1e-8), ctypes.c_float(1.0),
                                           flat.data_ptr(), state.data_ptr(), ws.data_ptr(), ws.numel(),
                                           torch.cuda.current_stream().cuda_stream)
    assert st == P.EDTYPE
    torch.cuda.synchronize()
    assert float(out.min()) == 7.0 and float(flat.abs().max()) == 0.0
    tbe.close()
