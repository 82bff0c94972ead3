"""GPU parity of Algorithm 1 end to end on one device: M replicas of a small table set, each taking its own batch
through forward + backward with the moment-scaled step, then the weight sync and the moment sync
(tbe_replica_mean); the CPU oracle does the same."""
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


@pytest.mark.parametrize("name,kw,M", [
    ("C2", dict(T=4, B=256, rows_scale=0.02), 4),
    ("C4", dict(T=4, B=128, rows_scale=2e-4), 2),      # fp16 tables: the mean is rounded once to binary16
    ("C5", dict(T=16, B=256, rows_scale=1e-3), 3),     # mean pooling; M not a power of two
])
def test_algorithm1_iterations_match_oracle(H, name, kw, M):
    import oracle
    from paper_2508_03854_amd import TBE
    cfg = W.config(name, c=float(M), **kw)
    tabs0 = H.host_tables(cfg)
    iv = np.uint32 if cfg.weight_dtype == "f32" else np.uint16
    ref_w = [[a.copy() for a in tabs0] for _ in range(M)]
    ref_v = [np.zeros(cfg.total_rows, np.float32) for _ in range(M)]
    dev_w = [H.flat_from_tables(tabs0) for _ in range(M)]
    dev_v = [torch.zeros(cfg.total_rows, device="cuda") for _ in range(M)]
    tbe = TBE(cfg.rows, cfg.D, cfg.weight_dtype)
    for it in range(3):
        for m in range(M):
            k = it * M + m                                  # every replica sees its own batch
            idx, off = W.make_batch(cfg, k)
            gout = W.make_grad_out(cfg, k)
            ws = tbe.alloc_workspace(cfg.B, max(1, idx.numel()))
            out_ref = oracle.forward(ref_w[m], idx.numpy(), off.numpy(), cfg.B, cfg.pooling)
            out = tbe.forward(dev_w[m], idx.cuda(), off.cuda(), cfg.B, cfg.pooling)
            rt = H.RTOL_F32 if (cfg.weight_dtype == "f32" or it == 0) else H.RTOL_F16
            H.assert_close(out.cpu().numpy(), out_ref, rt, cfg.w_scale, f"forward it {it} replica {m}")
            oracle.backward_rowwise_adagrad(ref_w[m], ref_v[m], gout.numpy(), idx.numpy(), off.numpy(), cfg.B, cfg.pooling,
                                            cfg.lr, cfg.eps, cfg.c, want_indices=False)
            tbe.backward_rowwise_adagrad(gout.cuda(), idx.cuda(), off.cuda(), cfg.B, dev_w[m], dev_v[m], ws,
                                         pooling=cfg.pooling, lr=cfg.lr, eps=cfg.eps, momentum_scale=cfg.c)
        # weight sync and moment sync
        for t in range(cfg.T):
            oracle.replica_mean([ref_w[m][t] for m in range(M)])
        oracle.replica_mean(ref_v)
        tbe.replica_mean(dev_w)
        tbe.replica_mean(dev_v)
        torch.cuda.synchronize()
        w0 = dev_w[0].cpu().numpy()
        v0 = dev_v[0].cpu().numpy()
        for m in range(1, M):                               # consensus: all replicas hold the same bits
            assert np.array_equal(dev_w[m].cpu().numpy().view(iv), w0.view(iv))
            assert np.array_equal(dev_v[m].cpu().numpy().view(np.uint32), v0.view(np.uint32))
        rtol = H.RTOL_F32 if cfg.weight_dtype == "f32" else H.RTOL_F16
        gpu_tabs = H.split_flat(w0, cfg)
        for t in range(cfg.T):
            H.assert_close(gpu_tabs[t], ref_w[0][t], rtol, cfg.w_scale, f"weights of table {t} after sync {it}")
        H.assert_close(v0, ref_v[0], H.RTOL_F32, 1e-6, f"moments after sync {it}")
    tbe.close()


def test_replica_mean_values_tail_and_argument_checks(H):
    from paper_2508_03854_amd import TBE, binding as P
    import oracle
    tbe = TBE([16], [8], "f32")
    rng = np.random.default_rng(0)
    for dtype, n in ((np.float32, 4099), (np.float16, 8197), (np.float32, 3), (np.float16, 5)):   # ragged tails
        for M in (1, 2, 5, 16):
            host = [rng.standard_normal(n).astype(dtype) for _ in range(M)]
            dev = [torch.from_numpy(h.copy()).cuda() for h in host]
            oracle.replica_mean(host)
            tbe.replica_mean(dev)
            got = dev[0].cpu().numpy()
            for d in dev[1:]:
                assert np.array_equal(d.cpu().numpy().view(np.uint16 if dtype == np.float16 else np.uint32),
                                      got.view(np.uint16 if dtype == np.float16 else np.uint32))
            if dtype == np.float32:
                np.testing.assert_allclose(got, host[0], rtol=1e-6, atol=1e-7)
            else:
                assert H.half_ulp_distance(got, host[0]).max() <= 1
            if M == 1:
                assert np.array_equal(got, host[0])
    a = torch.zeros(64, device="cuda")
    import ctypes
    L = P.load_library()
    two = (ctypes.c_void_p * 2)(a.data_ptr(), a.data_ptr())
    assert L.tbe_replica_mean(tbe._h, two, 2, 64, P.F32, torch.cuda.current_stream().cuda_stream) == P.EINVAL
    mis = (ctypes.c_void_p * 2)(a.data_ptr(), a.data_ptr() + 4)
    assert L.tbe_replica_mean(tbe._h, mis, 2, 8, P.F32, torch.cuda.current_stream().cuda_stream) == P.EINVAL
    assert L.tbe_replica_mean(tbe._h, two, 17, 64, P.F32, torch.cuda.current_stream().cuda_stream) == P.EINVAL
    # distinct, aligned pointers whose ranges overlap: 32 floats starting 16 floats apart
    lap = (ctypes.c_void_p * 2)(a.data_ptr(), a.data_ptr() + 64)
    assert L.tbe_replica_mean(tbe._h, lap, 2, 32, P.F32, torch.cuda.current_stream().cuda_stream) == P.EINVAL
    assert L.tbe_replica_mean(tbe._h, lap, 2, 16, P.F32, torch.cuda.current_stream().cuda_stream) == P.OK   # adjacent
    assert L.tbe_replica_mean(tbe._h, two, 2, 64, 7, torch.cuda.current_stream().cuda_stream) == P.EDTYPE
    tbe.close()
