"""Shared driver of the GPU parity tests: runs the HIP path (through the C ABI binding) and the CPU
oracle on the same seeded inputs and compares them.  Not a test module itself."""
from __future__ import annotations

import numpy as np
import torch

import oracle
import workloads as W
from paper_2508_03854_amd import TBE

# float tolerances of the parity bar: |gpu - ref| <= rtol*|ref| + rtol*scale, with `scale` the magnitude
# of the operands (max |w| for weights and pooled sums): a purely relative test is ill-posed for sums
# that cancel.  fp32 tables and moments: rtol 1e-5.  fp16 tables: rtol 1e-2, and additionally at most one
# binary16 ulp away from the oracle's correctly rounded value.
RTOL_F32 = 1e-5
RTOL_F16 = 1e-2


def host_tables(cfg: W.Config):
    tabs = []
    for t in range(cfg.T):
        w = W.weight_rows(cfg, t, torch.arange(cfg.rows[t]))
        tabs.append(w.numpy() if cfg.weight_dtype == "f32" else w.to(torch.float16).numpy())
    return tabs


def flat_from_tables(tabs, device="cuda"):
    return torch.from_numpy(np.concatenate([a.reshape(-1) for a in tabs])).to(device)


def split_flat(flat_np: np.ndarray, cfg: W.Config):
    woff = cfg.w_offsets()
    return [flat_np[woff[t]:woff[t + 1]].reshape(cfg.rows[t], cfg.D[t]) for t in range(cfg.T)]


def forward_scale(cfg: W.Config, off_np: np.ndarray, B: int, same_inputs: bool):
    """Operand magnitude per element of the pooled output, the `scale` of assert_close.
    While both sides pool bit-identical weights: max|w|, and for a sum-pooled bag of L > 42 ids max|w| * L/42, i.e. an
    absolute term of 4 * 2^-24 * L * max|w| - four units in the last place of the largest partial sum the bag can
    reach (every fp32 addition rounds at the magnitude of the running sum, which the final value, after cancellation,
    may be far below; observed: 1.5e-7 on a 509-id bag whose sum is 0.0027).
    After a step each side pools its OWN weights, which agree only to the weight tolerance (up to 2 * rtol * max|w|
    per element); over a sum-pooled bag of L ids - L copies of one row's difference, if the bag repeats a row - these
    add up, so 2 L is added.  Mean pooling divides sum and error by L: its scale is max|w|, resp. 3 max|w|."""
    f = np.full((B, cfg.sum_D), 1.0 if same_inputs else 3.0)
    if cfg.pooling == "sum":
        lens = np.diff(np.asarray(off_np, dtype=np.int64)).reshape(cfg.T, B).astype(np.float64)
        d_off = cfg.D_offsets()
        for t in range(cfg.T):
            f[:, d_off[t]:d_off[t + 1]] = (np.maximum(1.0, lens[t] / 42.0) + (0.0 if same_inputs else 2.0 * lens[t]))[:, None]
    return cfg.w_scale * f


def assert_close(got: np.ndarray, ref: np.ndarray, rtol: float, scale, what: str):
    got64, ref64 = got.astype(np.float64), ref.astype(np.float64)
    err = np.abs(got64 - ref64)
    tol = rtol * np.abs(ref64) + rtol * scale
    bad = err > tol
    if bad.any():
        i = np.unravel_index(np.argmax(err - tol), err.shape)
        raise AssertionError(f"{what}: {int(bad.sum())} of {bad.size} outside tolerance; worst at {i}: "
                             f"got {got64[i]!r} ref {ref64[i]!r} err {err[i]:.3e} tol {tol[i]:.3e}")
    return float(err.max()) if err.size else 0.0


def half_ulp_distance(a: np.ndarray, b: np.ndarray) -> np.ndarray:
    """Distance in binary16 ulps between two float16 arrays (finite values)."""
    def ordered(x):
        u = x.view(np.uint16).astype(np.int32)
        return np.where(u & 0x8000, -(u & 0x7FFF), u)
    return np.abs(ordered(a) - ordered(b))


_IO_TORCH = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}


def io_to_numpy(t: torch.Tensor, io: str) -> np.ndarray:
    """Host tensor -> the array type the oracle takes for that element type (bfloat16 travels as uint16 bits)."""
    if io == "bf16":
        return t.contiguous().view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def decode16(a: np.ndarray, io: str) -> np.ndarray:
    """16-bit float array (float16, or uint16 holding bfloat16 bits) -> float64 values."""
    if io == "bf16":
        return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


def ulp16_distance(a: np.ndarray, b: np.ndarray) -> np.ndarray:
    """Distance in units of the last place between two arrays of 16-bit float bit patterns (binary16 or bfloat16;
    sign-magnitude ordering is the same for both), finite values."""
    def ordered(x):
        u = x.view(np.uint16).astype(np.int32)
        return np.where(u & 0x8000, -(u & 0x7FFF), u)
    return np.abs(ordered(a) - ordered(b))


def check_step(cfg: W.Config, tbe: TBE, flat: torch.Tensor, state: torch.Tensor, tabs, state_np: np.ndarray,
               idx: torch.Tensor, off: torch.Tensor, gout: torch.Tensor, ws: torch.Tensor, check_sorted: bool = True,
               same_inputs: bool = True, index_dtype: torch.dtype = torch.int64, io: str = "f32",
               ulp_rate: float = 2e-3):
    """One forward + backward on both sides, in place; compares everything.  Returns a dict of error figures.
    same_inputs: both sides start this step from bit-identical weights (true for the first step).  After a
    step on fp16 tables the two sides may already differ by one binary16 ulp where the fp32 and fp64 results
    straddle a rounding boundary, so later steps are held to the fp16 tolerance only."""
    B = cfg.B
    extended = (index_dtype != torch.int64) or (io != "f32")     # the *_ex entry points
    gout = gout.to(_IO_TORCH[io])                                 # both sides receive the same rounded gradient
    idx_np, off_np, go_np = idx.numpy(), off.numpy(), io_to_numpy(gout, io)
    d_idx, d_off, d_go = idx.to(index_dtype).cuda(), off.to(index_dtype).cuda(), gout.cuda()
    w_scale = cfg.w_scale
    report = {}

    # ---- forward
    out_ref = oracle.forward(tabs, idx_np, off_np, B, cfg.pooling, out_dtype=io)
    if extended:
        out_gpu = io_to_numpy(tbe.forward_ex(flat, d_idx, d_off, B, cfg.pooling, out_dtype=_IO_TORCH[io]).cpu(), io)
    else:
        out_gpu = tbe.forward(flat, d_idx, d_off, B, cfg.pooling).cpu().numpy()
    assert not tbe.poll_index_error()
    fwd_rtol = RTOL_F32 if (cfg.weight_dtype == "f32" or same_inputs) else RTOL_F16
    if io == "f32":
        report["fwd_max_err"] = assert_close(out_gpu, out_ref, fwd_rtol, forward_scale(cfg, off_np, B, same_inputs), "forward")
    else:
        # 16-bit output: the fp32 sum is rounded once.  Values: the fp32 tolerance plus one unit in the last place
        # of the format.  Where the sum did not cancel (|ref| >= scale/10, so the fp32 error is far below the
        # format's spacing) the result is the oracle's value or, rarely, its neighbour.
        ulp_rel = 2.0 ** -10 if io == "f16" else 2.0 ** -7
        ref64 = decode16(out_ref, io)
        report["fwd_max_err"] = assert_close(decode16(out_gpu, io), ref64, fwd_rtol + ulp_rel, forward_scale(cfg, off_np, B, same_inputs), "forward")
        if same_inputs:
            big = np.abs(ref64) >= 0.1 * w_scale
            d = ulp16_distance(out_gpu, out_ref)[big]
            if d.size:
                assert d.max() <= 1, f"{io} forward: {int(d.max())} ulps from the oracle"
                # how often the fp32 and the fp64 sum straddle a rounding boundary of the format grows with the
                # fp32 sum's error, i.e. with the number of terms: 2e-3 up to 32 ids per bag, in proportion beyond
                longest = int(np.diff(np.asarray(off_np, dtype=np.int64)).max()) if len(off_np) > 1 else 0
                rate16 = 2e-3 * max(1.0, longest / 32.0)
                assert (d > 0).sum() <= max(2, rate16 * d.size), f"{int((d > 0).sum())}/{d.size} {io} outputs round differently"
                report["fwd_ulp_mismatch_frac"] = float((d > 0).mean())

    # ---- backward + optimizer
    prev_tabs = split_flat(flat.cpu().numpy(), cfg)      # the GPU's own weights and moments before the step
    prev_state = state.cpu().numpy()
    res = oracle.backward_rowwise_adagrad(tabs, state_np, go_np, idx_np, off_np, B, cfg.pooling, cfg.lr, cfg.eps, cfg.c,
                                          grad_dtype=io)
    step_fn = tbe.backward_rowwise_adagrad_ex if extended else tbe.backward_rowwise_adagrad
    step_fn(d_go, d_idx, d_off, B, flat, state, ws, pooling=cfg.pooling, lr=cfg.lr, eps=cfg.eps, momentum_scale=cfg.c)
    assert not tbe.poll_index_error()
    nnz = idx.numel()
    if check_sorted and nnz > 0:
        dbg = tbe.debug_sorted(ws, B, nnz)
        assert dbg["num_unique"] == res.U, (dbg["num_unique"], res.U)
        assert np.array_equal(dbg["keys_sorted"].numpy(), res.keys_sorted), "keys_sorted differs"
        # the payload of the sort is the bag of each lookup: the oracle's stable order, mapped position -> bag
        bag_of_order = np.searchsorted(off_np, res.order, side="right") - 1
        assert np.array_equal(dbg["vals_sorted"].numpy(), bag_of_order), "stable order differs"
        assert np.array_equal(dbg["unique_rows"].numpy(), res.unique_rows), "unique_rows differs"
        assert np.array_equal(dbg["seg_start"].numpy(), res.seg_start), "seg_start differs"
    report["U"] = res.U
    report["max_seg"] = int(np.diff(res.seg_start).max()) if res.U else 0

    flat_np = flat.cpu().numpy()
    state_gpu = state.cpu().numpy()
    gpu_tabs = split_flat(flat_np, cfg)
    touched = np.zeros(cfg.total_rows, dtype=bool)
    touched[res.unique_rows] = True
    hits = np.zeros(cfg.total_rows, dtype=np.int64)      # lookups per row
    hits[res.unique_rows] = np.diff(res.seg_start)
    base = cfg.row_base()
    # untouched rows keep their bits (weights and moments)
    iv = np.uint32 if cfg.weight_dtype == "f32" else np.uint16
    for t in range(cfg.T):
        m = ~touched[base[t]:base[t + 1]]
        assert np.array_equal(gpu_tabs[t][m].view(iv), prev_tabs[t][m].view(iv)), f"untouched rows of table {t} changed"
    assert np.array_equal(state_gpu[~touched].view(np.uint32), prev_state[~touched].view(np.uint32))
    # touched rows: floats within tolerance
    werr, ulp_bad, ulp_n = 0.0, 0, 0
    for t in range(cfg.T):
        m = touched[base[t]:base[t + 1]]
        if not m.any():
            continue
        if cfg.weight_dtype == "f32":
            werr = max(werr, assert_close(gpu_tabs[t][m], tabs[t][m], RTOL_F32, w_scale, f"weights of table {t}"))
            if same_inputs:
                # the step itself (Algorithm 1, step 6): w_after - w_before on both sides, to 1e-5 of the row's
                # largest update plus the rounding of the subtraction (one fp32 ulp of the weights).  A row whose
                # gradient is an fp32 sum of n terms of either sign carries that sum's error, about sqrt(n) * 2^-24
                # of the result; four times that replaces 1e-5 where it is larger (rows with more than ~1750 lookups).
                dw_g = gpu_tabs[t][m].astype(np.float64) - prev_tabs[t][m].astype(np.float64)
                dw_r = tabs[t][m].astype(np.float64) - prev_tabs[t][m].astype(np.float64)
                row_max = np.abs(dw_r).max(axis=1, keepdims=True)
                row_rtol = np.maximum(RTOL_F32, 4.0 * np.sqrt(hits[base[t]:base[t + 1]][m]) * 2.0 ** -24)[:, None]
                bound = row_rtol * row_max + 2.0 ** -23 * (np.abs(prev_tabs[t][m]).astype(np.float64) + np.abs(dw_r))
                bad = np.abs(dw_g - dw_r) > bound
                assert not bad.any(), (f"updates of table {t}: {int(bad.sum())} elements outside 1e-5 of the row's step; "
                                       f"worst {np.abs(dw_g - dw_r).max():.3e}")
        else:
            werr = max(werr, assert_close(gpu_tabs[t][m], tabs[t][m], RTOL_F16, w_scale, f"weights of table {t}"))
            if same_inputs:
                d = half_ulp_distance(gpu_tabs[t][m], tabs[t][m])
                assert d.max() <= 1, f"fp16 weights of table {t}: {int(d.max())} ulps from the oracle"
                ulp_bad += int((d > 0).sum())
                ulp_n += d.size
    if ulp_n:
        # (each such element is exactly one ulp off; how often the fp32 and fp64 results straddle a rounding boundary
        # depends on how much w and its update cancel, hence a rate the caller may widen for larger learning rates)
        assert ulp_bad <= max(2, ulp_rate * ulp_n), f"{ulp_bad}/{ulp_n} fp16 weights round differently from the oracle"
        report["fp16_ulp_mismatch_frac"] = ulp_bad / ulp_n
    report["w_max_err"] = werr
    report["v_max_err"] = assert_close(state_gpu[touched], state_np[touched], RTOL_F32, 1e-6, "moments")
    return report


def run_config(cfg: W.Config, steps: int = 1, state_kind: str = "zeros", check_sorted: bool = True,
               index_dtype: torch.dtype = torch.int64, io: str = "f32", tunables=None):
    tabs = host_tables(cfg)
    flat = flat_from_tables(tabs)
    state_np = np.zeros(cfg.total_rows, dtype=np.float32)
    if state_kind == "hash":
        state_np = W.state_rows(cfg, torch.arange(cfg.total_rows)).numpy()
    state = torch.from_numpy(state_np.copy()).cuda()
    tbe = TBE(cfg.rows, cfg.D, cfg.weight_dtype)
    for k, v in (tunables or {}).items():
        tbe.set_tunable(k, v)
    reports = []
    for step in range(steps):
        idx, off = W.make_batch(cfg, step)
        gout = W.make_grad_out(cfg, step)
        ws = tbe.alloc_workspace(cfg.B, max(1, idx.numel()))
        reports.append(check_step(cfg, tbe, flat, state, tabs, state_np, idx, off, gout, ws, check_sorted,
                                  same_inputs=(step == 0), index_dtype=index_dtype, io=io))
    tbe.close()
    return reports
