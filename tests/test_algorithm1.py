"""CPU pins of the oracle's replica synchronisation and of Algorithm 1 as a whole: closed forms, special cases and
the statements of Proposition 1 and Scaling Rule 1 checked numerically.  Oracle only, no GPU."""
import numpy as np


def test_replica_mean_worked_values_and_special_cases(oracle_mod):
    a = [np.array([1.0, -2.0, 0.5], np.float32), np.array([2.0, 2.0, 0.5], np.float32),
         np.array([3.0, 0.0, 0.5], np.float32), np.array([6.0, 4.0, 0.5], np.float32)]
    oracle_mod.replica_mean(a)
    for x in a:
        assert x.tolist() == [3.0, 1.0, 0.5]
    # M = 1: nothing changes, bit for bit
    rng = np.random.default_rng(3)
    x = rng.standard_normal(1000).astype(np.float32)
    y = x.copy()
    oracle_mod.replica_mean([y])
    assert np.array_equal(x.view(np.uint32), y.view(np.uint32))
    # all replicas agree afterwards, a second application changes nothing, and the value is the library's mean
    reps = [rng.standard_normal(257).astype(np.float32) for _ in range(5)]
    want = np.mean(np.stack(reps).astype(np.float64), axis=0)
    oracle_mod.replica_mean(reps)
    for r in reps[1:]:
        assert np.array_equal(r.view(np.uint32), reps[0].view(np.uint32))
    np.testing.assert_allclose(reps[0], want, rtol=1e-7, atol=0)
    again = [r.copy() for r in reps]
    oracle_mod.replica_mean(again)
    assert np.array_equal(again[0].view(np.uint32), reps[0].view(np.uint32))


def test_replica_mean_binary16_rounds_once_to_nearest_even(oracle_mod):
    # mean of 1 and 1 + 2^-10 is 1 + 2^-11, halfway between two binary16 values: ties to the even one (1.0)
    a = [np.array([1.0], np.float16), np.array([1.0 + 2.0 ** -10], np.float16)]
    oracle_mod.replica_mean(a)
    assert a[0].view(np.uint16)[0] == 0x3C00 and a[1].view(np.uint16)[0] == 0x3C00
    # 1 + 2^-10 and 1 + 2^-9 -> 1 + 1.5 * 2^-10: ties to even picks 1 + 2^-9 (mantissa 2)
    b = [np.array([1.0 + 2.0 ** -10], np.float16), np.array([1.0 + 2.0 ** -9], np.float16)]
    oracle_mod.replica_mean(b)
    assert b[0].view(np.uint16)[0] == 0x3C02
    # three replicas: the sum is not rounded before the division
    c = [np.array([x], np.float16) for x in (0.1, 0.2, 0.4)]
    exact = (float(c[0][0]) + float(c[1][0]) + float(c[2][0])) / 3.0
    oracle_mod.replica_mean(c)
    assert c[0][0] == np.float16(exact)


def _problem(rng, R=40, D=8, B=64, L=3):
    W0 = (rng.standard_normal((R, D)) * 0.1).astype(np.float32)
    idx = rng.integers(0, R, size=B * L).astype(np.int64)
    off = (np.arange(B + 1) * L).astype(np.int64)
    return W0, idx, off


def _local_steps(oracle_mod, W0, v0, idx, off, B, grads, lr, eps, c):
    """The local half of one iteration of Algorithm 1 (steps 4-6) in every replica; returns weights and moments."""
    ws, vs = [], []
    for g in grads:
        w, v = [W0.copy()], v0.copy()
        oracle_mod.backward_rowwise_adagrad(w, v, g, idx, off, B, "sum", lr, eps, c)
        ws.append(w[0])
        vs.append(v)
    return ws, vs


def test_one_group_without_sync_is_plain_rowwise_adagrad(oracle_mod):
    # with M = 1 the two sync steps are the identity, and c = 1 is the unscaled optimizer: the iteration then is
    # the closed-form row-wise AdaGrad step (checked here on a row hit exactly once)
    rng = np.random.default_rng(5)
    W0, idx, off = _problem(rng, R=1000, B=4, L=1)      # 4 lookups into 1000 rows: all distinct with this seed
    assert len(set(idx.tolist())) == 4
    B, D = 4, W0.shape[1]
    g = rng.standard_normal((B, D)).astype(np.float32)
    v0 = np.full(1000, 0.5, np.float32)
    ws, vs = _local_steps(oracle_mod, W0, v0, idx, off, B, [g], 0.1, 1e-8, 1.0)
    oracle_mod.replica_mean(ws)
    oracle_mod.replica_mean(vs)
    for b in range(B):
        r = idx[b]
        gb = g[b].astype(np.float64)
        v = 0.5 + float(gb @ gb)
        want = W0[r].astype(np.float64) - 0.1 / (np.sqrt(v) + 1e-8) * gb
        np.testing.assert_allclose(ws[0][r], want, rtol=1e-6)
        np.testing.assert_allclose(vs[0][r], v, rtol=1e-6)


def test_identical_replicas_stay_identical_to_a_single_run(oracle_mod):
    # M = 4 replicas fed the same batch and gradient: the mean of four equal floats is that float (exact for a
    # power-of-two M), so the synchronised result is the single-replica result bit for bit
    rng = np.random.default_rng(6)
    W0, idx, off = _problem(rng)
    B, D = 64, W0.shape[1]
    g = rng.standard_normal((B, D)).astype(np.float32)
    v0 = np.zeros(W0.shape[0], np.float32)
    ws, vs = _local_steps(oracle_mod, W0, v0, idx, off, B, [g] * 4, 0.05, 1e-8, 2.0)
    single_w, single_v = ws[0].copy(), vs[0].copy()
    oracle_mod.replica_mean(ws)
    oracle_mod.replica_mean(vs)
    for m in range(4):
        assert np.array_equal(ws[m].view(np.uint32), single_w.view(np.uint32))
        assert np.array_equal(vs[m].view(np.uint32), single_v.view(np.uint32))


def test_proposition1_moment_increment_is_larger_under_2d(oracle_mod):
    # Proposition 1 (ii).  M groups draw i.i.d. gradients for the same rows.  Under the 2D scheme every group adds
    # ||g^(m)||^2 and the moment sync averages: increment mean_m ||g^(m)||^2.  Without it the one group sees the
    # averaged gradient: increment ||mean_m g^(m)||^2.  The first is never smaller (Jensen), row by row.
    rng = np.random.default_rng(7)
    M = 4
    W0, idx, off = _problem(rng)
    B, D = 64, W0.shape[1]
    grads = [rng.standard_normal((B, D)).astype(np.float32) for _ in range(M)]
    v0 = np.zeros(W0.shape[0], np.float32)
    _, vs = _local_steps(oracle_mod, W0, v0, idx, off, B, grads, 0.05, 1e-8, 1.0)
    oracle_mod.replica_mean(vs)
    g_mean = np.mean(np.stack(grads).astype(np.float64), axis=0).astype(np.float32)
    _, v_non2d = _local_steps(oracle_mod, W0, v0, idx, off, B, [g_mean], 0.05, 1e-8, 1.0)
    touched = np.zeros(W0.shape[0], bool)
    touched[idx] = True
    assert touched.sum() > 20
    assert np.all(vs[0][touched] >= v_non2d[0][touched] * (1 - 1e-6))
    assert np.all(vs[0][~touched] == 0) and np.all(v_non2d[0][~touched] == 0)
    # pure-noise gradients: E||mean_m g||^2 = E||g||^2 / M, so the 2D moment is about M times the other
    ratio = vs[0][touched].sum() / v_non2d[0][touched].sum()
    assert abs(ratio / M - 1.0) < 0.15, ratio


def test_scaling_rule_c_equal_M_restores_the_step_size_for_pure_noise(oracle_mod):
    # Scaling Rule 1: c lies in (0, M], large c for noisy gradients.  For pure noise the 2D moment is ~M times the
    # non-2D one, so c = M brings eta / sqrt(v / c) back to the non-2D step size, while c = 1 shrinks it by sqrt(M).
    rng = np.random.default_rng(8)
    M = 8
    W0, idx, off = _problem(rng, R=30, D=16, B=256, L=4)
    B, D = 256, W0.shape[1]
    grads = [rng.standard_normal((B, D)).astype(np.float32) for _ in range(M)]
    v0 = np.zeros(W0.shape[0], np.float32)
    g_mean = np.mean(np.stack(grads).astype(np.float64), axis=0).astype(np.float32)
    w_ref, _ = _local_steps(oracle_mod, W0, v0, idx, off, B, [g_mean], 0.05, 1e-12, 1.0)
    step_ref = np.linalg.norm((w_ref[0] - W0).astype(np.float64))
    steps = {}
    for c in (1.0, float(M)):
        ws, vs = _local_steps(oracle_mod, W0, v0, idx, off, B, grads, 0.05, 1e-12, c)
        oracle_mod.replica_mean(ws)
        steps[c] = np.linalg.norm((ws[0] - W0).astype(np.float64))
    # first iteration from v = 0: each replica's own step has unit-free size eta*sqrt(c)*g/||g||; after the weight
    # sync the averaged step is ~1/sqrt(M) of that for independent noise, so c = M gives the non-2D size back
    assert abs(steps[float(M)] / step_ref - 1.0) < 0.15, (steps, step_ref)
    assert abs(steps[1.0] / step_ref - 1.0 / np.sqrt(M)) < 0.1, (steps, step_ref)
