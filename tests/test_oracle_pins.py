"""Pins for the CPU oracle: each test ties one oracle function to something that is not the oracle -
a dense brute-force formulation, a closed form, an invariant, or a library routine that the path
reduces to in a special case.  The paper prints no worked numeric example for this path, so there is
no paper fixture to compare with; the citations say which passage fixes the property."""
import math

import numpy as np
import pytest
import torch

import workloads as W


def tiny_problem(rng, T=3, B=5, maxL=4, Rs=(7, 3, 8), Ds=(4, 2, 3), dtype=np.float32, allow_empty=True):
    tables = [rng.standard_normal((Rs[t], Ds[t])).astype(dtype) for t in range(T)]
    lens = rng.integers(0 if allow_empty else 1, maxL + 1, size=T * B)
    offsets = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    idx = np.concatenate([rng.integers(0, Rs[t], size=int(lens[t * B:(t + 1) * B].sum())) for t in range(T)]).astype(np.int64)
    return tables, idx, offsets


def count_matrix(t, R, idx, offsets, B, pooling):
    """P[b, r] = (pooling factor of bag (t,b)) x (number of times id r occurs in it) - dense brute force."""
    P = np.zeros((B, R), dtype=np.float64)
    for b in range(B):
        s, e = offsets[t * B + b], offsets[t * B + b + 1]
        for p in range(s, e):
            P[b, idx[p]] += 1.0
        if pooling == "mean" and e > s:
            P[b] /= (e - s)
    return P


# ---------------------------------------------------------------- forward
@pytest.mark.parametrize("pooling", ["sum", "mean"])
def test_forward_equals_dense_count_matrix_product(oracle_mod, pooling):
    # a pooled sum is the sum of its rows: out_t = P_t . W_t
    rng = np.random.default_rng(1)
    for trial in range(5):
        tables, idx, offsets = tiny_problem(rng)
        B = 5
        out = oracle_mod.forward(tables, idx, offsets, B, pooling)
        col = 0
        for t, Wt in enumerate(tables):
            P = count_matrix(t, Wt.shape[0], idx, offsets, B, pooling)
            ref = P @ Wt.astype(np.float64)
            np.testing.assert_allclose(out[:, col:col + Wt.shape[1]], ref, rtol=1e-6, atol=1e-7)
            col += Wt.shape[1]


def test_forward_one_hot_bags_return_rows_bit_exact(oracle_mod):
    rng = np.random.default_rng(2)
    Wt = rng.standard_normal((11, 8)).astype(np.float32)
    idx = rng.integers(0, 11, size=6).astype(np.int64)
    offsets = np.arange(7, dtype=np.int64)
    for pooling in ("sum", "mean"):
        out = oracle_mod.forward([Wt], idx, offsets, 6, pooling)
        assert np.array_equal(out.view(np.uint32), Wt[idx].view(np.uint32))


def test_forward_empty_bag_is_zero_and_mean_is_sum_over_L(oracle_mod):
    Wt = np.arange(12, dtype=np.float32).reshape(4, 3)
    idx = np.array([1, 1, 3, 0], dtype=np.int64)
    offsets = np.array([0, 3, 3, 4], dtype=np.int64)      # bags: [1,1,3], [], [0]
    s = oracle_mod.forward([Wt], idx, offsets, 3, "sum")
    m = oracle_mod.forward([Wt], idx, offsets, 3, "mean")
    assert np.array_equal(s[0], 2 * Wt[1] + Wt[3])          # a repeated id counts twice
    assert np.array_equal(s[1], np.zeros(3)) and np.array_equal(m[1], np.zeros(3))
    np.testing.assert_allclose(m[0], s[0] / 3.0, rtol=1e-7)
    assert np.array_equal(m[2], Wt[0])


@pytest.mark.parametrize("pooling", ["sum", "mean"])
def test_forward_matches_library_embedding_bag(oracle_mod, pooling):
    # special case that reduces to a library routine: one table == an embedding-bag
    rng = np.random.default_rng(3)
    R, D, B = 50, 16, 9
    Wt = rng.standard_normal((R, D)).astype(np.float32)
    lens = rng.integers(1, 6, size=B)
    offsets = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    idx = rng.integers(0, R, size=int(lens.sum())).astype(np.int64)
    out = oracle_mod.forward([Wt], idx, offsets, B, pooling)
    ref = torch.nn.functional.embedding_bag(torch.from_numpy(idx), torch.from_numpy(Wt).double(),
                                            torch.from_numpy(offsets[:-1]), mode=pooling).numpy()
    np.testing.assert_allclose(out, ref, rtol=1e-6, atol=1e-7)


def test_forward_rejects_out_of_range_id(oracle_mod):
    Wt = np.zeros((4, 2), dtype=np.float32)
    with pytest.raises(IndexError):
        oracle_mod.forward([Wt], np.array([4], dtype=np.int64), np.array([0, 1], dtype=np.int64), 1)


# ---------------------------------------------------------------- fp16 conversion
def test_half_conversions_match_ieee_binary16(oracle_mod):
    # every finite binary16 pattern decodes to numpy's value; encoding rounds to nearest even like numpy's direct cast
    bits = np.arange(0, 1 << 16, dtype=np.uint16)
    ref = bits.view(np.float16).astype(np.float64)
    got = np.array([oracle_mod.half_to_double(int(b)) for b in bits])
    fin = np.isfinite(ref)
    assert np.array_equal(got[fin], ref[fin]) and np.all(np.isnan(got[np.isnan(ref)]))
    rng = np.random.default_rng(4)
    xs = np.concatenate([rng.standard_normal(4000) * 10.0 ** rng.integers(-9, 5, size=4000),
                         (ref[fin][:-1] + ref[fin][1:]) / 2.0,            # exact ties between neighbours
                         [0.0, -0.0, 65504.0, 65519.99, 65520.0, 1e6, -1e6, 2.0 ** -25, 2.0 ** -24, 5.9e-8]])
    xs = xs[np.isfinite(xs)]
    with np.errstate(over="ignore"):
        want = xs.astype(np.float16).view(np.uint16)
    got = np.array([oracle_mod.double_to_half(float(x)) for x in xs], dtype=np.uint16)
    assert np.array_equal(got, want)


# ---------------------------------------------------------------- sort / dedup / segments
def test_sort_and_segments_are_exact(oracle_mod):
    rng = np.random.default_rng(5)
    for trial in range(4):
        Rs = (7, 3, 8)
        tables, idx, offsets = tiny_problem(rng, Rs=Rs, B=6, maxL=5)
        keys, bag_of = oracle_mod.linearize(Rs, idx, offsets, 6)
        # brute-force keys: table of position p from its bag
        base = np.concatenate([[0], np.cumsum(Rs)])
        for p in range(len(idx)):
            bag = np.searchsorted(offsets, p, side="right") - 1
            assert bag_of[p] == bag and keys[p] == base[bag // 6] + idx[p]
        ks, order = oracle_mod.stable_sort(keys)
        assert np.array_equal(order, np.argsort(keys, kind="stable"))
        assert np.array_equal(ks, keys[order]) and np.all(np.diff(ks) >= 0)
        uniq, seg = oracle_mod.run_lengths(ks)
        u_ref, cnt_ref = np.unique(keys, return_counts=True)
        assert np.array_equal(uniq, u_ref) and np.array_equal(np.diff(seg), cnt_ref)
        assert seg[0] == 0 and seg[-1] == len(keys) and np.all(np.diff(uniq) > 0)
        hist = np.bincount(keys, minlength=int(base[-1]))
        assert np.array_equal(hist[uniq], np.diff(seg)) and hist.sum() == len(keys)


def test_same_id_in_two_tables_is_two_rows(oracle_mod):
    keys, _ = oracle_mod.linearize([5, 5], np.array([2, 2], dtype=np.int64), np.array([0, 1, 2], dtype=np.int64), 1)
    assert keys.tolist() == [2, 7]


# ---------------------------------------------------------------- AdaGrad step
def test_single_hit_closed_form(oracle_mod):
    # Algorithm 1 steps 5-6 with v0 = 0:  dw = -lr*g / (||g||/sqrt(c) + eps);  ||dw|| = lr*sqrt(c) up to O(eps)
    rng = np.random.default_rng(6)
    D, lr, eps = 16, 0.05, 1e-8
    for c in (1.0, 4.0, 0.25):
        for scale in (1e-3, 1.0, 1e3):
            w0 = rng.standard_normal((3, D)).astype(np.float32)
            tab = w0.copy()
            g = rng.standard_normal(D) * scale
            v = np.zeros(1, dtype=np.float32)
            oracle_mod.adagrad_row(tab, 1, v, g, lr, eps, c)
            gn = math.sqrt(float(np.dot(g, g)))
            dw = tab[1].astype(np.float64) - w0[1]
            np.testing.assert_allclose(dw, -lr * g / (gn / math.sqrt(c) + eps), rtol=0, atol=2e-7 * np.abs(w0[1]).max() + 1e-9)
            assert abs(np.linalg.norm(dw) - lr * math.sqrt(c)) < 1e-6       # independent of the gradient's scale
            assert v[0] == np.float32(gn * gn)                               # the stored moment is NOT divided by c
            assert np.array_equal(tab[[0, 2]], w0[[0, 2]])                   # neighbours untouched


def test_prior_moment_closed_form_and_scaling_identity(oracle_mod):
    # lr/(sqrt(v/c)+eps) == (lr*sqrt(c))/(sqrt(v)+eps*sqrt(c)): (lr,eps,c) equals plain row-wise AdaGrad with (lr*sqrt(c), eps*sqrt(c), 1)
    rng = np.random.default_rng(7)
    D, lr, eps, c, v0 = 8, 0.01, 1e-3, 4.0, 2.5
    w0 = rng.standard_normal((1, D)).astype(np.float32)
    g = rng.standard_normal(D)
    a, b = w0.copy(), w0.copy()
    va, vb = np.array([v0], dtype=np.float32), np.array([v0], dtype=np.float32)
    oracle_mod.adagrad_row(a, 0, va, g, lr, eps, c)
    oracle_mod.adagrad_row(b, 0, vb, g, lr * math.sqrt(c), eps * math.sqrt(c), 1.0)
    np.testing.assert_allclose(a, b, rtol=1e-6)
    assert va[0] == vb[0] == np.float32(v0 + np.dot(g, g))
    expect = w0[0] - lr * g / (math.sqrt((v0 + np.dot(g, g)) / c) + eps)   # uses the UPDATED moment
    np.testing.assert_allclose(a[0], expect, rtol=1e-6)
    stale = w0[0] - lr * g / (math.sqrt(v0 / c) + eps)                      # a step with the old moment must differ
    assert np.abs(a[0] - stale).max() > 1e-4


def test_zero_gradient_at_zero_moment_leaves_the_row_for_every_eps(oracle_mod):
    # Algorithm 1 step 6 at v = 0, g = 0: the update term eta * 0 / (0 + eps) is 0 for every eps > 0, and the limit is
    # the value taken at eps = 0 (no 0/0): the row and its moment keep their bits.  A nonzero gradient at eps = 0 is
    # the closed form lr * sqrt(c) * g / ||g|| - finite.
    w0 = np.array([[0.25, -1.5, 3.0, 0.0]], dtype=np.float32)
    for eps in (0.0, 1e-8, 1.0):
        tab, v = w0.copy(), np.zeros(1, dtype=np.float32)
        oracle_mod.adagrad_row(tab, 0, v, np.zeros(4), 0.01, eps, 2.0)
        assert np.array_equal(tab.view(np.uint32), w0.view(np.uint32)) and v[0] == 0.0
    tab, v = w0.copy(), np.zeros(1, dtype=np.float32)
    g = np.array([3.0, 0.0, -4.0, 0.0])
    oracle_mod.adagrad_row(tab, 0, v, g, 0.01, 0.0, 4.0)
    np.testing.assert_allclose(tab[0].astype(np.float64) - w0[0], -0.01 * 2.0 * g / 5.0, atol=1e-7)
    assert v[0] == 25.0
    # with a moment already there a zero gradient still changes nothing (step * 0)
    tab, v = w0.copy(), np.array([2.0], dtype=np.float32)
    oracle_mod.adagrad_row(tab, 0, v, np.zeros(4), 0.01, 0.0, 1.0)
    assert np.array_equal(tab.view(np.uint32), w0.view(np.uint32)) and v[0] == 2.0


def test_larger_c_means_larger_step(oracle_mod):
    rng = np.random.default_rng(8)
    g = rng.standard_normal(8)
    w0 = np.zeros((1, 8), dtype=np.float32)
    norms = []
    for c in (0.5, 1.0, 2.0, 4.0, 8.0):
        tab = w0.copy()
        v = np.array([3.0], dtype=np.float32)
        oracle_mod.adagrad_row(tab, 0, v, g, 0.01, 1e-8, c)
        norms.append(np.linalg.norm(tab[0]))
    assert all(n2 > n1 for n1, n2 in zip(norms, norms[1:]))
    np.testing.assert_allclose(norms[3] / norms[1], 2.0, rtol=1e-5)          # step ~ sqrt(c)


def test_d1_tables_match_library_sparse_adagrad(oracle_mod):
    # For D = 1 a row IS a parameter, so c = 1 row-wise AdaGrad is the library's element-wise AdaGrad; the library
    # coalesces duplicate ids of a sparse gradient before the step.  Pins forward + dedup + sum + step end to end.
    rng = np.random.default_rng(9)
    R, B, lr, eps, v0 = 13, 7, 0.1, 1e-6, 0.3
    lens = rng.integers(0, 5, size=B)
    offsets = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    idx = rng.integers(0, R, size=int(lens.sum())).astype(np.int64)
    w0 = rng.standard_normal((R, 1)).astype(np.float32)
    gout = rng.standard_normal((B, 1)).astype(np.float32)

    emb = torch.nn.EmbeddingBag(R, 1, mode="sum", sparse=True, dtype=torch.float64)
    with torch.no_grad():
        emb.weight.copy_(torch.from_numpy(w0).double())
    opt = torch.optim.Adagrad(emb.parameters(), lr=lr, eps=eps, initial_accumulator_value=v0)
    out_ref = emb(torch.from_numpy(idx), torch.from_numpy(offsets[:-1]))
    out_ref.backward(torch.from_numpy(gout).double())
    opt.step()

    tab = w0.copy()
    out = oracle_mod.forward([tab], idx, offsets, B, "sum")
    np.testing.assert_allclose(out, out_ref.detach().numpy(), rtol=1e-6, atol=1e-7)
    state = np.full(R, v0, dtype=np.float32)
    res = oracle_mod.backward_rowwise_adagrad([tab], state, gout, idx, offsets, B, "sum", lr, eps, 1.0)
    np.testing.assert_allclose(tab, emb.weight.detach().numpy(), rtol=2e-6, atol=1e-7)
    np.testing.assert_allclose(state, opt.state[emb.weight]["sum"].numpy()[:, 0], rtol=1e-6)
    assert np.array_equal(res.unique_rows, np.unique(idx))


# ---------------------------------------------------------------- backward as a whole
@pytest.mark.parametrize("pooling", ["sum", "mean"])
def test_backward_equals_dense_brute_force(oracle_mod, pooling):
    # G_t = P_t^T . grad_out_t, then the closed-form step for rows with a nonzero column of P; all else bit-identical
    rng = np.random.default_rng(10)
    lr, eps, c, B = 0.02, 1e-8, 2.0, 6
    for trial in range(4):
        tables, idx, offsets = tiny_problem(rng, B=B, maxL=5)
        Ds = [a.shape[1] for a in tables]
        Rs = [a.shape[0] for a in tables]
        gout = rng.standard_normal((B, sum(Ds))).astype(np.float32)
        state0 = rng.random(sum(Rs)).astype(np.float32)
        new_tabs = [a.copy() for a in tables]
        state = state0.copy()
        res = oracle_mod.backward_rowwise_adagrad(new_tabs, state, gout, idx, offsets, B, pooling, lr, eps, c)
        col, base, touched_total = 0, 0, 0
        for t, Wt in enumerate(tables):
            P = count_matrix(t, Rs[t], idx, offsets, B, pooling)
            cnt = count_matrix(t, Rs[t], idx, offsets, B, "sum").sum(0)
            G = P.T @ gout[:, col:col + Ds[t]].astype(np.float64)
            for r in range(Rs[t]):
                if cnt[r] == 0:
                    assert np.array_equal(new_tabs[t][r].view(np.uint32), Wt[r].view(np.uint32))
                    assert state[base + r].view(np.uint32) == state0[base + r].view(np.uint32)
                else:
                    touched_total += 1
                    vn = float(state0[base + r]) + float(G[r] @ G[r])
                    np.testing.assert_allclose(state[base + r], vn, rtol=1e-6)
                    np.testing.assert_allclose(new_tabs[t][r], Wt[r] - lr / (math.sqrt(vn / c) + eps) * G[r],
                                               rtol=1e-5, atol=1e-7)
                    g_scan, hits = oracle_mod.row_gradient_by_scan(t, r, Ds[t], col, gout, idx, offsets, B, pooling)
                    assert hits == cnt[r]
                    np.testing.assert_allclose(g_scan, G[r], rtol=1e-12, atol=1e-12)
            col += Ds[t]
            base += Rs[t]
        assert res.U == touched_total


def test_duplicates_collapse_to_one_update_with_summed_gradient(oracle_mod):
    # a row hit twice with g and -g: summed gradient is zero => weights and moment keep their values
    # (two separate updates would have added 2*||g||^2 to the moment)
    Wt = np.ones((3, 4), dtype=np.float32)
    idx = np.array([1, 1], dtype=np.int64)
    offsets = np.array([0, 1, 2], dtype=np.int64)
    g = np.array([[1.0, -2.0, 3.0, 0.5]], dtype=np.float32)
    gout = np.concatenate([g, -g])
    state = np.array([0.5, 0.25, 0.125], dtype=np.float32)
    tab = Wt.copy()
    res = oracle_mod.backward_rowwise_adagrad([tab], state, gout, idx, offsets, 2, "sum", 0.1, 1e-8, 1.0)
    assert res.U == 1 and res.unique_rows.tolist() == [1] and res.seg_start.tolist() == [0, 2]
    assert np.array_equal(tab, Wt) and state.tolist() == [0.5, 0.25, 0.125]
    # and with g, g: moment grows by ||2g||^2, not 2||g||^2
    tab = Wt.copy()
    state = np.zeros(3, dtype=np.float32)
    oracle_mod.backward_rowwise_adagrad([tab], state, np.concatenate([g, g]), idx, offsets, 2, "sum", 0.1, 1e-8, 1.0)
    assert state[1] == np.float32(4.0 * float((g.astype(np.float64) ** 2).sum()))


def test_same_id_twice_in_one_bag_counts_twice(oracle_mod):
    Wt = np.zeros((2, 2), dtype=np.float32)
    gout = np.array([[1.0, 2.0]], dtype=np.float32)
    state = np.zeros(2, dtype=np.float32)
    tab = Wt.copy()
    oracle_mod.backward_rowwise_adagrad([tab], state, gout, np.array([0, 0], dtype=np.int64),
                                        np.array([0, 2], dtype=np.int64), 1, "sum", 1.0, 0.0 + 1e-12, 1.0)
    assert state[0] == np.float32(4.0 + 16.0)                        # ||2*g||^2
    np.testing.assert_allclose(tab[0], -np.array([2.0, 4.0]) / math.sqrt(20.0), rtol=1e-6)


def test_zero_gradient_touched_row_keeps_its_bits(oracle_mod):
    Wt = np.full((2, 2), 0.3, dtype=np.float32)
    state = np.zeros(2, dtype=np.float32)
    tab = Wt.copy()
    res = oracle_mod.backward_rowwise_adagrad([tab], state, np.zeros((1, 2), dtype=np.float32), np.array([1], dtype=np.int64),
                                              np.array([0, 1], dtype=np.int64), 1, "sum", 0.1, 1e-8, 1.0)
    assert res.U == 1 and np.array_equal(tab, Wt) and state.tolist() == [0.0, 0.0]


def test_checkpoint_resume_is_bit_identical(oracle_mod):
    # state is only (weights, moments): two steps in a row == step, copy out/in, step
    cfg = W.config("C1", B=16, rows_scale=1e-3)
    w0 = W.weight_rows(cfg, 0, torch.arange(cfg.rows[0])).numpy()
    runs = []
    for copy_between in (False, True):
        tab, st = w0.copy(), np.zeros(cfg.rows[0], dtype=np.float32)
        for step in range(2):
            idx, off = (x.numpy() for x in W.make_batch(cfg, step))
            go = W.make_grad_out(cfg, step).numpy()
            oracle_mod.backward_rowwise_adagrad([tab], st, go, idx, off, cfg.B, "sum", cfg.lr, cfg.eps, 4.0)
            if copy_between:
                tab, st = tab.copy(), st.copy()
        runs.append((tab, st))
    assert np.array_equal(runs[0][0], runs[1][0]) and np.array_equal(runs[0][1], runs[1][1])


def test_fp16_tables_round_once_to_nearest_even(oracle_mod):
    rng = np.random.default_rng(11)
    D = 8
    w0 = (rng.standard_normal((2, D)) * 0.01).astype(np.float16)
    g = rng.standard_normal(D)
    tab = w0.copy()
    v = np.array([1.0], dtype=np.float32)
    oracle_mod.adagrad_row(tab, 0, v, g, 0.01, 1e-8, 1.0)
    exact = w0[0].astype(np.float64) - 0.01 / (math.sqrt(1.0 + g @ g) + 1e-8) * g
    assert np.array_equal(tab[0].view(np.uint16), exact.astype(np.float16).view(np.uint16))
    assert np.array_equal(tab[1].view(np.uint16), w0[1].view(np.uint16))


# ---- 16-bit element types of the pooled output and of the upstream gradient ------------------------------------
def test_bf16_conversions_match_truncated_binary32(oracle_mod):
    # every finite bfloat16 pattern decodes to the binary32 value whose upper half it is
    bits = np.arange(0, 1 << 16, dtype=np.uint32)
    as_f32 = (bits << 16).astype(np.uint32).view(np.float32)
    for b in list(range(0, 1 << 16, 37)) + [0x0001, 0x007F, 0x0080, 0x7F7F, 0x8001, 0xFF7F]:
        x = oracle_mod.bf16_to_double(b)
        if np.isnan(as_f32[b]):
            assert math.isnan(x)
        else:
            assert x == float(as_f32[b]), hex(b)
    # encoding: against the library's float32 -> bfloat16 (round to nearest even) on values exact in binary32
    rng = np.random.default_rng(5)
    xs = np.concatenate([rng.standard_normal(3000).astype(np.float32) * np.float32(10.0) ** rng.integers(-30, 30, 3000),
                         np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38, 3.4e38, 1e-40, 9.2e-41,
                                   4.6e-41, 4.5e-41, np.inf, -np.inf], dtype=np.float32)]).astype(np.float32)
    want = torch.from_numpy(xs).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    for x, w in zip(xs, want):
        assert oracle_mod.double_to_bf16(float(x)) == int(w), (float(x), hex(int(w)))
    # ties go to the even mantissa: 1 + 2^-8 is halfway between 1 and 1 + 2^-7
    assert oracle_mod.double_to_bf16(1.0 + 2.0 ** -8) == 0x3F80
    assert oracle_mod.double_to_bf16(1.0 + 3 * 2.0 ** -8) == 0x3F82
    # a double just above the tie rounds up although binary32 would first round it onto the tie
    assert oracle_mod.double_to_bf16(1.0 + 2.0 ** -8 + 2.0 ** -40) == 0x3F81


def test_16bit_output_is_the_fp64_sum_rounded_once(oracle_mod):
    rng = np.random.default_rng(11)
    B = 6
    tabs, idx, off = tiny_problem(rng, T=3, B=B, maxL=5, Rs=(9, 4, 6), Ds=(4, 2, 3))
    # exact fp64 pooled sums, from the dense count-matrix form
    exact = np.concatenate([count_matrix(t, tabs[t].shape[0], idx, off, B, "sum") @ tabs[t].astype(np.float64)
                            for t in range(3)], axis=1)
    o16 = oracle_mod.forward(tabs, idx, off, B, "sum", out_dtype="f16")
    want16 = torch.from_numpy(exact).to(torch.float16).numpy()      # float64 -> binary16 in one rounding
    assert np.array_equal(o16.view(np.uint16), want16.view(np.uint16))
    ob = oracle_mod.forward(tabs, idx, off, B, "sum", out_dtype="bf16")
    back = np.array([oracle_mod.bf16_to_double(int(b)) for b in ob.reshape(-1)]).reshape(exact.shape)
    # nearest bfloat16: within half a unit in the last place (2^-8 relative), and exactly representable
    assert np.all(np.abs(back - exact) <= np.abs(exact) * 2.0 ** -8 + 1e-300)
    assert np.array_equal((back.astype(np.float32).view(np.uint32) & 0xFFFF), np.zeros(exact.shape, dtype=np.uint32))


def test_mean_of_equal_rows_is_the_row_also_where_a_16bit_output_ties(oracle_mod):
    # mean(w, w, ..., w) = w.  Every binary16 pattern of a small exponent range as table values: one in eight of them
    # lies exactly half-way between two bfloat16 values, so the bfloat16 output must be the row rounded to nearest
    # even - which a mean formed as sum * (1/L) misses for some L by the rounding error of the reciprocal.
    bits = np.arange(0x2000, 0x2400, dtype=np.uint16)                 # 1024 consecutive positive binary16 values
    Wt = np.concatenate([bits, bits | 0x8000]).view(np.float16).reshape(1, -1)
    as_f32 = Wt.astype(np.float32).view(np.uint32).astype(np.uint64)
    rne_bf16 = ((as_f32 + 0x7FFF + ((as_f32 >> 16) & 1)) >> 16).astype(np.uint16)   # float32 -> bfloat16, ties to even
    assert ((as_f32 & 0xFFFF) == 0x8000).sum() == Wt.size // 8         # the ties are really there
    for L in (1, 3, 7, 10, 49, 127, 200):
        idx = np.zeros(L, dtype=np.int64)
        off = np.array([0, L], dtype=np.int64)
        assert np.array_equal(oracle_mod.forward([Wt], idx, off, 1, "mean").view(np.uint32),
                              Wt.astype(np.float32).view(np.uint32)), L
        assert np.array_equal(oracle_mod.forward([Wt], idx, off, 1, "mean", out_dtype="f16").view(np.uint16),
                              Wt.view(np.uint16)), L
        assert np.array_equal(oracle_mod.forward([Wt], idx, off, 1, "mean", out_dtype="bf16").view(np.uint16),
                              rne_bf16), L


@pytest.mark.parametrize("io", ["f16", "bf16"])
def test_16bit_gradient_equals_its_exact_float32_image(oracle_mod, io):
    # a 16-bit upstream gradient converts to float32 without error, so the step must equal the float32 step
    rng = np.random.default_rng(13)
    B = 6
    tabs, idx, off = tiny_problem(rng, T=3, B=B, maxL=5, Rs=(9, 4, 6), Ds=(4, 2, 3))
    sumD = sum(a.shape[1] for a in tabs)
    g32 = torch.from_numpy(rng.standard_normal((B, sumD)).astype(np.float32))
    g16 = g32.to(torch.float16 if io == "f16" else torch.bfloat16)
    g16_np = g16.numpy() if io == "f16" else g16.view(torch.int16).numpy().view(np.uint16)
    ta, tb = [a.copy() for a in tabs], [a.copy() for a in tabs]
    va = np.zeros(sum(a.shape[0] for a in tabs), dtype=np.float32)
    vb = va.copy()
    ra = oracle_mod.backward_rowwise_adagrad(ta, va, g16_np, idx, off, B, "mean", 0.05, 1e-8, 2.0, grad_dtype=io)
    rb = oracle_mod.backward_rowwise_adagrad(tb, vb, g16.to(torch.float32).numpy(), idx, off, B, "mean", 0.05, 1e-8, 2.0)
    assert ra.U == rb.U and ra.U > 0
    for a, b in zip(ta, tb):
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
    assert np.array_equal(va.view(np.uint32), vb.view(np.uint32))
    assert not np.array_equal(ta[0], tabs[0])


# ---- plain SGD variant -------------------------------------------------------------------------------------
@pytest.mark.parametrize("pooling", ["sum", "mean"])
def test_sgd_equals_dense_gradient_step(oracle_mod, pooling):
    # the gradient of the pooled output with respect to the table is P^T . grad_out; SGD subtracts lr times it
    rng = np.random.default_rng(21)
    B = 5
    tables, idx, offsets = tiny_problem(rng)
    sumD = sum(a.shape[1] for a in tables)
    go = rng.standard_normal((B, sumD)).astype(np.float32)
    new = [a.copy() for a in tables]
    res = oracle_mod.backward_sgd(new, go, idx, offsets, B, pooling, lr=0.3)
    col = 0
    touched = 0
    for t, Wt in enumerate(tables):
        P = count_matrix(t, Wt.shape[0], idx, offsets, B, pooling)
        dense = Wt.astype(np.float64) - 0.3 * (P.T @ go[:, col:col + Wt.shape[1]].astype(np.float64))
        np.testing.assert_allclose(new[t], dense, rtol=1e-6, atol=1e-7)
        hit = P.sum(axis=0) > 0
        assert np.array_equal(new[t][~hit].view(np.uint32), Wt[~hit].view(np.uint32))     # untouched rows keep their bits
        touched += int(hit.sum())
        col += Wt.shape[1]
    assert res.U == touched


@pytest.mark.parametrize("mode", ["sum", "mean"])
def test_sgd_matches_library_embedding_bag_with_sgd(oracle_mod, mode):
    rng = np.random.default_rng(22)
    R, D, B = 11, 6, 7
    W0 = rng.standard_normal((R, D)).astype(np.float32)
    lens = rng.integers(0, 5, size=B)
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    idx = rng.integers(0, R, size=int(off[-1])).astype(np.int64)
    go = rng.standard_normal((B, D)).astype(np.float32)
    emb = torch.nn.EmbeddingBag(R, D, mode=mode, sparse=False)
    with torch.no_grad():
        emb.weight.copy_(torch.from_numpy(W0))
    opt = torch.optim.SGD(emb.parameters(), lr=0.25)
    out = emb(torch.from_numpy(idx), torch.from_numpy(off[:-1]))
    out.backward(torch.from_numpy(go))
    opt.step()
    mine = [W0.copy()]
    oracle_mod.backward_sgd(mine, go, idx, off, B, mode, lr=0.25)
    np.testing.assert_allclose(mine[0], emb.weight.detach().numpy(), rtol=1e-5, atol=1e-6)


# ---- non-pooled lookup --------------------------------------------------------------------------------------
def _seq_problem(rng, Rs=(9, 4, 6), Ds=(4, 8, 4), ns=(11, 0, 7), dtype=np.float32):
    tables = [rng.standard_normal((R, D)).astype(dtype) for R, D in zip(Rs, Ds)]
    toff = np.concatenate([[0], np.cumsum(ns)]).astype(np.int64)
    idx = np.concatenate([rng.integers(0, R, size=n) for R, n in zip(Rs, ns)]).astype(np.int64)
    return tables, idx, toff


def test_lookup_seq_is_row_indexing(oracle_mod):
    rng = np.random.default_rng(31)
    tables, idx, toff = _seq_problem(rng)
    out = oracle_mod.lookup_seq(tables, idx, toff)
    want = np.concatenate([tables[t][idx[toff[t]:toff[t + 1]]].reshape(-1) for t in range(3)])   # the library's gather
    assert np.array_equal(out.view(np.uint32), want.view(np.uint32))
    # 16-bit output: each element rounded once
    out16 = oracle_mod.lookup_seq(tables, idx, toff, out_dtype="f16")
    assert np.array_equal(out16.view(np.uint16), want.astype(np.float16).view(np.uint16))
    with pytest.raises(IndexError):
        oracle_mod.lookup_seq(tables, np.where(np.arange(idx.size) == 3, 99, idx), toff)


def test_backward_seq_equals_one_lookup_bags_and_dense_one_hot(oracle_mod):
    rng = np.random.default_rng(32)
    tables, idx, toff = _seq_problem(rng, Rs=(9,), Ds=(4,), ns=(25,))
    n, D = 25, 4
    g = rng.standard_normal((n, D)).astype(np.float32)
    v0 = rng.uniform(0.0, 1.0, 9).astype(np.float32)
    # (a) a sequence is the pooled layout with one lookup per bag: same rows, same bits
    a_w, a_v = [tables[0].copy()], v0.copy()
    U = oracle_mod.backward_seq(a_w, a_v, g.reshape(-1), idx, toff, lr=0.1, eps=1e-8, c=2.0)
    b_w, b_v = [tables[0].copy()], v0.copy()
    res = oracle_mod.backward_rowwise_adagrad(b_w, b_v, g, idx, np.arange(n + 1), n, "sum", 0.1, 1e-8, 2.0)
    assert U == res.U == len(set(idx.tolist()))
    assert np.array_equal(a_w[0].view(np.uint32), b_w[0].view(np.uint32)) and np.array_equal(a_v.view(np.uint32), b_v.view(np.uint32))
    # (b) dense form: G = onehot^T . g, v += ||G_r||^2, w -= lr / (sqrt(v/c) + eps) * G_r
    onehot = np.zeros((n, 9))
    onehot[np.arange(n), idx] = 1.0
    G = onehot.T @ g.astype(np.float64)
    v = v0.astype(np.float64) + (G * G).sum(axis=1)
    hit = onehot.sum(axis=0) > 0
    want = tables[0].astype(np.float64) - (0.1 / (np.sqrt(v / 2.0) + 1e-8))[:, None] * G
    np.testing.assert_allclose(a_w[0][hit], want[hit], rtol=1e-6)
    np.testing.assert_allclose(a_v[hit], v[hit], rtol=1e-6)
    assert np.array_equal(a_w[0][~hit].view(np.uint32), tables[0][~hit].view(np.uint32))
    assert np.array_equal(a_v[~hit].view(np.uint32), v0[~hit].view(np.uint32))


def test_backward_seq_several_tables_and_sgd(oracle_mod):
    rng = np.random.default_rng(33)
    tables, idx, toff = _seq_problem(rng)
    Ds, ns = (4, 8, 4), (11, 0, 7)
    total = sum(n * D for n, D in zip(ns, Ds))
    g = rng.standard_normal(total).astype(np.float32)
    new = [a.copy() for a in tables]
    U = oracle_mod.backward_seq(new, None, g, idx, toff, lr=0.5)
    base = 0
    count = 0
    for t in range(3):
        n, D = ns[t], Ds[t]
        gt = g[base:base + n * D].reshape(n, D).astype(np.float64)
        ids = idx[toff[t]:toff[t + 1]]
        want = tables[t].astype(np.float64)
        np.subtract.at(want, ids, 0.5 * gt)           # the library's scatter-add, duplicates accumulate
        np.testing.assert_allclose(new[t], want, rtol=1e-6, atol=1e-7)
        count += len(set(ids.tolist()))
        base += n * D
    assert U == count
    assert np.array_equal(new[1].view(np.uint32), tables[1].view(np.uint32))   # the empty table is untouched
