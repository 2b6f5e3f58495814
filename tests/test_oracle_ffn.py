"""Pins for the oracle's threshold / selection, sparse FFN, router, layer and staging (CPU only)."""
import math

import numpy as np
import pytest
from scipy import special, stats

import floe_synth as S
import oracle as O
from helpers import compact_from_paper_orientation, golden_values

G = golden_values("lemma_gaussian_threshold.txt")


# ---------------------------------------------------------------- threshold + selection
def test_threshold_is_order_statistic_and_count_matches():
    v = S.normal(S.stream_key(1, 98, S.KIND_MISC), 3584, 0.7).astype(np.float32)
    for pct, K in [(0, 3584), (50, 1792), (80, 716), (85, 537), (90, 358), (100, 0)]:
        tau = O.threshold_for_sparsity(v, pct)
        idx = O.select(v, tau)
        assert idx.size == int((np.abs(v) > tau).sum()) == K               # Alg. 1 line 3 invariant
        assert np.array_equal(idx, np.nonzero(np.abs(v) > np.float32(tau))[0])
        if 0 < pct:
            z = -(-3584 * pct // 100)
            assert tau == np.sort(np.abs(v))[z - 1]
            # smallest t with F(t) >= pct/100 (Eq. 6): F(tau) reaches the target, any smaller sample value does not
            F = lambda t: (np.abs(v) <= t).mean()
            assert F(tau) >= pct / 100 and F(np.nextafter(np.float32(tau), np.float32(0))) < pct / 100
    # paper-workload counts: K = f - ceil(f * pct / 100)
    for f, pct, K in [(3584, 80, 716), (14336, 50, 7168), (14336, 80, 2867), (14336, 90, 1433), (1408, 85, 211)]:
        vv = S.normal(S.stream_key(2, 98, S.KIND_MISC, f, pct), f).astype(np.float32)
        assert O.select(vv, O.threshold_for_sparsity(vv, pct)).size == K


def test_strict_comparison_on_exact_ties():
    v = np.array([0.5, -0.5, 0.25, -0.75, 0.5000001, 0.0], dtype=np.float32)
    assert list(O.select(v, 0.5)) == [3, 4]
    assert list(O.select(v, -1.0)) == [0, 1, 2, 3, 4, 5]
    assert list(O.select(v, 10.0)) == []


def test_gaussian_closed_form_threshold_and_dropped_energy():
    # App. A, Gaussian threshold lemma, with the numbers the paper prints.
    n, sigma = 1_000_000, 1.28
    v = S.normal(S.stream_key(3, 98, S.KIND_MISC), n, sigma).astype(np.float32)
    se = 3.0 / math.sqrt(n)
    # eta = 0.5 <-> 50 % sparsity: tau / sigma -> Phi^-1(0.75) ~ 0.674;  eta = 0.05 <-> 95 %: Phi^-1(0.975) ~ 1.960
    for pct, key in [(50, "inv_cdf_0.75"), (95, "inv_cdf_0.975")]:
        val, tol = G[key]
        tau = O.threshold_for_sparsity(v, pct)
        assert abs(tau / sigma - val) < tol + 6 * se
    # dropped energy fraction 1 - eta - 2 z phi(z) with the printed 2 z phi(z) at eta = 0.5 and eta = e^-4
    e = (v.astype(np.float64) ** 2).sum()
    for eta, key in [(0.5, "m2_at_eta_0.5"), (math.exp(-4), "m2_at_eta_exp_-4")]:
        m2, tol = G[key]
        tau = sigma * stats.norm.ppf(1 - eta / 2)                            # closed-form threshold of the lemma
        idx = O.select(v, tau)
        assert abs(idx.size / n - eta) < 3 * math.sqrt(eta * (1 - eta) / n) + 1e-4
        kept = (v[idx].astype(np.float64) ** 2).sum()
        assert abs((e - kept) / e - (1 - eta - m2)) < tol + 0.004


# ---------------------------------------------------------------- SiLU and the sparse FFN
def test_silu_spot_values():
    # d = 1: y = SiLU(x * w_gate) * v * w_down with x = v = w_down = 1
    gs = np.arange(-3.0, 0.5, 1 / 256, dtype=np.float64).astype(np.float16)
    ys = []
    for g in gs:
        gd = np.array([[[g], [1.0]]], dtype=np.float16)
        h, y = O.sparse_ffn(gd, np.array([1.0], np.float16), np.array([1.0], np.float32), np.array([0], np.int32))
        assert h[0] == y[0]
        ys.append(y[0])
    ys = np.array(ys)
    val, tol = G["silu_min"]
    assert abs(ys.min() - val) < tol
    assert abs(ys.min() - (-0.27846)) < 1e-4 and abs(float(gs[ys.argmin()]) - (-1.2785)) < 4e-3
    assert ys[np.where(gs == 0)[0][0]] == 0.0
    np.testing.assert_allclose(ys, gs.astype(np.float64) * special.expit(gs.astype(np.float64)), rtol=1e-13, atol=1e-15)


def _paper_orientation_case(seed, d, f):
    w_gate = S.normal_f16(S.stream_key(seed, 97, S.KIND_W_GATE), (d, f), 0.05)
    w_up = S.normal_f16(S.stream_key(seed, 97, S.KIND_W_UP), (d, f), 0.05)
    w_down = S.normal_f16(S.stream_key(seed, 97, S.KIND_W_DOWN), (f, d), 0.05)
    x = S.normal_f16(S.stream_key(seed, 97, S.KIND_X), (d,), 1.0)
    return w_gate, w_up, w_down, x


def test_dense_ffn_is_equation_one():
    d, f = 96, 160
    w_gate, w_up, w_down, x = _paper_orientation_case(11, d, f)
    x64, wg, wu, wd = (a.astype(np.float64) for a in (x, w_gate, w_up, w_down))
    ref = ((x64 @ wg) * special.expit(x64 @ wg) * (x64 @ wu)) @ wd          # Eq. 1 with library mat-vecs
    gd = compact_from_paper_orientation(w_gate, w_down)
    y = O.dense_ffn(np.ascontiguousarray(w_up.T).astype(np.float32), gd, x)
    np.testing.assert_allclose(y, ref, rtol=1e-11, atol=1e-13)


@pytest.mark.parametrize("pct", [0, 50, 90, 100])
def test_sparse_ffn_equals_masked_dense(pct):
    d, f = 96, 160
    w_gate, w_up, w_down, x = _paper_orientation_case(12, d, f)
    x64, wg, wu, wd = (a.astype(np.float64) for a in (x, w_gate, w_up, w_down))
    gd = compact_from_paper_orientation(w_gate, w_down)
    v = (x64 @ wu).astype(np.float32)
    tau = O.threshold_for_sparsity(v, pct)
    idx = O.select(v, tau)
    h, y = O.sparse_ffn(gd, x, v, idx)
    vs = np.where(np.abs(v) > np.float32(tau), v, np.float32(0)).astype(np.float64)   # S_t, Eq. 5 (strict as Alg. 1)
    ref = ((x64 @ wg) * special.expit(x64 @ wg) * vs) @ wd
    np.testing.assert_allclose(y, ref, rtol=1e-10, atol=1e-13)
    np.testing.assert_allclose(h, ((x64 @ wg) * special.expit(x64 @ wg) * vs)[idx], rtol=1e-12, atol=1e-15)
    y_lit = O.masked_dense_ffn(np.ascontiguousarray(w_up.T).astype(np.float32), gd, x, tau)
    np.testing.assert_allclose(y_lit, ref, rtol=1e-10, atol=1e-13)
    if pct == 0:     # zero sparsity: the sparse definition reduces to Eq. 1 (up to v being carried as binary32)
        np.testing.assert_allclose(y, O.dense_ffn(np.ascontiguousarray(w_up.T).astype(np.float32), gd, x), rtol=1e-6, atol=1e-7)
    if pct == 100:
        assert idx.size == 0 and np.all(y == 0)


def test_sparse_ffn_staged_rows_give_same_result():
    d, f = 64, 80
    w_gate, w_up, w_down, x = _paper_orientation_case(13, d, f)
    gd = compact_from_paper_orientation(w_gate, w_down)
    v = (x.astype(np.float64) @ w_up.astype(np.float64)).astype(np.float32)
    idx = O.select(v, O.threshold_for_sparsity(v, 70))
    staged = O.stage_rows(gd, idx)
    assert staged.tobytes() == gd[idx].tobytes() and staged.nbytes == idx.size * 4 * d   # K * 2d * num_bytes
    h0, y0 = O.sparse_ffn(gd, x, v, idx)
    h1, y1 = O.sparse_ffn(staged, x, v, idx, staged=True)
    assert np.array_equal(y0, y1) and np.array_equal(h0, h1)


def test_tiny_brute_force_with_python_floats():
    # 2 channels, d = 2, every product written out
    gd = np.array([[[0.5, -1.0], [2.0, 0.25]], [[1.5, 0.5], [-1.0, 4.0]]], dtype=np.float16)
    x = np.array([2.0, 1.0], dtype=np.float16)
    v = np.array([0.75, -3.0], dtype=np.float32)
    g0, g1 = 2.0 * 0.5 + 1.0 * -1.0, 2.0 * 1.5 + 1.0 * 0.5           # 0.0, 3.5
    h0, h1 = g0 / (1 + math.exp(-g0)) * 0.75, g1 / (1 + math.exp(-g1)) * -3.0
    h, y = O.sparse_ffn(gd, x, v, np.array([0, 1], np.int32))
    assert h[0] == h0 and h[1] == h1
    assert y[0] == h0 * 2.0 + h1 * -1.0 and y[1] == h0 * 0.25 + h1 * 4.0
    h, y = O.sparse_ffn(gd, x, v, np.array([1], np.int32))
    assert y[0] == h1 * -1.0 and y[1] == h1 * 4.0


# ---------------------------------------------------------------- router and layer
def test_router_softmax_topk():
    n, d = 8, 256
    wr = S.normal_f16(S.stream_key(21, 96, S.KIND_ROUTER), (n, d), 0.05)
    x = S.normal_f16(S.stream_key(21, 96, S.KIND_X), (d,), 1.0)
    logits = wr.astype(np.float64) @ x.astype(np.float64)
    p_ref = special.softmax(logits)
    ids, w, p = O.router(wr, x, 2, True)
    np.testing.assert_allclose(p, p_ref, rtol=1e-12)
    assert abs(p.sum() - 1) < 1e-12 and abs(w.sum() - 1) < 1e-12
    order = np.argsort(-p_ref, kind="stable")
    assert list(ids) == list(order[:2])
    np.testing.assert_allclose(w, p_ref[order[:2]] / p_ref[order[:2]].sum(), rtol=1e-12)
    ids3, w3, _ = O.router(wr, x, 3, False)
    assert list(ids3) == list(order[:3])
    np.testing.assert_allclose(w3, p_ref[order[:3]], rtol=1e-12)
    # permuting the experts permutes the ids only
    perm = np.array([3, 0, 7, 1, 6, 2, 5, 4])
    ids_p, w_p, _ = O.router(wr[perm], x, 2, True)
    assert list(perm[ids_p]) == list(ids)
    np.testing.assert_allclose(w_p, w, rtol=1e-12)
    # ties go to the lower expert id
    ids_t, w_t, _ = O.router(np.zeros((4, d), np.float16), x, 2, True)
    assert list(ids_t) == [0, 1] and np.allclose(w_t, 0.5)


def _small_layer(seed, n_all, d, f, bits, group):
    experts, raw = [], []
    for e in range(n_all):
        w_up, gd = S.expert_weights(seed, 95, d, f, 0, e)
        experts.append(O.quantize(w_up, bits, group) + (gd,))
        raw.append((w_up, gd))
    return experts, raw


def test_layer_is_weighted_sum_of_expert_ffns():
    d, f, bits, group, n, top_k, n_shared, T = 128, 96, 3, 32, 6, 2, 1, 3
    experts, _ = _small_layer(31, n + n_shared, d, f, bits, group)
    wr = S.router_weights(31, 95, n, d)
    x = S.tokens(31, 95, T, d)
    tau = np.zeros((T, n + n_shared), np.float32)
    for t in range(T):
        for e in range(n + n_shared):
            v = O.up_gemv(*experts[e][:3], d, bits, group, x[t])
            tau[t, e] = O.threshold_for_sparsity(v, 75)
    for renorm in (True, False):
        res = O.moe_layer(experts, n_shared, top_k, renorm, wr, x, tau, bits, group)
        for t in range(T):
            ids, w, _ = O.router(wr, x[t], top_k, renorm)
            assert list(res["ids"][t]) == list(ids)
            acc = np.zeros(d)
            slots = list(zip(ids, w)) + [(n + s, 1.0) for s in range(n_shared)]
            for s, (e, we) in enumerate(slots):
                v = O.up_gemv(*experts[e][:3], d, bits, group, x[t])
                idx = O.select(v, tau[t, e])
                assert res["counts"][t, s] == idx.size == f - (-(-f * 75 // 100))
                acc += we * O.sparse_ffn(experts[e][3], x[t], v, idx)[1]
            np.testing.assert_allclose(res["y"][t], acc, rtol=1e-12, atol=1e-15)
            assert np.array_equal(res["out"][t], acc.astype(np.float16))        # one rounding, to nearest even


def test_layer_with_all_experts_and_equal_logits_is_the_mean():
    d, f, bits, group, n = 64, 64, 4, 64, 4
    experts, _ = _small_layer(32, n, d, f, bits, group)
    x = S.tokens(32, 95, 1, d)
    tau = np.full((1, n), -1.0, np.float32)                                       # keep every channel
    res = O.moe_layer(experts, 0, n, True, np.zeros((n, d), np.float16), x, tau, bits, group)
    ys = []
    for e in range(n):
        w_hat = O.dequantize(*experts[e][:3], d, bits, group)
        ys.append(O.dense_ffn(w_hat, experts[e][3], x[0]))                         # 0 % sparsity == Eq. 1
    np.testing.assert_allclose(res["y"][0], np.mean(ys, axis=0), rtol=1e-5, atol=1e-9)   # v carried as binary32
    assert np.all(res["counts"] == f)


# ---------------------------------------------------------------- the three sparsification candidates (Sec. 3.2.1)
def _paper_orientation_expert(seed, d, f):
    rng_key = S.stream_key(seed, 97, S.KIND_MISC)
    w_gate = S.normal(rng_key, d * f, 0.05).reshape(d, f).astype(np.float16)          # R^{d x f}
    w_up = S.normal(S.stream_key(seed, 96, S.KIND_MISC), d * f, 0.05).reshape(d, f).astype(np.float16)
    w_down = S.normal(S.stream_key(seed, 95, S.KIND_MISC), f * d, 0.05).reshape(f, d).astype(np.float16)
    x = S.normal(S.stream_key(seed, 94, S.KIND_MISC), d, 1.0).astype(np.float16)
    return w_gate, w_up, w_down, x


def test_sparsified_ffn_is_eq1_with_the_sparsity_function_on_the_chosen_activation():
    """Eq. 1 with S_t (Eq. 5) on a_up, a_gate or a_down (Eq. 3-4), written with library mat-vecs in the paper's
    orientation: catches a wrong activation, a swapped operand, a non-strict comparison."""
    d, f = 96, 160
    w_gate, w_up, w_down, x = _paper_orientation_expert(5, d, f)
    gd = compact_from_paper_orientation(w_gate, w_down)
    x64 = x.astype(np.float64)
    a_up = (x64 @ w_up.astype(np.float64)).astype(np.float32)                          # the caller's a_up, binary32
    g = x64 @ w_gate.astype(np.float64)
    a_gate = g / (1.0 + np.exp(-g))
    a_down = a_gate * a_up.astype(np.float64)
    for which, act in [(O.SPARSIFY_UP, a_up.astype(np.float64)), (O.SPARSIFY_GATE, a_gate), (O.SPARSIFY_DOWN, a_down)]:
        mags = np.sort(np.abs(act.astype(np.float32)))
        for tau in [-1.0, float(mags[f // 2]), float(mags[(9 * f) // 10]), float(mags[-1])]:
            keep = np.abs(act.astype(np.float32)) > np.float32(tau)                    # strict, in binary32
            ref = (np.where(keep, a_down, 0.0)) @ w_down.astype(np.float64)
            y, idx, got_act = O.sparsified_ffn(which, gd, x, a_up, tau)
            assert np.array_equal(idx, np.nonzero(keep)[0])
            np.testing.assert_allclose(got_act, act, rtol=1e-12, atol=1e-15)
            np.testing.assert_allclose(y, ref, rtol=1e-10, atol=1e-12)
    # a threshold that sits exactly on one value keeps that channel out (strict comparison of Alg. 1)
    tau = float(np.abs(a_up)[7])
    _, idx, _ = O.sparsified_ffn(O.SPARSIFY_UP, gd, x, a_up, tau)
    assert 7 not in idx


def test_sparsified_ffn_on_a_up_is_the_sparse_expert_forward_and_all_three_are_dense_below_zero():
    d, f = 128, 192
    w_gate, w_up, w_down, x = _paper_orientation_expert(6, d, f)
    gd = compact_from_paper_orientation(w_gate, w_down)
    w_up_cm = np.ascontiguousarray(w_up.T.astype(np.float32))
    a_up = (x.astype(np.float64) @ w_up.astype(np.float64)).astype(np.float32)
    tau = float(np.sort(np.abs(a_up))[f // 2])
    y_up, idx, _ = O.sparsified_ffn(O.SPARSIFY_UP, gd, x, a_up, tau)
    np.testing.assert_allclose(y_up, O.masked_dense_ffn(w_up_cm, gd, x, tau), rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(y_up, O.sparse_ffn(gd, x, a_up, idx)[1], rtol=1e-9, atol=1e-12)
    dense = O.dense_ffn(w_up_cm, gd, x)                   # (keeps x.W_up in double; a_up above is its binary32 rounding)
    for which in (O.SPARSIFY_UP, O.SPARSIFY_GATE, O.SPARSIFY_DOWN):
        np.testing.assert_allclose(O.sparsified_ffn(which, gd, x, a_up, -1.0)[0], dense, rtol=0, atol=2e-7 * np.abs(dense).max())


def test_loss_ordering_of_the_three_candidates_on_gaussian_inputs():
    """Theorem of Sec. 3.2.1 (L_down <= L_up < L_gate), the part that holds whatever the distributions: at equal
    sparsity, thresholding a_down loses least, because it drops the smallest terms of the very sum it approximates.
    (L_up < L_gate rests on the paper's assumption about the gate activations of real models, App. A; with zero-mean
    Gaussian synthetic weights half of the SiLU outputs are near zero and the order of those two is the other way
    round, which the test only records.)  Averaged over tokens; the margins are far above the sampling noise."""
    d, f, n_tok = 256, 1024, 24
    w_gate, w_up, w_down, _ = _paper_orientation_expert(7, d, f)
    gd = compact_from_paper_orientation(w_gate, w_down)
    w_up_cm = np.ascontiguousarray(w_up.T.astype(np.float32))
    for pct in (50, 80):
        loss = {0: 0.0, 1: 0.0, 2: 0.0}
        for t in range(n_tok):
            x = S.normal(S.stream_key(8, 93, S.KIND_MISC, t), d, 1.0).astype(np.float16)
            a_up = (x.astype(np.float64) @ w_up.astype(np.float64)).astype(np.float32)
            dense = O.dense_ffn(w_up_cm, gd, x)
            for which in (0, 1, 2):
                _, _, act = O.sparsified_ffn(which, gd, x, a_up, -1.0)
                tau = O.threshold_for_sparsity(act.astype(np.float32), pct)
                y, idx, _ = O.sparsified_ffn(which, gd, x, a_up, tau)
                assert idx.size == f - (-(-f * pct // 100))
                loss[which] += float(((dense - y) ** 2).sum())
        assert loss[2] < 0.8 * loss[0] and loss[2] < 0.8 * loss[1], (pct, loss)
        print(f"sparsity {pct} %: L_down {loss[2]:.1f}  L_up {loss[0]:.1f}  L_gate {loss[1]:.1f}")
