"""GPU parity of the prefetched offloaded layer: floe_moe_layer_prefetch + floe_moe_layer_decode_prefetched.

Expected sets come from the oracle (router, up GEMV, selection on the earlier and on the real hidden state); the
thresholds sit in wide gaps of |v|, so the lists do not hinge on rounding order and every count is exact."""
import numpy as np
import pytest
import torch

import floe_synth as S
import oracle as O

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _threads():
    O.set_threads(16)
    yield
    O.set_threads(1)


def _gap_threshold(values, pct):
    """Middle of the widest gap between neighbouring |v| (pooled over the tokens) near the pct-th percentile."""
    a = np.sort(np.abs(np.concatenate(values).astype(np.float64)))
    z = int(a.size * pct / 100)
    lo, hi = max(1, z - 12), min(a.size - 1, z + 12)
    k = max(range(lo, hi), key=lambda i: a[i] - a[i - 1])
    return np.float32(0.5 * (a[k] + a[k - 1]))


def _case(seed, d, f, group, n, n_shared, top_k, renorm, T, pct, rho, cap):
    import gpu_common as G
    import paper_2505_05950_amd as F
    bits = 2
    n_all = n + n_shared
    experts_np, experts_dev, pinned = [], [], []
    for e in range(n_all):
        w_up, gd = S.expert_weights(seed, 4, d, f, 0, e)
        ex_np, _ = G.make_expert(w_up, gd, bits, group)
        host = torch.from_numpy(gd).pin_memory()
        pinned.append(host)
        c, s_, z = (G.dev(ex_np[0].view(np.int32)).view(torch.int32), G.dev(ex_np[1]), G.dev(ex_np[2]))
        experts_np.append(ex_np)
        experts_dev.append(F.Expert(d, f, bits, group, c, s_, z, host))
    wr = S.router_weights(seed, 4, n, d)
    x_cur = S.tokens(seed, 4, T, d, layer=300)
    noise = S.tokens(seed, 4, T, d, layer=301)
    x_new = (rho * x_cur.astype(np.float64) + np.sqrt(1 - rho * rho) * noise.astype(np.float64)).astype(np.float16)

    def routed(x):
        ids, w, _ = O.router(wr, x, top_k, renorm)
        return list(zip(ids.tolist(), w.tolist())) + [(n + s, 1.0) for s in range(n_shared)]

    # every (input, expert) pair that is evaluated, for the thresholds
    v_of = {}
    for tag, xs in (("cur", x_cur), ("new", x_new)):
        for t in range(T):
            for e, _ in routed(xs[t]):
                v_of[(tag, t, e)] = O.up_gemv(*experts_np[e][:3], d, bits, group, xs[t])
    tau = np.zeros(n_all, np.float32)
    for e in range(n_all):
        vals = [v for (tag, t, ee), v in v_of.items() if ee == e]
        tau[e] = _gap_threshold(vals, pct) if vals else np.float32(1.0)

    L = F.Layer(experts_dev, n_shared, top_k, renorm, G.dev(wr), G.dev(tau), False, gd_on_host=True)
    slots = top_k + n_shared
    n_tasks = T * slots
    side, miss = torch.cuda.Stream(), torch.cuda.Stream()
    P = F.Prefetch(L, T, cap, side)
    M = F.MissPath(miss, n_tasks, G.DEV)
    stats = torch.zeros((T, slots, 4), dtype=torch.int32, device=G.DEV)
    pstats = torch.zeros((n_tasks, 4), dtype=torch.int32, device=G.DEV)
    ws_pref = L.new_workspace(T)
    xc, xn = G.dev(x_cur), G.dev(x_new)
    torch.cuda.synchronize()
    F.floe_moe_layer_prefetch(L, P, xc, ws_pref)
    y = F.floe_moe_layer_decode_prefetched(L, P, M, xn, stats=stats, prefetch_stats=pstats)
    torch.cuda.synchronize()

    # the same layer through the plain offloaded path (everything staged after selection)
    staging = torch.empty((n_tasks, f, 2, d), dtype=torch.float16, device=G.DEV)
    ev_a, ev_b = torch.cuda.Event(), torch.cuda.Event()
    y_off = F.floe_moe_layer_decode_offloaded(L, xn, staging, f, side, ev_a, ev_b)
    torch.cuda.synchronize()

    st = stats.cpu().numpy().reshape(T, slots, 4).copy().view(F.SLOT_STAT_DTYPE).reshape(T, slots)
    ps = pstats.cpu().numpy().copy().view(F.PREFETCH_STAT_DTYPE).reshape(T, slots)
    row_of = P.row_of.cpu().numpy()
    pred_expert = P.pred_expert.cpu().numpy().reshape(T, slots)
    pred_count = P.pred_count.cpu().numpy().reshape(T, slots)
    stg = P.staging.cpu().numpy()
    ovf = M.overflow.cpu().numpy().reshape(T, slots)
    any_overflow = False
    y_ref = np.zeros((T, d))
    for t in range(T):
        pred = routed(x_cur[t])
        act = routed(x_new[t])
        for s, (e, we) in enumerate(act):
            A = O.select(v_of[("new", t, e)], float(tau[e]))
            assert st[t, s]["expert"] == e and st[t, s]["count"] == A.size
            # which predicted slab held this expert?
            sp = next((k for k, (ep, _) in enumerate(pred) if ep == e), None)
            if sp is None:
                Pset, kept = np.zeros(0, np.int32), 0
                assert ps[t, s]["expert_predicted"] == 0 and ps[t, s]["predicted"] == 0
                slab = n_tasks + t * slots + s
            else:
                Pset = O.select(v_of[("cur", t, e)], float(tau[e]))
                kept = min(Pset.size, cap)
                assert pred_expert[t, sp] == e and pred_count[t, sp] == kept
                assert ps[t, s]["expert_predicted"] == 1 and ps[t, s]["predicted"] == kept
                slab = t * slots + sp
                # predicted rows: byte for byte the host chunks, in list order; the map points at them
                rmap = row_of[t * slots + sp]
                assert np.array_equal(np.nonzero(rmap >= 0)[0], np.sort(Pset[:kept]))
                assert np.array_equal(rmap[Pset[:kept]], np.arange(kept))
                assert np.array_equal(stg[slab, :kept], pinned[e].numpy()[Pset[:kept]])
            staged_set = Pset[:kept]
            hits = np.intersect1d(A, staged_set)
            misses = np.setdiff1d(A, staged_set)            # ascending, as the kernel lists them
            assert ps[t, s]["hits"] == hits.size and ps[t, s]["misses"] == misses.size
            fit = max(0, min(misses.size, cap - kept))
            assert ovf[t, s] == (1 if kept + misses.size > cap else 0)
            any_overflow |= bool(ovf[t, s])
            assert np.array_equal(stg[slab, kept:kept + fit], pinned[e].numpy()[misses[:fit]])
            used = np.union1d(hits, misses[:fit]).astype(np.int32)
            y_ref[t] += we * O.sparse_ffn(experts_np[e][3], x_new[t], v_of[("new", t, e)], used)[1]
    yn = y.cpu().numpy().astype(np.float64)
    for t in range(T):
        assert G.rel_err(yn[t], y_ref[t]) <= G.Y_TIGHT
    if not any_overflow:
        assert torch.equal(y, y_off), "prefetched and plainly offloaded decode must agree bit for bit"
    return ps


def test_prefetched_layer_matches_offloaded_layer_and_oracle():
    ps = _case(31, 1024, 700, 64, 6, 1, 2, True, 2, 80, 0.95, 400)
    assert ps["hits"].sum() > 0 and ps["misses"].sum() > 0


def test_prefetch_with_unrelated_hidden_state_still_gives_the_right_result():
    # rho = 0: the prediction is useless (other experts, other channels); spare slabs and fresh rows carry the layer
    _case(32, 2048, 500, 128, 8, 0, 2, False, 3, 85, 0.0, 500)


def test_prefetch_slab_overflow_is_flagged_and_leaves_channels_out():
    # capacity below the list length: predicted lists are cut, misses beyond the slab are dropped and flagged
    ps = _case(33, 1024, 600, 64, 4, 0, 2, True, 1, 50, 0.9, 200)
    assert ps["misses"].sum() > 0
