"""A short stack of MoE layers whose gate/down matrices live in different places, decoded through the matching entry
points one after the other with everything they can share shared (workspace, staging buffer, streams, events): whole
layer resident in HBM, offloaded, offloaded with resident channels, offloaded with the next layer's channels staged
ahead.  Every layer's output is compared with the oracle on the same input, and the hidden state is carried from layer
to layer as in bench.py's stack workload."""
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


@pytest.mark.parametrize("d,f,T", [(1024, 1536, 1), (2048, 700, 3)])
def test_stack_of_resident_offloaded_cached_and_prefetched_layers(d, f, T):
    import gpu_common as G
    import paper_2505_05950_amd as F
    bits, group, n, top_k, pct = 2, 64, 4, 2, 85
    kinds = ["resident", "offloaded", "cached", "prefetched", "resident", "prefetched", "offloaded"]
    n_layers = len(kinds)
    wr = S.router_weights(81, 4, n, d)
    layers_np, layers = [], []
    tau0 = G.dev(np.zeros((T, n), np.float32))       # replaced per layer once its input is known
    for l in range(n_layers):
        experts = [G.make_expert(*S.expert_weights(81, 4, d, f, l, e), bits, group) for e in range(n)]
        layers_np.append([e[0] for e in experts])
        if kinds[l] == "resident":
            ex = [e[1] for e in experts]
            layers.append((F.Layer(ex, 0, top_k, True, G.dev(wr), tau0, True), None))
        else:
            pinned = [torch.from_numpy(e[0][3]).pin_memory() for e in experts]
            ex = [F.Expert(d, f, bits, group, e[1].up_codes, e[1].up_scale, e[1].up_zero, pinned[i]) for i, e in enumerate(experts)]
            layers.append((F.Layer(ex, 0, top_k, True, G.dev(wr), tau0, True, gd_on_host=True), pinned))
    slots, cap = top_k, f
    side, pre, miss = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
    ev_a, ev_b = torch.cuda.Event(), torch.cuda.Event()
    staging = torch.zeros((T * slots, cap, 2, d), dtype=torch.float16, device=G.DEV)
    M = F.MissPath(miss, T * slots, G.DEV)
    off_layer = next(L for (L, p), k in zip(layers, kinds) if k != "resident")
    P = [F.Prefetch(off_layer, T, cap, pre), F.Prefetch(off_layer, T, cap, pre)]
    ws = off_layer.workspace(T)                      # one workspace for every offloaded call
    ws_pre = off_layer.new_workspace(T)              # the prefetch runs beside a decode: a workspace of its own
    x = S.tokens(81, 4, T, d)
    n_pre = 0
    for l in range(n_layers):
        L, pinned = layers[l]
        ex_np = layers_np[l]
        # thresholds of this layer for this input, off the order statistic
        tau = np.zeros((T, n), np.float32)
        for t in range(T):
            for e in range(n):
                # in a gap between neighbouring |v|: no channel is close enough to its threshold for the rounding of the
                # kernels to decide it (the tight bar below has no room for a flipped channel)
                tau[t, e], margin = G.tau_in_widest_gap(O.up_gemv(*ex_np[e][:3], d, bits, group, x[t]), pct, window=8)
                assert margin > 1e-4 * tau[t, e]
        L.set_tau(G.dev(tau), True)
        ref = O.moe_layer(ex_np, 0, top_k, True, wr, x, tau, bits, group)
        xd = G.dev(x)
        stats = torch.zeros((T, slots, 4), dtype=torch.int32, device=G.DEV)
        print(f"layer {l}: {kinds[l]}", flush=True)
        if kinds[l] == "resident":
            y = F.floe_moe_layer_decode(L, xd, stats=stats)
        elif kinds[l] == "offloaded":
            y = F.floe_moe_layer_decode_offloaded(L, xd, staging, cap, side, ev_a, ev_b, stats=stats, workspace=ws)
        elif kinds[l] == "cached":
            res = [np.arange(e, f, 2, dtype=np.int32) for e in range(n)]      # every other channel resident
            cache = F.ChannelCache(L, T, sum(r.size for r in res), cap)
            first = 0
            for e in range(n):
                F.floe_channel_cache_load(L, cache, e, G.dev(res[e]), torch.tensor([res[e].size], dtype=torch.int32, device=G.DEV),
                                          first, res[e].size)
                first += res[e].size
            y = F.floe_moe_layer_decode_cached(L, cache, M, xd, stats=stats, workspace=ws)
        else:
            # predicted from a hidden state close to, but not equal to, the real input: some hits, some misses
            x_prev = (x.astype(np.float32) + 0.3 * S.tokens(82, 4, T, d, layer=l).astype(np.float32)).astype(np.float16)
            Pl = P[n_pre % 2]
            n_pre += 1
            F.floe_moe_layer_prefetch(L, Pl, G.dev(x_prev), ws_pre)
            pst = torch.zeros((T * slots, 4), dtype=torch.int32, device=G.DEV)
            y = F.floe_moe_layer_decode_prefetched(L, Pl, M, xd, stats=stats, prefetch_stats=pst, workspace=ws)
            torch.cuda.synchronize()
            ps = pst.cpu().numpy().view(F.PREFETCH_STAT_DTYPE).reshape(T, slots)
            assert ps["hits"].sum() > 0 and ps["misses"].sum() > 0
        torch.cuda.synchronize()
        yh = y.cpu().numpy()
        st = stats.cpu().numpy().reshape(T, slots, 4).copy().view(F.SLOT_STAT_DTYPE).reshape(T, slots)
        for t in range(T):
            assert [int(st[t, s_]["expert"]) for s_ in range(slots)] == [int(v) for v in ref["ids"][t]], (l, t)
            assert G.rel_err(yh[t].astype(np.float64), ref["y"][t]) <= G.Y_TIGHT, (l, kinds[l], t)
        assert M.overflow.cpu().numpy().sum() == 0
        # next hidden state, as in the stack benchmark
        yf = yh.astype(np.float32)
        x = (yf / yf.std(axis=1, keepdims=True)).astype(np.float16)
