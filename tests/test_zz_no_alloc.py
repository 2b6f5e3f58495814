"""The entry point that allocates nothing (floe_moe_layer_decode_static) against floe_moe_layer_decode: same kernels,
same fixed summation order, so the outputs must be equal bit for bit; two calls in a row share the library's scratch
array, the second with a smaller input; a layer whose workspace exceeds the array is refused."""
import numpy as np
import pytest
import torch

import floe_synth as S

pytestmark = pytest.mark.gpu


def _layer(F, G, seed, d, f, bits, group, n, top_k):
    experts = [G.make_expert(*S.expert_weights(seed, 3, d, f, 0, e), bits, group)[1] for e in range(n)]
    wr = G.dev(S.router_weights(seed, 3, n, d))
    tau = G.dev(np.full((n,), 1.1, np.float32))
    return F.Layer(experts, 0, top_k, True, wr, tau, False)


def test_static_scratch_entry_point_matches_the_workspace_entry_point():
    import gpu_common as G
    import paper_2505_05950_amd as F
    big = _layer(F, G, 31, 4096, 1792, 2, 64, 8, 2)       # fused kernel, routed in place, several blocks per task
    small = _layer(F, G, 32, 1024, 700, 4, 32, 5, 2)      # router kernel + fused INT4, ragged f
    calls = [(big, 3, 40), (small, 2, 41), (big, 1, 42), (small, 9, 43)]   # second call smaller than the first; T=9: GEMV + gate/down kernels
    for L, T, _ in calls:
        assert F.floe_layer_workspace_bytes(L, T) <= F.STATIC_SCRATCH_BYTES
    xs = [G.dev(S.tokens(seed, 3, T, L.d)) for L, T, seed in calls]
    ref = []
    for (L, T, _), x in zip(calls, xs):
        st = torch.zeros((T, 2, 4), dtype=torch.int32, device=G.DEV)
        ref.append((F.floe_moe_layer_decode(L, x, stats=st).clone(), st.clone()))
    torch.cuda.synchronize()
    # outputs pre-allocated; nothing between the calls but the calls themselves
    outs = [(torch.zeros((T, L.d), dtype=torch.float16, device=G.DEV), torch.zeros((T, 2, 4), dtype=torch.int32, device=G.DEV))
            for L, T, _ in calls]
    torch.cuda.synchronize()
    for (L, T, _), x, (y, st) in zip(calls, xs, outs):
        F.floe_moe_layer_decode_static(L, x, y, st)
    torch.cuda.synchronize()
    for i, ((y_ref, st_ref), (y, st)) in enumerate(zip(ref, outs)):
        assert torch.equal(y, y_ref), f"call {i}: output differs from floe_moe_layer_decode"
        assert torch.equal(st, st_ref), f"call {i}: statistics differ"
    # and against the oracle's bar through the shared checker: y_ref itself is covered by the layer parity tests


def test_static_scratch_entry_point_refuses_what_does_not_fit():
    import gpu_common as G
    import paper_2505_05950_amd as F
    L = _layer(F, G, 33, 4096, 1792, 2, 64, 8, 2)
    T = 1
    while F.floe_layer_workspace_bytes(L, T) <= F.STATIC_SCRATCH_BYTES:
        T *= 2
    x = G.dev(S.tokens(33, 3, T, 4096))
    y = torch.full((T, 4096), 7.0, dtype=torch.float16, device=G.DEV)
    with pytest.raises(F.FloeError) as err:
        F.floe_moe_layer_decode_static(L, x, y)
    assert err.value.status == -4
    torch.cuda.synchronize()
    assert bool((y == 7.0).all()), "a refused call must not touch the output"
