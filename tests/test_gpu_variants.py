"""GPU parity of the three sparsification candidates of Sec. 3.2.1 (S_t on a_up, a_gate or a_down) through
floe_expert_ffn_sparsified against the oracle's literal evaluation of Eq. 1 with Eq. 5 in place."""
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


@pytest.mark.parametrize("d,f,bits,group,T,pct", [
    (1024, 3584, 2, 64, 1, 80),      # config-1 shape
    (4096, 1100, 2, 64, 3, 90),      # Mixtral width, ragged f, several tokens
    (2048, 1408, 3, 32, 2, 85),      # config-5 expert
    (512, 333, 4, 64, 2, 50),
    (1536, 200, 8, 64, 1, 0),        # nothing dropped: the dense expert of Eq. 1
])
@pytest.mark.parametrize("which", [O.SPARSIFY_UP, O.SPARSIFY_GATE, O.SPARSIFY_DOWN])
def test_sparsified_ffn_matches_the_oracle(which, d, f, bits, group, T, pct):
    import gpu_common as G
    import paper_2505_05950_amd as F
    w_up, gd = S.expert_weights(60, 2, d, f)
    ex_np, ex_dev = G.make_expert(w_up, gd, bits, group)
    x = S.tokens(60, 2, T, d)
    taus, refs = np.zeros(T, np.float32), []
    for t in range(T):
        a_up = O.up_gemv(*ex_np[:3], d, bits, group, x[t])
        _, _, act = O.sparsified_ffn(which, gd, x[t], a_up, -1.0)
        # a threshold in the widest gap near the order statistic of Eq. 6: nothing hinges on rounding order
        a = np.sort(np.abs(act))
        z = -(-f * pct // 100)
        if z == 0:
            taus[t] = -1.0
        else:
            lo, hi = max(1, z - 16), min(f - 1, z + 16)
            k = max(range(lo, hi + 1), key=lambda i: a[i] - a[i - 1])
            taus[t] = np.float32(0.5 * (a[k] + a[k - 1]))
        refs.append((a_up, act, O.sparsified_ffn(which, gd, x[t], a_up, float(taus[t]))))
    y = torch.zeros((T, d), dtype=torch.float32, device=G.DEV)
    y, idx, count = F.floe_expert_ffn_sparsified(ex_dev, which, G.dev(x), G.dev(taus), None, y)
    torch.cuda.synchronize()
    y = y.cpu().numpy().astype(np.float64)
    for t in range(T):
        a_up, act, (y_ref, idx_ref, _) = refs[t]
        got = idx[t, : int(count[t].item())].cpu().numpy()
        assert np.all(np.diff(got) > 0)
        # identical outside the relative band of 1e-3 around the threshold (here the gap keeps the band empty of
        # everything but rounding noise, so the lists are normally equal)
        band = np.abs(np.abs(act) - float(taus[t])) <= G.BAND * abs(float(taus[t]))
        sym = np.setxor1d(got, idx_ref)
        assert np.all(band[sym]), (t, sym[:8])
        if sym.size == 0:
            assert G.rel_err(y[t], y_ref) <= G.Y_TIGHT, (t, G.rel_err(y[t], y_ref))
        else:
            assert G.rel_err(y[t], y_ref) <= G.Y_BAR + 1e-2
