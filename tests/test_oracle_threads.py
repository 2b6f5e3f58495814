"""The oracle's worker threads only split independent outer loops: results must not depend on their number."""
import numpy as np

import floe_synth as S
import oracle as O


def test_results_do_not_depend_on_thread_count():
    d, f, bits, group = 512, 300, 3, 32
    w_up, gd = S.expert_weights(40, 90, d, f)
    x = S.tokens(40, 90, 1, d)[0]
    out = []
    for n in (1, 5):
        O.set_threads(n)
        assert O.get_threads() == n
        c, s, z = O.quantize(w_up, bits, group)
        v = O.up_gemv(c, s, z, d, bits, group, x)
        idx = O.select(v, O.threshold_for_sparsity(v, 60))
        h, y = O.sparse_ffn(gd, x, v, idx)
        out.append((c, s, z, v, idx, h, y, O.dense_ffn(O.dequantize(c, s, z, d, bits, group), gd, x)))
    O.set_threads(1)
    for a, b in zip(*out):
        assert np.array_equal(a, b)
