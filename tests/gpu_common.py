"""Helpers of the GPU parity tests: device upload, tolerances, band logic (no method arithmetic of
their own: every reference number comes from the oracle package)."""
import numpy as np
import torch

import oracle as O
import paper_2505_05950_amd as F

DEV = torch.device("cuda:0")

# Tolerances:
#  - v: the fp32 GEMV differs from the oracle's double sum by accumulation rounding only; the packed-fp16
#    fast path adds about 3e-5 absolute at rms(v) ~ 1.3.  Bar: 2.5e-4 * rms(v) absolute.
#  - index sets: exact outside the relative band |(|v| - tau)| <= 1e-3 * tau (the stated target).
#  - y: max_i |y - y_ref| / max_i |y_ref| <= 1e-2 (the stated target); channels inside the band may go either
#    way, their largest possible contribution is added to the allowance explicitly.
V_RTOL_RMS = 2.5e-4
BAND = 1e-3
Y_BAR = 1e-2
Y_TIGHT = 2e-3


def dev(a: np.ndarray) -> torch.Tensor:
    if a.dtype == np.uint32:
        a = a.view(np.int32)
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def host_u32(t: torch.Tensor) -> np.ndarray:
    return t.cpu().numpy().view(np.uint32)


def make_expert(w_up, gd, bits, group):
    """Quantize on both sides; returns (oracle tuple, device Expert) after checking bit equality."""
    f, d = w_up.shape
    codes, scale, zero = O.quantize(w_up, bits, group)
    gc, gs, gz = F.floe_quantize_expert(dev(w_up), bits, group)
    torch.cuda.synchronize()
    assert np.array_equal(host_u32(gc), codes), "packed codes differ"
    assert np.array_equal(gs.cpu().numpy().view(np.uint16), scale.view(np.uint16)), "scales differ"
    assert np.array_equal(gz.cpu().numpy().view(np.uint16), zero.view(np.uint16)), "zeros differ"
    return (codes, scale, zero, gd), F.Expert(d, f, bits, group, gc, gs, gz, dev(gd))


def in_band(v_ref: np.ndarray, tau: float) -> np.ndarray:
    return np.abs(np.abs(v_ref) - np.float32(tau)) <= BAND * abs(tau)


def check_index_set(idx_gpu: np.ndarray, v_ref: np.ndarray, tau: float):
    """GPU list must be ascending, duplicate-free and equal to the oracle's outside the band."""
    assert np.all(np.diff(idx_gpu) > 0), "index list not strictly ascending"
    ref = O.select(v_ref, tau)
    band = in_band(v_ref, tau)
    sym = np.setxor1d(idx_gpu, ref)
    assert np.all(band[sym]), f"selection differs outside the band at channels {sym[~band[sym]][:8]}"
    return ref, sym


def rel_err(y, y_ref):
    return float(np.abs(y - y_ref).max() / np.abs(y_ref).max())


def tau_in_widest_gap(v, pct, window=64):
    """A threshold for about pct % sparsity that no channel sits close to: the middle of the widest gap between
    neighbouring |v| within `window` ranks of the order statistic of Eq. 6.  Returns (tau, distance to the nearest |v|)."""
    a = np.sort(np.abs(v.astype(np.float64)))
    z = -(-v.size * pct // 100)
    lo, hi = max(1, z - window), min(v.size - 1, z + window)
    k = max(range(lo, hi + 1), key=lambda i: a[i] - a[i - 1])
    tau = np.float32(0.5 * (a[k] + a[k - 1]))
    return tau, float(min(float(tau) - a[k - 1], a[k] - float(tau)))
