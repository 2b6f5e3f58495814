"""Pins for the oracle's fp16 conversions, quantizer, packing and dequant-GEMV (CPU only)."""
import numpy as np
import pytest

import floe_synth as S
import oracle as O


# ---------------------------------------------------------------- fp16 conversions
def test_half_to_float_all_patterns_match_numpy():
    bits = np.arange(65536, dtype=np.uint16)
    ref = bits.view(np.float16).astype(np.float32)
    got = np.array([O.half_to_float(int(b)) for b in bits], dtype=np.float32)
    finite = np.isfinite(ref)
    assert np.array_equal(got[finite], ref[finite])
    assert np.array_equal(np.isnan(got), np.isnan(ref))
    assert np.array_equal(np.isinf(got), np.isinf(ref))


def test_narrowing_is_round_to_nearest_even():
    rng = np.random.default_rng(5)
    xs = np.concatenate([
        rng.normal(0, 1, 4000), rng.normal(0, 1e-5, 2000), rng.normal(0, 3e4, 2000),
        # exact ties between neighbouring fp16 values, subnormal ties, overflow boundary
        np.array([1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, 2.0 ** -25, 3 * 2.0 ** -25, 65519.99, 65520.0, -65520.0,
                  0.0, -0.0, 2.0 ** -24, 2.0 ** -14 - 2.0 ** -25, 6.1e-5]),
    ])
    for x in xs:
        ref = int(np.float64(x).astype(np.float16).view(np.uint16))
        assert O.double_to_half(float(x)) == ref, x
        xf = np.float32(x)
        assert O.float_to_half(float(xf)) == int(xf.astype(np.float16).view(np.uint16)), x


# ---------------------------------------------------------------- quantizer: hand-enumerated cases
def _pack_bigint(levels, bits):
    """Definition of a little-endian bit stream, on Python integers: code i at bits [bits*i, bits*i+bits)."""
    big = 0
    for i, q in enumerate(levels):
        big |= int(q) << (bits * i)
    nwords = (len(levels) * bits + 31) // 32
    return [(big >> (32 * w)) & 0xFFFFFFFF for w in range(nwords)]


def test_hand_enumerated_group_int2():
    # one channel, one group of 16: min -0.75, max 1.5 -> scale 0.75, zero 1.0 (all exact in fp16)
    w = np.array([-0.75, 1.5, 0.0, 0.75, -0.375, 0.375, 1.125, -0.74, 1.49, 0.3, -0.75, 1.5, 0.0, 0.0, 0.75, 0.75],
                 dtype=np.float16).reshape(1, 16)
    # w/0.75 + 1 = 0, 3, 1, 2, 0.5 (tie -> 0), 1.5 (tie -> 2), 2.5 (tie -> 2), 0.013 -> 0, 2.99 -> 3, 1.4 -> 1, ...
    expect = [0, 3, 1, 2, 0, 2, 2, 0, 3, 1, 0, 3, 1, 1, 2, 2]
    codes, scale, zero = O.quantize(w, 2, 16)
    assert scale[0, 0] == np.float16(0.75) and zero[0, 0] == np.float16(1.0)
    assert codes.shape == (1, 1)
    assert [int(codes[0, 0] >> (2 * i)) & 3 for i in range(16)] == expect
    assert codes[0, 0] == _pack_bigint(expect, 2)[0]
    w_hat = O.dequantize(codes, scale, zero, 16, 2, 16)
    assert np.array_equal(w_hat[0], (np.array(expect, np.float32) - 1.0) * 0.75)


def test_degenerate_group_is_exact():
    w = np.full((2, 32), 0.0123, dtype=np.float16)
    w[1, :] = 0.0
    codes, scale, zero = O.quantize(w, 4, 8)
    assert np.all(codes == 0) and np.all(scale == np.float16(1.0))
    assert np.array_equal(O.dequantize(codes, scale, zero, 32, 4, 8), w.astype(np.float32))


def test_group_whose_step_is_below_the_smallest_normal_half_is_degenerate():
    """Second degenerate branch of the quantizer (Sec. 3.2.2 reading: a group whose step (max - min) / qmax falls
    below 2^-14, the smallest normal binary16, is stored as scale 1, zero = fp16(-min), codes 0).  Expected values
    written out by hand; the boundary step 2^-14 itself is still an ordinary group."""
    # INT2 (qmax 3), group 16: min = -0.25, max = -0.25 + 2^-13 (its fp16 neighbour): step 2^-13 / 3 = 4.07e-5 < 6.10e-5
    w = np.full((3, 16), -0.25, dtype=np.float16)
    w[0, 5] = np.float16(-0.25 + 2.0 ** -13)
    assert float(w[0, 5]) == -0.2498779296875          # exactly representable, so max != min
    # row 1, the boundary: values 0 and 3 * 2^-14: step exactly 2^-14 -> scale 0x0400, zero -0.0, codes 0, 2 and 3
    w[1, :] = 0.0
    w[1, 2] = np.float16(3 * 2.0 ** -14)
    w[1, 9] = np.float16(2 * 2.0 ** -14)
    # row 2, INT2 again: 0 and 2^-15 (a subnormal half): step 2^-15 / 3, far below -> degenerate with zero = -0.0
    w[2, :] = 0.0
    w[2, 0] = np.float16(2.0 ** -15)
    codes, scale, zero = O.quantize(w, 2, 16)
    sc, zr = scale.view(np.uint16), zero.view(np.uint16)
    assert sc[0, 0] == 0x3C00 and zr[0, 0] == 0x3400 and codes[0, 0] == 0          # scale 1, zero +0.25, codes 0
    assert sc[1, 0] == 0x0400 and zr[1, 0] == 0x8000                              # 2^-14; zero = (-0) / scale = -0.0
    assert int(codes[1, 0]) == (3 << (2 * 2)) | (2 << (2 * 9))                     # code 3 at i = 2, code 2 at i = 9
    assert sc[2, 0] == 0x3C00 and zr[2, 0] == 0x8000 and codes[2, 0] == 0          # scale 1, zero -0.0, codes 0
    w_hat = O.dequantize(codes, scale, zero, 16, 2, 16)
    assert np.all(w_hat[0] == np.float32(-0.25))                                  # the whole group collapses onto min
    assert np.array_equal(w_hat[1], w[1].astype(np.float32))
    assert np.all(w_hat[2] == 0.0)
    # INT4 (qmax 15): 0 and 15 * 2^-15 -> step 2^-15 (subnormal) -> degenerate; 0 and 15 * 2^-14 -> ordinary, codes 0 / 15
    w4 = np.zeros((2, 8), dtype=np.float16)
    w4[0, 3] = np.float16(15 * 2.0 ** -15)
    w4[1, 3] = np.float16(15 * 2.0 ** -14)
    c4, s4, z4 = O.quantize(w4, 4, 8)
    assert s4.view(np.uint16)[0, 0] == 0x3C00 and c4[0, 0] == 0
    assert s4.view(np.uint16)[1, 0] == 0x0400 and int(c4[1, 0]) == 15 << (4 * 3)


@pytest.mark.parametrize("bits,group", [(2, 16), (2, 64), (3, 32), (3, 64), (4, 8), (4, 64), (1, 32), (1, 64), (8, 4), (8, 64)])
def test_packing_is_little_endian_bitstream(bits, group):
    # weights that sit exactly on the quantization grid: level * 0.5 with both end levels present in
    # every group, so scale = 0.5, zero = 0 and code == level by construction
    qmax = (1 << bits) - 1
    d, f = 4 * group, 3
    rng = np.random.default_rng(bits * 100 + group)
    levels = rng.integers(0, qmax + 1, size=(f, d))
    levels[:, 0::group] = 0
    levels[:, 1::group] = qmax
    w = (levels * 0.5).astype(np.float16)
    codes, scale, zero = O.quantize(w, bits, group)
    assert np.all(scale == np.float16(0.5)) and np.all(zero == 0)
    assert codes.shape == (f, d * bits // 32)
    for j in range(f):
        assert [int(c) for c in codes[j]] == _pack_bigint(levels[j], bits)
    assert np.array_equal(O.dequantize(codes, scale, zero, d, bits, group), w.astype(np.float32))


# ---------------------------------------------------------------- quantizer: properties on workload-like data
@pytest.mark.parametrize("bits,group", [(2, 64), (3, 32), (4, 64), (1, 64), (8, 64)])
def test_roundtrip_bound_and_end_codes(bits, group):
    d, f = 512, 96
    w = S.normal_f16(S.stream_key(3, 99, S.KIND_W_UP, 0, bits), (f, d), S.W_SIGMA)
    codes, scale, zero = O.quantize(w, bits, group)
    w_hat = O.dequantize(codes, scale, zero, d, bits, group)
    s = np.repeat(scale.astype(np.float32), group, axis=1)
    err = np.abs(w_hat - w.astype(np.float32))
    assert np.all(err <= 0.51 * s), float((err / s).max())
    # the error is a genuine rounding error: some elements must come close to half a step
    assert (err / s).max() > 0.45
    # unpack with the big-int definition and check that each group's minimum sits on code 0 and maximum on qmax
    qmax = (1 << bits) - 1
    for j in range(0, f, 7):
        big = 0
        for wd, c in enumerate(codes[j]):
            big |= int(c) << (32 * wd)
        q = np.array([(big >> (bits * i)) & qmax for i in range(d)])
        wj = w[j].astype(np.float32).reshape(-1, group)
        qg = q.reshape(-1, group)
        rows = np.arange(wj.shape[0])
        assert np.all(qg[rows, wj.argmin(axis=1)] == 0)
        assert np.all(qg[rows, wj.argmax(axis=1)] == qmax)
        assert q.min() >= 0 and q.max() <= qmax


def test_codes_match_vectorised_float32_restatement():
    # cross-check (not a pin on its own): the same quantizer written with numpy float32 array ops
    bits, group, d, f = 2, 64, 1024, 64
    w = S.normal_f16(S.stream_key(4, 99, S.KIND_W_UP), (f, d), S.W_SIGMA)
    codes, scale, zero = O.quantize(w, bits, group)
    wf = w.astype(np.float32).reshape(f, d // group, group)
    mn, mx = wf.min(axis=2), wf.max(axis=2)
    sh = ((mx - mn) / np.float32(3)).astype(np.float16)
    Sf = sh.astype(np.float32)
    zh = ((-mn) / Sf).astype(np.float16)
    q = np.clip(np.rint(wf / Sf[..., None] + zh.astype(np.float32)[..., None]), 0, 3).astype(np.uint32)
    assert np.array_equal(sh, scale) and np.array_equal(zh, zero)
    q = q.reshape(f, d // 16, 16)
    words = np.zeros((f, d // 16), dtype=np.uint32)
    for m in range(16):
        words |= q[:, :, m] << np.uint32(2 * m)
    assert np.array_equal(words, codes)


def test_compression_arithmetic():
    from helpers import golden_values
    g = golden_values("lemma_gaussian_threshold.txt")
    d, f, b, grp = 4096, 14336, 2, 64
    codes_bytes = f * O.words_per_channel(d, b) * 4
    meta_bytes = 2 * 2 * f * (d // grp)
    assert codes_bytes == d * f * b // 8
    assert (codes_bytes + meta_bytes) * 8 / (d * f) == 2.5            # bits per weight incl. fp16 scale+zero
    ratio = 48.0 / (b + 2 * 16 * 0.1)                                  # metadata ignored, 10 % of gate+down kept
    val, tol = g["compression_ratio"]
    assert abs(ratio - val) <= tol
    val, _ = g["chunk_bytes_d4096"]
    assert 2 * d * 2 == val


# ---------------------------------------------------------------- dequant GEMV
@pytest.mark.parametrize("bits,group", [(2, 64), (3, 32), (4, 64), (1, 128), (8, 32)])
def test_up_gemv_is_plain_matvec_on_dequantized_matrix(bits, group):
    d, f = 768, 40
    w = S.normal_f16(S.stream_key(6, 99, S.KIND_W_UP, 0, bits), (f, d), S.W_SIGMA)
    x = S.normal_f16(S.stream_key(6, 99, S.KIND_X, 0, bits), (d,), 1.0)
    codes, scale, zero = O.quantize(w, bits, group)
    w_hat = O.dequantize(codes, scale, zero, d, bits, group)
    ref = w_hat.astype(np.float64) @ x.astype(np.float64)             # library mat-vec
    v = O.up_gemv(codes, scale, zero, d, bits, group, x)
    assert v.dtype == np.float32
    np.testing.assert_allclose(v, ref.astype(np.float32), rtol=0, atol=1e-6)
    # distance from the unquantized projection obeys the per-element round-trip bound
    exact = w.astype(np.float64) @ x.astype(np.float64)
    s = np.repeat(scale.astype(np.float64), group, axis=1)
    bound = (0.51 * s * np.abs(x.astype(np.float64))[None, :]).sum(axis=1)
    assert np.all(np.abs(v - exact) <= bound)


def test_up_gemv_variance_follows_gaussian_matrix_lemma():
    # App. A, lemma on E||xW||^2 = n sigma^2 E||x||^2: per channel E[v_j^2] = sigma_W^2 ||x||^2.
    # INT4 adds only step^2/12 of quantization noise per weight (about 1 % here).
    d, f, bits, group = 1024, 2048, 4, 64
    w = S.normal_f16(S.stream_key(7, 99, S.KIND_W_UP), (f, d), S.W_SIGMA)
    x = S.normal_f16(S.stream_key(7, 99, S.KIND_X), (d,), 1.0)
    codes, scale, zero = O.quantize(w, bits, group)
    v = O.up_gemv(codes, scale, zero, d, bits, group, x).astype(np.float64)
    expect = S.W_SIGMA ** 2 * float((x.astype(np.float64) ** 2).sum())
    assert abs((v ** 2).mean() / expect - 1.0) < 0.08                 # 2048 samples: ~3 % sampling error
