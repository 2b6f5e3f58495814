"""GPU parity, step by step (S0, S2, S3, S4+S5, S7) through the C ABI against the CPU oracle."""
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


def _gc():
    import gpu_common as G
    return G


# ------------------------------------------------------------------------------------------- S0
@pytest.mark.parametrize("bits,group,d,f", [
    (2, 64, 1024, 257), (2, 64, 4096, 96), (2, 128, 2048, 33), (2, 32, 512, 64), (2, 256, 1536, 17),
    (3, 32, 2048, 65), (3, 64, 4096, 40), (3, 128, 1024, 9),
    (4, 32, 512, 31), (4, 64, 4096, 48), (4, 256, 2560, 12), (2, 64, 8192, 8),
    (1, 64, 4096, 40), (1, 32, 1024, 33), (8, 64, 4096, 24), (8, 128, 1536, 19),   # the other widths of the sensitivity study
])
def test_quantize_bit_exact(bits, group, d, f):
    G = _gc()
    import paper_2505_05950_amd as F
    w = S.normal_f16(S.stream_key(0, 50, S.KIND_W_UP, bits, group, d), (f, d), S.W_SIGMA)
    # plant special groups: constant, all-zero, tiny range (scale underflows fp16 normals), exact half-way codes
    w[0, :group] = np.float16(0.0123)
    w[1 % f, :group] = 0
    w[2 % f, :group] = np.float16(0.01)
    w[2 % f, 0] = np.nextafter(np.float16(0.01), np.float16(1.0))
    lv = np.array([0, 1, 2, 3, 0.5, 1.5, 2.5, 3][: 8], dtype=np.float32) * 0.75 - 0.75
    w[3 % f, :group] = np.resize(lv, group).astype(np.float16)
    codes, scale, zero = O.quantize(w, bits, group)
    gcodes, gscale, gzero = F.floe_quantize_expert(G.dev(w), bits, group)
    torch.cuda.synchronize()
    assert np.array_equal(G.host_u32(gcodes), codes)
    assert np.array_equal(gscale.cpu().numpy().view(np.uint16), scale.view(np.uint16))
    assert np.array_equal(gzero.cpu().numpy().view(np.uint16), zero.view(np.uint16))


def test_quantize_config1_shape_bit_exact():
    G = _gc()
    w, gd = S.expert_weights(0, 1, 1024, 3584)
    G.make_expert(w, gd, 2, 64)


# ------------------------------------------------------------------------------------------- S2
@pytest.mark.parametrize("bits,group,d,f,T", [
    (2, 64, 1024, 3584, 1),     # config 1 shape, packed-fp16 fast path (16 lanes per channel)
    (2, 64, 4096, 1000, 3),     # fast path, ragged f (not a multiple of the 32 channels per workgroup)
    (2, 128, 2048, 515, 2),     # fast path with a group that spans two lanes
    (2, 32, 1024, 130, 1),      # packed path, two (scale, zero) pairs per 64-code unit
    (2, 64, 1536, 77, 2),       # generic path (d not a power of two)
    (3, 32, 2048, 1408, 2),     # config 5 shape: packed INT3 (96-bit half units), group 32
    (3, 64, 4096, 300, 1),      # packed INT3
    (3, 128, 1024, 70, 3),
    (4, 64, 4096, 300, 1),      # packed INT4
    (4, 128, 2048, 99, 2),
    (4, 32, 1024, 65, 2),
    (4, 32, 512, 64, 5),        # generic path (d = 512)
    (3, 64, 2560, 41, 1),       # generic path
    (1, 64, 4096, 130, 2),      # INT1 and INT8 run the generic kernels
    (1, 32, 1024, 70, 1),
    (8, 64, 4096, 99, 1),
    (8, 128, 2048, 65, 3),
])
def test_up_gemv_matches_oracle(bits, group, d, f, T):
    G = _gc()
    import paper_2505_05950_amd as F
    w = S.normal_f16(S.stream_key(1, 51, S.KIND_W_UP, bits, group, d), (f, d), S.W_SIGMA)
    x = S.tokens(1, 51, T, d)
    codes, scale, zero = O.quantize(w, bits, group)
    v = F.floe_up_gemv(G.dev(codes), G.dev(scale), G.dev(zero), G.dev(x), d, bits, group)
    torch.cuda.synchronize()
    v = v.cpu().numpy()
    for t in range(T):
        ref = O.up_gemv(codes, scale, zero, d, bits, group, x[t])
        rms = float(np.sqrt((ref.astype(np.float64) ** 2).mean()))
        err = float(np.abs(v[t] - ref).max())
        assert err <= G.V_RTOL_RMS * rms, (err, rms)


def test_up_gemv_large_activations_do_not_overflow_the_packed_path():
    G = _gc()
    import paper_2505_05950_amd as F
    d, f, bits, group = 4096, 200, 2, 64
    w = S.normal_f16(S.stream_key(2, 51, S.KIND_W_UP), (f, d), S.W_SIGMA)
    x = (S.tokens(2, 51, 2, d).astype(np.float32) * np.array([[900.0], [30000.0]], np.float32))
    x = np.clip(x, -65000, 65000).astype(np.float16)
    codes, scale, zero = O.quantize(w, bits, group)
    v = F.floe_up_gemv(G.dev(codes), G.dev(scale), G.dev(zero), G.dev(x), d, bits, group).cpu().numpy()
    for t in range(2):
        ref = O.up_gemv(codes, scale, zero, d, bits, group, x[t])
        rms = float(np.sqrt((ref.astype(np.float64) ** 2).mean()))
        assert np.all(np.isfinite(v[t]))
        assert float(np.abs(v[t] - ref).max()) <= 2e-3 * rms   # x' = x * 2^-k may drop low bits of small elements


# ------------------------------------------------------------------------------------------- S3
@pytest.mark.parametrize("f,T", [(1, 1), (63, 2), (64, 1), (1000, 3), (3584, 2), (14336, 4), (70001, 1)])
def test_select_is_bit_exact_on_identical_v(f, T):
    G = _gc()
    import paper_2505_05950_amd as F
    v = S.normal(S.stream_key(3, 52, S.KIND_MISC, f), T * f, 1.28).astype(np.float32).reshape(T, f)
    pcts = [90, 0, 100, 50]
    tau = np.array([O.threshold_for_sparsity(v[t], pcts[t % 4]) for t in range(T)], np.float32)
    if T > 1:
        tau[1] = -1.0                      # keep everything
    idx, count = F.floe_select_channels(G.dev(v), G.dev(tau))
    torch.cuda.synchronize()
    idx, count = idx.cpu().numpy(), count.cpu().numpy()
    for t in range(T):
        ref = O.select(v[t], float(tau[t]))
        assert count[t] == ref.size
        assert np.array_equal(idx[t, : ref.size], ref)
        assert np.all(idx[t, ref.size:] == -1)          # entries past the count are untouched


def test_select_ties_are_strict():
    G = _gc()
    import paper_2505_05950_amd as F
    v = np.array([[0.5, -0.5, 0.25, -0.75, 0.5000001, 0.0, np.nan, np.inf]], np.float32)
    idx, count = F.floe_select_channels(G.dev(v), G.dev(np.array([0.5], np.float32)))
    assert count.item() == 3 and idx[0, :3].tolist() == [3, 4, 7]
    assert list(O.select(v[0], 0.5)) == [3, 4, 7]


# ------------------------------------------------------------------------------------------- S4+S5 and Alg. 1
def _expert_case(seed, cfg, d, f, bits, group, T):
    G = _gc()
    w_up, gd = S.expert_weights(seed, cfg, d, f)
    x = S.tokens(seed, cfg, T, d)
    ex_np, ex_dev = G.make_expert(w_up, gd, bits, group)
    return ex_np, ex_dev, x


@pytest.mark.parametrize("d,f,bits,group,T,pct", [
    (1024, 3584, 2, 64, 1, 80),     # config 1
    (1024, 700, 2, 64, 3, 50),
    (2048, 1408, 3, 32, 2, 85),     # config 5 expert
    (1536, 300, 4, 64, 2, 90),      # d = 3 * 512
    (512, 64, 2, 32, 1, 0),
    (4096, 1024, 2, 64, 2, 90),
])
def test_gate_down_on_oracle_lists(d, f, bits, group, T, pct):
    """S4+S5 alone: same v and same index list on both sides, so no band is involved."""
    G = _gc()
    import paper_2505_05950_amd as F
    ex_np, ex_dev, x = _expert_case(4, 53, d, f, bits, group, T)
    v = np.stack([O.up_gemv(*ex_np[:3], d, bits, group, x[t]) for t in range(T)])
    idx = np.full((T, f), -1, np.int32)
    count = np.zeros(T, np.int32)
    refs = []
    scale = np.linspace(0.5, 1.5, T).astype(np.float32)
    for t in range(T):
        tau = O.threshold_for_sparsity(v[t], pct)
        sel = O.select(v[t], tau)
        idx[t, : sel.size] = sel
        count[t] = sel.size
        refs.append(O.sparse_ffn(ex_np[3], x[t], v[t], sel)[1] * float(scale[t]))
    y0 = S.normal(S.stream_key(4, 53, S.KIND_MISC, d), T * d, 0.1).astype(np.float32).reshape(T, d)
    y = G.dev(y0.copy())
    F.floe_gate_down_sparse(ex_dev, G.dev(x), G.dev(v), G.dev(idx), G.dev(count), G.dev(scale), y)
    torch.cuda.synchronize()
    y = y.cpu().numpy().astype(np.float64) - y0          # the call accumulates into y_acc
    for t in range(T):
        if count[t] == 0:
            assert np.abs(y[t]).max() < 1e-6
        else:
            assert G.rel_err(y[t], refs[t]) <= 2e-4, G.rel_err(y[t], refs[t])


@pytest.mark.parametrize("d,f,bits,group,T,pcts", [
    (1024, 3584, 2, 64, 1, [80]),                   # config 1
    (1024, 3584, 2, 64, 4, [80, 0, 100, 50]),       # dense, empty and half lists in one call
    (2048, 1408, 3, 32, 3, [85, 85, 60]),           # config 5 expert
    (1536, 515, 4, 64, 2, [90, 70]),
    (4096, 2000, 2, 128, 2, [90, 80]),
    (2048, 600, 1, 64, 2, [80, 50]),                # INT1 and INT8 (generic kernels)
    (1024, 900, 8, 32, 2, [90, 70]),
])
def test_expert_ffn_sparse_matches_oracle(d, f, bits, group, T, pcts):
    G = _gc()
    import paper_2505_05950_amd as F
    ex_np, ex_dev, x = _expert_case(5, 54, d, f, bits, group, T)
    v_ref = [O.up_gemv(*ex_np[:3], d, bits, group, x[t]) for t in range(T)]
    tau = np.array([O.threshold_for_sparsity(v_ref[t], pcts[t]) for t in range(T)], np.float32)
    y = torch.zeros((T, d), dtype=torch.float32, device=G.DEV)
    y, idx, count = F.floe_expert_ffn_sparse(ex_dev, G.dev(x), G.dev(tau), None, y)
    torch.cuda.synchronize()
    y, idx, count = y.cpu().numpy().astype(np.float64), idx.cpu().numpy(), count.cpu().numpy()
    for t in range(T):
        got = idx[t, : count[t]]
        ref_idx, sym = G.check_index_set(got, v_ref[t], float(tau[t]))
        if pcts[t] == 100:
            assert count[t] <= sym.size
        # reference on the GPU's own list (identical outside the band): tight bar
        y_same = O.sparse_ffn(ex_np[3], x[t], v_ref[t], got)[1]
        if got.size:
            assert G.rel_err(y[t], y_same) <= G.Y_TIGHT
        # reference on the oracle's list: the spec bar, plus what in-band channels can contribute
        y_ref = O.sparse_ffn(ex_np[3], x[t], v_ref[t], ref_idx)[1]
        if ref_idx.size:
            h_sym = O.sparse_ffn(ex_np[3], x[t], v_ref[t], sym)[0] if sym.size else np.zeros(0)
            slack = (np.abs(h_sym)[:, None] * np.abs(ex_np[3][sym, 1, :].astype(np.float64))).sum(axis=0) if sym.size else 0.0
            assert np.all(np.abs(y[t] - y_ref) <= G.Y_BAR * np.abs(y_ref).max() + slack)


def test_expert_ffn_randomized_shapes():
    """Seeded sweep of the one-expert entry point over shapes, widths, batch sizes and sparsity levels."""
    import random
    rng = random.Random(505950)
    for i in range(16):
        d = rng.choice([1024, 2048, 4096, 1536])
        bits = rng.choice([2, 2, 3, 4])
        group = rng.choice([32, 64, 128])
        f = rng.randint(120, 1500) if d >= 2048 else rng.randint(120, 3000)
        T = rng.choice([1, 1, 2, 4, 7, 16, 20])
        pcts = [rng.choice([0, 50, 80, 90, 95]) for _ in range(T)]
        print(f"case {i}: d={d} f={f} bits={bits} group={group} T={T} pcts={pcts}", flush=True)
        test_expert_ffn_sparse_matches_oracle(d, f, bits, group, T, pcts)


@pytest.mark.parametrize("d,f,bits,group,T", [(4096, 530, 2, 64, 3), (2048, 1000, 3, 32, 2), (1024, 300, 4, 128, 17),
                                              (512, 400, 2, 64, 2)])
def test_expert_ffn_without_a_list_gives_the_same_result(d, f, bits, group, T):
    """idx = count = NULL: the same y, whether the list is skipped (small batches of packed shapes) or built in the workspace."""
    G = _gc()
    import paper_2505_05950_amd as F
    ex_np, ex_dev, x = _expert_case(12, 57, d, f, bits, group, T)
    v_ref = [O.up_gemv(*ex_np[:3], d, bits, group, x[t]) for t in range(T)]
    tau = np.array([O.threshold_for_sparsity(v_ref[t], 80) * 1.002 for t in range(T)], np.float32)
    scale = G.dev(np.linspace(0.5, 1.5, T).astype(np.float32))
    y1 = torch.zeros((T, d), dtype=torch.float32, device=G.DEV)
    y2 = torch.zeros((T, d), dtype=torch.float32, device=G.DEV)
    y1, idx, count = F.floe_expert_ffn_sparse(ex_dev, G.dev(x), G.dev(tau), scale, y1)
    y2, none_idx, none_count = F.floe_expert_ffn_sparse(ex_dev, G.dev(x), G.dev(tau), scale, y2, want_list=False)
    torch.cuda.synchronize()
    assert none_idx is None and none_count is None
    assert torch.equal(y1, y2)
    y1, idx, count = y1.cpu().numpy().astype(np.float64), idx.cpu().numpy(), count.cpu().numpy()
    for t in range(T):
        got = idx[t, : count[t]]
        G.check_index_set(got, v_ref[t], float(tau[t]))
        w = 0.5 + t / max(T - 1, 1)
        assert G.rel_err(y1[t], w * O.sparse_ffn(ex_np[3], x[t], v_ref[t], got)[1]) <= G.Y_TIGHT


@pytest.mark.parametrize("f,T,want_list", [(448, 1, False), (448, 2, True), (450, 1, False), (2240, 1, False)])
def test_expert_ffn_with_every_channel_selected_meets_the_tight_bar(f, T, want_list):
    """tau < 0 selects every channel: every queue of the fused kernel runs full, so a consumer leaves its loop because
    the queue is exhausted, not because it saw its producer's flag.  The INT2 producer's staging ring lies in the slabs
    that the consumers store their results in, so a consumer has to wait for the flag before that store.  d = 4096,
    INT2, whole blocks of 112 channels (and one ragged), dense result compared with the oracle at the tight bar."""
    G = _gc()
    import paper_2505_05950_amd as F
    d, bits, group = 4096, 2, 64
    ex_np, ex_dev, x = _expert_case(31, 58, d, f, bits, group, T)
    tau = np.full((T,), -1.0, np.float32)
    y = torch.zeros((T, d), dtype=torch.float32, device=G.DEV)
    y, idx, count = F.floe_expert_ffn_sparse(ex_dev, G.dev(x), G.dev(tau), None, y, want_list=want_list)
    torch.cuda.synchronize()
    y = y.cpu().numpy().astype(np.float64)
    every = np.arange(f, dtype=np.int32)
    for t in range(T):
        v_ref = O.up_gemv(*ex_np[:3], d, bits, group, x[t])
        if want_list:
            assert count[t].item() == f and np.array_equal(idx[t].cpu().numpy(), every)
        assert G.rel_err(y[t], O.sparse_ffn(ex_np[3], x[t], v_ref, every)[1]) <= G.Y_TIGHT


def test_expert_ffn_with_more_than_65536_channels_uses_the_select_kernel():
    """Lists longer than 2048 mask words are compacted by the stand-alone select kernel; same results."""
    G = _gc()
    import paper_2505_05950_amd as F
    d, f, bits, group, T = 512, 66000, 2, 64, 2
    ex_np, ex_dev, x = _expert_case(9, 56, d, f, bits, group, T)
    v_ref = [O.up_gemv(*ex_np[:3], d, bits, group, x[t]) for t in range(T)]
    tau = np.array([O.threshold_for_sparsity(v_ref[t], 95) * 1.003 for t in range(T)], np.float32)
    y = torch.zeros((T, d), dtype=torch.float32, device=G.DEV)
    y, idx, count = F.floe_expert_ffn_sparse(ex_dev, G.dev(x), G.dev(tau), None, y)
    torch.cuda.synchronize()
    y, idx, count = y.cpu().numpy().astype(np.float64), idx.cpu().numpy(), count.cpu().numpy()
    for t in range(T):
        got = idx[t, : count[t]]
        G.check_index_set(got, v_ref[t], float(tau[t]))
        assert G.rel_err(y[t], O.sparse_ffn(ex_np[3], x[t], v_ref[t], got)[1]) <= G.Y_TIGHT


def test_zero_tokens_is_a_no_op():
    G = _gc()
    import paper_2505_05950_amd as F
    ex_np, ex_dev, x = _expert_case(6, 54, 1024, 128, 2, 64, 1)
    y = torch.zeros((0, 1024), dtype=torch.float32, device=G.DEV)
    F.floe_expert_ffn_sparse(ex_dev, G.dev(x[:0]), G.dev(np.zeros(0, np.float32)), None, y)
    torch.cuda.synchronize()


# ------------------------------------------------------------------------------------------- S7
@pytest.mark.parametrize("d,f,frac,cap_frac", [(1024, 512, 0.2, 1.0), (4096, 700, 0.2, 1.0), (2048, 300, 0.5, 0.6)])
def test_stage_channels_copies_exact_rows(d, f, frac, cap_frac):
    G = _gc()
    import paper_2505_05950_amd as F
    gd = S.expert_weights(7, 55, d, f)[1]
    host = torch.from_numpy(gd).pin_memory()
    K = int(f * frac)
    sel = S.random_channel_subset(7, 55, f, K)
    cap = int(K * cap_frac)
    idx = np.full(f, -1, np.int32)
    idx[:K] = sel
    dst = torch.zeros((max(cap, 1), 2, d), dtype=torch.float16, device=G.DEV)
    overflow = torch.full((1,), 7, dtype=torch.int32, device=G.DEV)
    side = torch.cuda.Stream()
    done = torch.cuda.Event()
    F.floe_stage_channels(host, G.dev(idx), G.dev(np.array([K], np.int32)), cap, dst, overflow, side, done)
    done.synchronize()
    got = dst.cpu().numpy()
    ref = O.stage_rows(gd, sel[:cap])
    assert got[:cap].tobytes() == ref.tobytes()
    assert ref.nbytes == cap * 4 * d                     # K * 2 * d_hidden * num_bytes
    assert overflow.item() == (1 if K > cap else 0)


def test_staged_rows_feed_gate_down():
    """Offloaded flow: S2+S3 pick the channels, S7 stages them, S4+S5 read the staged rows."""
    G = _gc()
    import paper_2505_05950_amd as F
    d, f, bits, group, pct = 1024, 900, 2, 64, 80
    ex_np, ex_dev, x = _expert_case(8, 55, d, f, bits, group, 1)
    xd = G.dev(x)
    v = F.floe_up_gemv(ex_dev.up_codes, ex_dev.up_scale, ex_dev.up_zero, xd, d, bits, group)
    v_ref = O.up_gemv(*ex_np[:3], d, bits, group, x[0])
    tau = O.threshold_for_sparsity(v_ref, pct)
    idx, count = F.floe_select_channels(v, G.dev(np.array([tau], np.float32)))
    host = torch.from_numpy(ex_np[3]).pin_memory()
    cap = 256
    staged = torch.zeros((cap, 2, d), dtype=torch.float16, device=G.DEV)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    done = torch.cuda.Event()
    F.floe_stage_channels(host, idx, count, cap, staged, None, side, done)
    torch.cuda.current_stream().wait_event(done)
    e_st = F.Expert(d, f, bits, group, ex_dev.up_codes, ex_dev.up_scale, ex_dev.up_zero, staged, staged=True, gd_rows=cap)
    y = torch.zeros((1, d), dtype=torch.float32, device=G.DEV)
    F.floe_gate_down_sparse(e_st, xd, v, idx, count, None, y)
    torch.cuda.synchronize()
    K = count.item()
    got_idx = idx[0, :K].cpu().numpy()
    G.check_index_set(got_idx, v_ref, tau)
    assert K <= cap
    y_ref = O.sparse_ffn(ex_np[3], x[0], v.cpu().numpy()[0], got_idx)[1]
    assert G.rel_err(y.cpu().numpy()[0].astype(np.float64), y_ref) <= 2e-4


# ------------------------------------------------------------------------------------------- staged code ring
@pytest.mark.parametrize("f,group,T", [(1, 64, 1), (27, 64, 1), (112, 64, 2), (113, 128, 1), (250, 256, 3), (341, 64, 1),
                                       (28 * 4 * 3 + 5, 64, 2), (2000, 64, 1), (14336, 64, 1)])
def test_fused_kernel_codes_through_the_lds_ring_match_the_register_path(f, group, T):
    """The INT2 producers of the fused kernel fetch their codes through a ring in LDS that is read back behind
    hand-counted waits (three memory requests per pass, in source order).  Should a compiler ever change that count,
    a pass would read the previous occupant of its slot: v would differ.  This compares the fused kernel's v (it stores
    v when the caller asks for the index list) with the GEMV kernel that keeps the codes in registers, bit for bit: both
    form every channel's sum in the same order.  Shapes: one channel, less than one pass per producer, exactly one block,
    one more, ragged last blocks, every block length (28 / 14 / 7 passes) and the full Mixtral width."""
    G = _gc()
    import paper_2505_05950_amd as F
    d, bits = 4096, 2
    w_up, gd = S.expert_weights(80, 2, d, f)
    ex_np, ex_dev = G.make_expert(w_up, gd, bits, group)
    x = G.dev(S.tokens(80, 2, T, d))
    v_ref = F.floe_up_gemv(ex_dev.up_codes, ex_dev.up_scale, ex_dev.up_zero, x, d, bits, group)
    tau = torch.full((T,), 0.5, dtype=torch.float32, device=G.DEV)
    y = torch.zeros((T, d), dtype=torch.float32, device=G.DEV)
    nbytes = F.floe_expert_workspace_bytes(d, f, bits, group, T)
    ws = torch.zeros((nbytes + 512,), dtype=torch.uint8, device=G.DEV)
    F.floe_expert_ffn_sparse(ex_dev, x, tau, None, y, workspace=ws)          # with the list: the fused kernel stores v
    torch.cuda.synchronize()
    off = (-ws.data_ptr()) % 256
    v_fused = ws[off: off + T * f * 4].view(torch.float32).reshape(T, f)     # v is the first array of the workspace
    assert torch.equal(v_fused, v_ref), (v_fused - v_ref).abs().max().item()
