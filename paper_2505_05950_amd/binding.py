"""ctypes binding of include/floe.h.  Argument marshalling only: torch owns device memory and streams,
the functions below pass raw pointers and sizes to the C ABI under the same names."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_NAME = "libfloe_hip.so"
_lib = None

SLOT_STAT_DTYPE = np.dtype([("expert", np.int32), ("count", np.int32), ("weight", np.float32), ("staged", np.int32)])


class FloeError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = load().floe_status_string(status).decode()
        if status == -5:
            msg += f" [hipError {load().floe_last_hip_error()}]"
        super().__init__(f"{where}: {msg} (status {status})")


class _Shape(C.Structure):
    _fields_ = [("d", C.c_int32), ("f", C.c_int32), ("bits", C.c_int32), ("group", C.c_int32)]


class _Expert(C.Structure):
    _fields_ = [("s", _Shape), ("up_codes", C.c_void_p), ("up_scale", C.c_void_p), ("up_zero", C.c_void_p),
                ("gd", C.c_void_p), ("gd_is_staged", C.c_int32), ("gd_rows", C.c_int32)]


class _Layer(C.Structure):
    _fields_ = [("n_experts", C.c_int32), ("top_k", C.c_int32), ("n_shared", C.c_int32), ("renormalize", C.c_int32),
                ("s", _Shape), ("router_cm", C.c_void_p), ("experts", C.POINTER(_Expert)), ("tau", C.c_void_p),
                ("tau_stride_t", C.c_int32), ("dev_table", C.c_void_p), ("gd_on_host", C.c_int32)]


class _Offload(C.Structure):
    _fields_ = [("staging", C.c_void_p), ("capacity_rows", C.c_int32), ("overflow", C.c_void_p),
                ("side_stream", C.c_void_p), ("ev_lists_ready", C.c_void_p), ("ev_staged", C.c_void_p)]


class _Prefetch(C.Structure):
    _fields_ = [("staging", C.c_void_p), ("capacity_rows", C.c_int32), ("pred_expert", C.c_void_p),
                ("pred_count", C.c_void_p), ("row_of", C.c_void_p), ("prefetch_stream", C.c_void_p),
                ("ev_inputs_ready", C.c_void_p), ("ev_prefetched", C.c_void_p)]


class _MissPath(C.Structure):
    _fields_ = [("miss_stream", C.c_void_p), ("ev_lists_ready", C.c_void_p), ("ev_staged", C.c_void_p),
                ("overflow", C.c_void_p)]


class _ChannelCache(C.Structure):
    _fields_ = [("pool", C.c_void_p), ("row_of", C.c_void_p), ("resident_rows", C.c_int32), ("capacity_rows", C.c_int32)]


def lib_path() -> str:
    return os.path.join(_HERE, _LIB_NAME)


def load():
    """Loads the in-tree HIP library; raises if it has not been built (there is no fallback)."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(or python paper_2505_05950_amd/build.py) first; this package has no CPU fallback")
    lib = C.CDLL(path)
    vp, i32, sz = C.c_void_p, C.c_int, C.c_size_t
    lib.floe_status_string.restype = C.c_char_p
    lib.floe_status_string.argtypes = [i32]
    lib.floe_last_hip_error.restype = i32
    lib.floe_abi_version.restype = i32
    lib.floe_profile_kernel.argtypes = [i32, vp, vp]
    lib.floe_tuning.argtypes = [i32, i32]
    lib.floe_quantize_expert.argtypes = [C.POINTER(_Shape), vp, vp, vp, vp, vp]
    lib.floe_up_gemv.argtypes = [C.POINTER(_Shape), vp, vp, vp, vp, i32, vp, vp]
    lib.floe_select_channels.argtypes = [vp, i32, i32, vp, vp, vp, vp]
    lib.floe_expert_workspace_bytes.restype = sz
    lib.floe_expert_workspace_bytes.argtypes = [C.POINTER(_Shape), i32]
    lib.floe_gate_down_sparse.argtypes = [C.POINTER(_Expert), vp, i32, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.floe_expert_ffn_sparse.argtypes = [C.POINTER(_Expert), vp, i32, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.floe_expert_sparsified_workspace_bytes.restype = sz
    lib.floe_expert_sparsified_workspace_bytes.argtypes = [C.POINTER(_Shape), i32]
    lib.floe_expert_ffn_sparsified.argtypes = [C.POINTER(_Expert), i32, vp, i32, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.floe_layer_table_bytes.restype = sz
    lib.floe_layer_table_bytes.argtypes = [C.POINTER(_Layer)]
    lib.floe_layer_build_table.argtypes = [C.POINTER(_Layer), vp, sz, vp]
    lib.floe_layer_workspace_bytes.restype = sz
    lib.floe_layer_workspace_bytes.argtypes = [C.POINTER(_Layer), i32]
    lib.floe_moe_layer_decode.argtypes = [C.POINTER(_Layer), vp, i32, vp, vp, vp, sz, vp]
    lib.floe_moe_layer_decode_static.argtypes = [C.POINTER(_Layer), vp, i32, vp, vp, vp]
    lib.floe_moe_layer_decode_offloaded.argtypes = [C.POINTER(_Layer), C.POINTER(_Offload), vp, i32, vp, vp, vp, sz, vp]
    lib.floe_moe_layer_prefetch.argtypes = [C.POINTER(_Layer), C.POINTER(_Prefetch), vp, i32, vp, sz, vp]
    lib.floe_moe_layer_decode_prefetched.argtypes = [C.POINTER(_Layer), C.POINTER(_Prefetch), C.POINTER(_MissPath), vp, i32,
                                                     vp, vp, vp, vp, sz, vp]
    lib.floe_channel_cache_load.argtypes = [C.POINTER(_Layer), C.POINTER(_ChannelCache), i32, vp, vp, i32, i32, vp]
    lib.floe_moe_layer_decode_cached.argtypes = [C.POINTER(_Layer), C.POINTER(_ChannelCache), C.POINTER(_MissPath), vp, i32,
                                                 vp, vp, vp, vp, sz, vp]
    lib.floe_stage_channels.argtypes = [vp, i32, i32, vp, vp, i32, vp, vp, vp, vp]
    _lib = lib
    return lib


def floe_status_string(status: int) -> str:
    return load().floe_status_string(status).decode()


KERNEL_IDS = {"none": 0, "quantize": 1, "router": 2, "up_gemv": 3, "select": 4, "gate_down": 5, "combine": 6, "stage": 7,
              "fused_ffn": 8}


def floe_profile_kernel(kernel: str, start_event=None, stop_event=None):
    """Arms (or, with "none", disarms) the event bracket around one kernel; events are torch.cuda.Event
    objects created with enable_timing=True and recorded at least once (torch creates them lazily)."""
    kid = KERNEL_IDS[kernel]
    a = None if start_event is None else C.c_void_p(start_event.cuda_event)
    b = None if stop_event is None else C.c_void_p(stop_event.cuda_event)
    _check(load().floe_profile_kernel(kid, a, b), "floe_profile_kernel")


TUNE_UNION_KERNELS = 1
TUNE_STAGE_WORKGROUPS = 2
TUNE_GROUPED_GEMV = 3
TUNE_FUSED_TASKS = 4


def floe_tuning(key: int, value: int):
    """Process-wide tuning switch (see include/floe.h); Layer objects cache workspaces, so set it before building them."""
    _check(load().floe_tuning(int(key), int(value)), "floe_tuning")


def words_per_channel(d: int, bits: int) -> int:
    return d * bits // 32


def _ptr(t):
    if t is None:
        return None
    assert t.is_contiguous(), "tensors handed to the C ABI must be contiguous"
    return C.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def _check(rc: int, where: str):
    if rc != 0:
        raise FloeError(rc, where)


def _shape(d, f, bits, group) -> _Shape:
    return _Shape(int(d), int(f), int(bits), int(group))


class Expert:
    """Plain holder of one compressed expert's device tensors (no ownership semantics beyond Python refs)."""

    def __init__(self, d, f, bits, group, up_codes, up_scale, up_zero, gd, staged=False, gd_rows=None):
        self.d, self.f, self.bits, self.group = int(d), int(f), int(bits), int(group)
        self.up_codes, self.up_scale, self.up_zero, self.gd = up_codes, up_scale, up_zero, gd
        self.staged = bool(staged)
        self.gd_rows = int(gd_rows if gd_rows is not None else (gd.shape[0] if gd is not None else f))

    def c_struct(self) -> _Expert:
        def p(t):
            return None if t is None else t.data_ptr()
        return _Expert(_shape(self.d, self.f, self.bits, self.group), p(self.up_codes), p(self.up_scale),
                       p(self.up_zero), p(self.gd), int(self.staged), self.gd_rows)


def floe_quantize_expert(w_up_cm: torch.Tensor, bits: int, group: int, stream=None):
    """w_up_cm fp16 [f][d] on the GPU -> (codes int32-viewed-uint32 [f][d*bits/32], scale fp16, zero fp16)."""
    f, d = w_up_cm.shape
    dev = w_up_cm.device
    codes = torch.empty((f, max(1, d * bits // 32)), dtype=torch.int32, device=dev)
    scale = torch.empty((f, max(1, d // group)), dtype=torch.float16, device=dev)
    zero = torch.empty_like(scale)
    s = _shape(d, f, bits, group)
    _check(load().floe_quantize_expert(C.byref(s), _ptr(w_up_cm), _ptr(codes), _ptr(scale), _ptr(zero), _stream(stream)),
           "floe_quantize_expert")
    return codes, scale, zero


def floe_up_gemv(codes, scale, zero, x, d, bits, group, stream=None) -> torch.Tensor:
    f = codes.shape[0]
    T = x.shape[0]
    v = torch.empty((T, f), dtype=torch.float32, device=x.device)
    s = _shape(d, f, bits, group)
    _check(load().floe_up_gemv(C.byref(s), _ptr(codes), _ptr(scale), _ptr(zero), _ptr(x), T, _ptr(v), _stream(stream)),
           "floe_up_gemv")
    return v


def floe_select_channels(v: torch.Tensor, tau: torch.Tensor, stream=None):
    T, f = v.shape
    idx = torch.full((T, f), -1, dtype=torch.int32, device=v.device)
    count = torch.empty((T,), dtype=torch.int32, device=v.device)
    _check(load().floe_select_channels(_ptr(v), f, T, _ptr(tau), _ptr(idx), _ptr(count), _stream(stream)),
           "floe_select_channels")
    return idx, count


def floe_expert_workspace_bytes(d, f, bits, group, T) -> int:
    s = _shape(d, f, bits, group)
    return int(load().floe_expert_workspace_bytes(C.byref(s), int(T)))


def _workspace(nbytes: int, device) -> torch.Tensor:
    return torch.empty((max(nbytes, 256) + 256,), dtype=torch.uint8, device=device)


def _aligned_ptr(ws: torch.Tensor):
    base = ws.data_ptr()
    off = (-base) % 256
    return C.c_void_p(base + off), ws.numel() - off


def floe_gate_down_sparse(e: Expert, x, v, idx, count, out_scale, y_acc, workspace=None, stream=None):
    T = x.shape[0]
    if workspace is None:
        workspace = _workspace(floe_expert_workspace_bytes(e.d, e.f, e.bits, e.group, T), x.device)
    wp, wn = _aligned_ptr(workspace)
    es = e.c_struct()
    _check(load().floe_gate_down_sparse(C.byref(es), _ptr(x), T, _ptr(v), _ptr(idx), _ptr(count), _ptr(out_scale),
                                        _ptr(y_acc), wp, wn, _stream(stream)), "floe_gate_down_sparse")
    return y_acc


def floe_expert_ffn_sparse(e: Expert, x, tau, out_scale, y_acc, idx=None, count=None, workspace=None, stream=None,
                           want_list=True):
    """Alg. 1 for T tokens; returns (y_acc, idx, count); want_list=False passes no list buffers (idx, count = None)."""
    T = x.shape[0]
    if want_list:
        if idx is None:
            idx = torch.full((T, e.f), -1, dtype=torch.int32, device=x.device)
        if count is None:
            count = torch.empty((T,), dtype=torch.int32, device=x.device)
    else:
        idx = count = None
    if workspace is None:
        workspace = _workspace(floe_expert_workspace_bytes(e.d, e.f, e.bits, e.group, T), x.device)
    wp, wn = _aligned_ptr(workspace)
    es = e.c_struct()
    _check(load().floe_expert_ffn_sparse(C.byref(es), _ptr(x), T, _ptr(tau), _ptr(out_scale), _ptr(y_acc), _ptr(idx),
                                         _ptr(count), wp, wn, _stream(stream)), "floe_expert_ffn_sparse")
    return y_acc, idx, count


SPARSIFY_UP, SPARSIFY_GATE, SPARSIFY_DOWN = 0, 1, 2


def floe_expert_ffn_sparsified(e: Expert, which: int, x, tau, out_scale, y_acc, workspace=None, stream=None):
    """Eq. 1 with the sparsity function on a_up / a_gate / a_down (Sec. 3.2.1); returns (y_acc, idx, count)."""
    T = x.shape[0]
    idx = torch.full((T, e.f), -1, dtype=torch.int32, device=x.device)
    count = torch.empty((T,), dtype=torch.int32, device=x.device)
    if workspace is None:
        s = _shape(e.d, e.f, e.bits, e.group)
        workspace = _workspace(int(load().floe_expert_sparsified_workspace_bytes(C.byref(s), T)), x.device)
    wp, wn = _aligned_ptr(workspace)
    es = e.c_struct()
    _check(load().floe_expert_ffn_sparsified(C.byref(es), int(which), _ptr(x), T, _ptr(tau), _ptr(out_scale), _ptr(y_acc),
                                             _ptr(idx), _ptr(count), wp, wn, _stream(stream)), "floe_expert_ffn_sparsified")
    return y_acc, idx, count


class Layer:
    """One MoE layer: routed experts first, shared experts last; builds the HBM pointer table once."""

    def __init__(self, experts, n_shared, top_k, renormalize, router_cm, tau, tau_per_token: bool, stream=None,
                 gd_on_host: bool = False):
        self.experts = list(experts)
        e0 = self.experts[0]
        self.d, self.f, self.bits, self.group = e0.d, e0.f, e0.bits, e0.group
        self.n_shared, self.top_k, self.renormalize = int(n_shared), int(top_k), bool(renormalize)
        self.n_experts = len(self.experts) - self.n_shared
        self.router_cm, self.tau = router_cm, tau
        self.tau_stride = len(self.experts) if tau_per_token else 0
        self._arr = (_Expert * len(self.experts))(*[e.c_struct() for e in self.experts])
        self._c = _Layer(self.n_experts, self.top_k, self.n_shared, int(self.renormalize),
                         _shape(self.d, self.f, self.bits, self.group),
                         None if router_cm is None else router_cm.data_ptr(), self._arr, tau.data_ptr(),
                         self.tau_stride, None, int(gd_on_host))
        self.gd_on_host = bool(gd_on_host)
        nbytes = floe_layer_table_bytes(self)
        self.table = torch.empty((nbytes + 256,), dtype=torch.uint8, device=tau.device)
        tp, tn = _aligned_ptr(self.table)
        floe_layer_build_table(self, tp, tn, stream)
        self._c.dev_table = tp
        self._ws = {}

    def set_tau(self, tau, tau_per_token: bool):
        self.tau = tau
        self.tau_stride = len(self.experts) if tau_per_token else 0
        self._c.tau = tau.data_ptr()
        self._c.tau_stride_t = self.tau_stride

    def new_workspace(self, T: int) -> torch.Tensor:
        """A workspace of its own (e.g. for a prefetch that runs beside a decode call)."""
        return _workspace(floe_layer_workspace_bytes(self, T), self.tau.device)

    def workspace(self, T: int) -> torch.Tensor:
        if T not in self._ws:
            self._ws[T] = _workspace(floe_layer_workspace_bytes(self, T), self.tau.device)
        return self._ws[T]


def floe_layer_table_bytes(L: Layer) -> int:
    return int(load().floe_layer_table_bytes(C.byref(L._c)))


def floe_layer_build_table(L: Layer, table_ptr, table_bytes, stream=None):
    _check(load().floe_layer_build_table(C.byref(L._c), table_ptr, table_bytes, _stream(stream)), "floe_layer_build_table")


def floe_layer_workspace_bytes(L: Layer, T: int) -> int:
    return int(load().floe_layer_workspace_bytes(C.byref(L._c), int(T)))


def floe_moe_layer_decode(L: Layer, x: torch.Tensor, y: torch.Tensor = None, stats: torch.Tensor = None,
                          workspace=None, stream=None):
    """x fp16 [T][d] -> y fp16 [T][d]; stats (optional) int32 [T][slots][4] viewed as floe_slot_stat."""
    T = x.shape[0]
    if y is None:
        y = torch.empty((T, L.d), dtype=torch.float16, device=x.device)
    if workspace is None:
        workspace = L.workspace(T)
    wp, wn = _aligned_ptr(workspace)
    _check(load().floe_moe_layer_decode(C.byref(L._c), _ptr(x), T, _ptr(y), _ptr(stats), wp, wn, _stream(stream)),
           "floe_moe_layer_decode")
    return y


STATIC_SCRATCH_BYTES = 16 << 20


def floe_moe_layer_decode_static(L: Layer, x: torch.Tensor, y: torch.Tensor, stats: torch.Tensor = None, stream=None):
    """floe_moe_layer_decode on the library's own scratch array; y must be supplied (nothing is allocated here)."""
    _check(load().floe_moe_layer_decode_static(C.byref(L._c), _ptr(x), x.shape[0], _ptr(y), _ptr(stats), _stream(stream)),
           "floe_moe_layer_decode_static")
    return y


def floe_moe_layer_decode_offloaded(L: Layer, x, staging, capacity_rows, side_stream, ev_lists_ready, ev_staged,
                                    y=None, stats=None, overflow=None, workspace=None, stream=None):
    """Offloaded layer: experts' gd are pinned host tensors; staging dev [T*slots][capacity_rows][2][d]."""
    T = x.shape[0]
    if y is None:
        y = torch.empty((T, L.d), dtype=torch.float16, device=x.device)
    if workspace is None:
        workspace = L.workspace(T)
    wp, wn = _aligned_ptr(workspace)
    cur = stream if stream is not None else torch.cuda.current_stream()
    # torch creates the hipEvent_t lazily on the first record(); the library records both again
    ev_lists_ready.record(cur)
    ev_staged.record(side_stream)
    off = _Offload(staging.data_ptr(), int(capacity_rows), None if overflow is None else overflow.data_ptr(),
                   side_stream.cuda_stream, ev_lists_ready.cuda_event, ev_staged.cuda_event)
    _check(load().floe_moe_layer_decode_offloaded(C.byref(L._c), C.byref(off), _ptr(x), T, _ptr(y), _ptr(stats), wp, wn,
                                                  _stream(stream)), "floe_moe_layer_decode_offloaded")
    return y


PREFETCH_STAT_DTYPE = np.dtype([("expert_predicted", np.int32), ("predicted", np.int32), ("hits", np.int32),
                                ("misses", np.int32)])


class Prefetch:
    """Buffers and events of one floe_prefetch object (two of them alternate between neighbouring layers):
    staging [2*T*slots][capacity][2][d], predicted expert / count per task, row map [T*slots][f]."""

    def __init__(self, L: "Layer", T: int, capacity_rows: int, prefetch_stream, device=None):
        dev = device if device is not None else L.tau.device
        slots = L.top_k + L.n_shared
        n = T * slots
        self.T, self.capacity_rows, self.stream = T, int(capacity_rows), prefetch_stream
        self.staging = torch.empty((2 * n, capacity_rows, 2, L.d), dtype=torch.float16, device=dev)
        self.pred_expert = torch.full((n,), -1, dtype=torch.int32, device=dev)
        self.pred_count = torch.zeros((n,), dtype=torch.int32, device=dev)
        self.row_of = torch.full((n, L.f), -1, dtype=torch.int32, device=dev)
        self.ev_inputs_ready, self.ev_prefetched = torch.cuda.Event(), torch.cuda.Event()
        # torch creates the hipEvent_t lazily on the first record(); after this the library alone records them
        self.ev_inputs_ready.record(torch.cuda.current_stream())
        self.ev_prefetched.record(prefetch_stream)
        self._c = _Prefetch(self.staging.data_ptr(), self.capacity_rows, self.pred_expert.data_ptr(),
                            self.pred_count.data_ptr(), self.row_of.data_ptr(), prefetch_stream.cuda_stream,
                            self.ev_inputs_ready.cuda_event, self.ev_prefetched.cuda_event)


class MissPath:
    """Stream and events on which the channels that were not predicted are copied."""

    def __init__(self, miss_stream, n_tasks: int, device):
        self.stream = miss_stream
        self.overflow = torch.zeros((n_tasks,), dtype=torch.int32, device=device)
        self.ev_lists_ready, self.ev_staged = torch.cuda.Event(), torch.cuda.Event()
        self.ev_lists_ready.record(torch.cuda.current_stream())
        self.ev_staged.record(miss_stream)
        self._c = _MissPath(miss_stream.cuda_stream, self.ev_lists_ready.cuda_event, self.ev_staged.cuda_event,
                            self.overflow.data_ptr())


def floe_moe_layer_prefetch(L: Layer, P: Prefetch, x_cur, workspace, stream=None):
    """Predicts layer L's experts and channels from x_cur and copies their chunks ahead (on P.stream)."""
    T = x_cur.shape[0]
    wp, wn = _aligned_ptr(workspace)
    _check(load().floe_moe_layer_prefetch(C.byref(L._c), C.byref(P._c), _ptr(x_cur), T, wp, wn, _stream(stream)),
           "floe_moe_layer_prefetch")


def floe_moe_layer_decode_prefetched(L: Layer, P: Prefetch, M: MissPath, x, y=None, stats=None, prefetch_stats=None,
                                     workspace=None, stream=None):
    """Layer decode on staging rows that floe_moe_layer_prefetch has (partly) filled; only the misses are copied now."""
    T = x.shape[0]
    if y is None:
        y = torch.empty((T, L.d), dtype=torch.float16, device=x.device)
    if workspace is None:
        workspace = L.workspace(T)
    wp, wn = _aligned_ptr(workspace)
    _check(load().floe_moe_layer_decode_prefetched(C.byref(L._c), C.byref(P._c), C.byref(M._c), _ptr(x), T, _ptr(y),
                                                   _ptr(stats), _ptr(prefetch_stats), wp, wn, _stream(stream)),
           "floe_moe_layer_decode_prefetched")
    return y


class ChannelCache:
    """Buffers of a floe_channel_cache: the pool (resident rows, then one slab per (token, slot)) and the row map."""

    def __init__(self, L: "Layer", T: int, resident_rows: int, capacity_rows: int, device=None):
        dev = device if device is not None else L.tau.device
        n = T * (L.top_k + L.n_shared)
        self.resident_rows, self.capacity_rows = int(resident_rows), int(capacity_rows)
        self.pool = torch.empty((self.resident_rows + n * self.capacity_rows, 2, L.d), dtype=torch.float16, device=dev)
        self.row_of = torch.full((len(L.experts), L.f), -1, dtype=torch.int32, device=dev)
        self._c = _ChannelCache(self.pool.data_ptr(), self.row_of.data_ptr(), self.resident_rows, self.capacity_rows)


def floe_channel_cache_load(L: Layer, cache: ChannelCache, expert: int, idx, count, first_row: int, max_rows: int, stream=None):
    _check(load().floe_channel_cache_load(C.byref(L._c), C.byref(cache._c), int(expert), _ptr(idx), _ptr(count), int(first_row),
                                          int(max_rows), _stream(stream)), "floe_channel_cache_load")


def floe_moe_layer_decode_cached(L: Layer, cache: ChannelCache, M: MissPath, x, y=None, stats=None, cache_stats=None,
                                 workspace=None, stream=None):
    T = x.shape[0]
    if y is None:
        y = torch.empty((T, L.d), dtype=torch.float16, device=x.device)
    if workspace is None:
        workspace = L.workspace(T)
    wp, wn = _aligned_ptr(workspace)
    _check(load().floe_moe_layer_decode_cached(C.byref(L._c), C.byref(cache._c), C.byref(M._c), _ptr(x), T, _ptr(y),
                                               _ptr(stats), _ptr(cache_stats), wp, wn, _stream(stream)),
           "floe_moe_layer_decode_cached")
    return y


def floe_stage_channels(host_gd: torch.Tensor, idx, count, capacity_rows: int, hbm_dst, overflow=None,
                        side_stream=None, done_event=None):
    """host_gd: pinned CPU fp16 tensor [f][2][d]; idx/count device; hbm_dst device [capacity][2][d]."""
    assert host_gd.is_pinned(), "host_gd must be pinned host memory"
    d = host_gd.shape[-1]
    f = host_gd.shape[0]
    ev = None
    if done_event is not None:
        # torch creates the underlying hipEvent_t lazily on the first record(); force that now.
        # The library records the same event again after the copy, which supersedes this one.
        done_event.record(side_stream if side_stream is not None else torch.cuda.current_stream())
        ev = C.c_void_p(done_event.cuda_event)
    _check(load().floe_stage_channels(C.c_void_p(host_gd.data_ptr()), d, f, _ptr(idx), _ptr(count), int(capacity_rows),
                                      _ptr(hbm_dst), _ptr(overflow), _stream(side_stream), ev), "floe_stage_channels")
    return hbm_dst
