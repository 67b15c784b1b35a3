"""ctypes binding of liblexi_moe.so: argument marshalling only, every step of the path runs in the HIP kernels.

PyTorch is used for device memory and streams, nothing else.  If the library has not been built the import of
this module fails loudly; there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os
from typing import Dict, Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblexi_moe.so")

LEXI_OK = 0
LEXI_F32, LEXI_BF16 = 0, 1
SHARED_NONE, SHARED_UNGATED, SHARED_SIGMOID = 0, 1, 2

EXPORTS = ("lexi_pack_weights", "lexi_moe_workspace_bytes", "lexi_moe_layer_forward", "lexi_moe_layer_forward_static",
           "lexi_moe_stack_forward",
           "lexi_moe_stack_forward_profiled", "lexi_moe_profile_workspace_bytes", "lexi_moe_profile_layer",
           "lexi_allocate_topk", "lexi_probe_mfma_bf16", "lexi_probe_hbm_read", "lexi_moe_down_plan", "lexi_strerror",
           "lexi_moe_version")
N_STAGE_EVENTS = 6
STAGE_NAMES = ("routing", "gate_up", "down", "shared", "combine")


class LexiError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {strerror(status)} (status {status})")


class lexi_layer_t(ctypes.Structure):
    _fields_ = [("d", ctypes.c_int32), ("E", ctypes.c_int32), ("F", ctypes.c_int32), ("F_shared", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("shared_kind", ctypes.c_int32),
                ("w_router", ctypes.c_void_p), ("router_bias", ctypes.c_void_p),
                ("w_gate", ctypes.c_void_p), ("w_up", ctypes.c_void_p), ("w_down", ctypes.c_void_p),
                ("ws_gate", ctypes.c_void_p), ("ws_up", ctypes.c_void_p), ("ws_down", ctypes.c_void_p),
                ("w_shared_gate", ctypes.c_void_p)]


class lexi_routing_out_t(ctypes.Structure):
    _fields_ = [("topk_idx", ctypes.c_void_p), ("gates", ctypes.c_void_p), ("counts", ctypes.c_void_p),
                ("offsets", ctypes.c_void_p), ("perm", ctypes.c_void_p), ("inv_perm", ctypes.c_void_p),
                ("moe_input", ctypes.c_void_p)]


class lexi_stage_events_t(ctypes.Structure):
    _fields_ = [("ev", ctypes.c_void_p * N_STAGE_EVENTS)]


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2509_02753_amd.build` "
                          "(there is no fallback implementation)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
    lib.lexi_pack_weights.restype = i32
    lib.lexi_pack_weights.argtypes = [vp, vp, i64, i32, i32, i32, vp]
    lib.lexi_moe_workspace_bytes.restype = sz
    lib.lexi_moe_workspace_bytes.argtypes = [ctypes.POINTER(lexi_layer_t), i32, i32, i32]
    lib.lexi_moe_layer_forward.restype = i32
    lib.lexi_moe_layer_forward.argtypes = [ctypes.POINTER(lexi_layer_t), vp, vp, i32, i32, i32, vp, sz, vp,
                                           ctypes.POINTER(lexi_routing_out_t)]
    lib.lexi_moe_layer_forward_static.restype = i32
    lib.lexi_moe_layer_forward_static.argtypes = [ctypes.POINTER(lexi_layer_t), vp, vp, i32, i32, i32, vp,
                                                  ctypes.POINTER(lexi_routing_out_t)]
    lib.lexi_moe_stack_forward.restype = i32
    lib.lexi_moe_stack_forward.argtypes = [ctypes.POINTER(lexi_layer_t), i32, ctypes.POINTER(i32), vp, i64, vp, i64,
                                           i32, i32, i32, vp, sz, vp, ctypes.POINTER(lexi_routing_out_t)]
    lib.lexi_moe_stack_forward_profiled.restype = i32
    lib.lexi_moe_stack_forward_profiled.argtypes = lib.lexi_moe_stack_forward.argtypes + [ctypes.POINTER(lexi_stage_events_t)]
    lib.lexi_moe_profile_workspace_bytes.restype = sz
    lib.lexi_moe_profile_workspace_bytes.argtypes = [ctypes.POINTER(lexi_layer_t), i32, i32, i32]
    lib.lexi_moe_profile_layer.restype = i32
    lib.lexi_moe_profile_layer.argtypes = [ctypes.POINTER(lexi_layer_t), vp, i32, i32, ctypes.POINTER(i32), i32, vp, vp, sz, vp]
    lib.lexi_allocate_topk.restype = i32
    lib.lexi_allocate_topk.argtypes = [ctypes.POINTER(ctypes.c_double), i32, i32, i32, i32, i32, i32, ctypes.c_double,
                                       ctypes.c_uint64, ctypes.POINTER(i32), ctypes.POINTER(ctypes.c_double)]
    lib.lexi_probe_mfma_bf16.restype = i32
    lib.lexi_probe_mfma_bf16.argtypes = [vp, vp, i32, i32, vp]
    lib.lexi_probe_hbm_read.restype = i32
    lib.lexi_probe_hbm_read.argtypes = [vp, sz, vp, vp]
    lib.lexi_moe_down_plan.restype = i32
    lib.lexi_moe_down_plan.argtypes = [ctypes.POINTER(lexi_layer_t), i32, i32, i32]
    lib.lexi_strerror.restype = ctypes.c_char_p
    lib.lexi_strerror.argtypes = [i32]
    lib.lexi_moe_version.restype = ctypes.c_char_p
    return lib


_lib = _load()


def strerror(status: int) -> str:
    return _lib.lexi_strerror(int(status)).decode()


def version() -> str:
    return _lib.lexi_moe_version().decode()


def _dp(t: Optional[torch.Tensor]):
    return None if t is None else t.data_ptr()


def _stream_ptr(stream: Optional[torch.cuda.Stream]):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _dtype_code(t: torch.dtype) -> int:
    if t == torch.float32:
        return LEXI_F32
    if t == torch.bfloat16:
        return LEXI_BF16
    raise ValueError(f"unsupported dtype {t}")


def lexi_pack_weights(w: torch.Tensor, stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """Row-major [..., rows, K] expert weights -> a new tensor of the same shape holding the packed layout."""
    if not (w.is_cuda and w.is_contiguous() and w.dim() >= 2):
        raise ValueError("lexi_pack_weights: contiguous CUDA tensor [..., rows, K] required")
    rows, K = int(w.shape[-2]), int(w.shape[-1])
    n = w.numel() // (rows * K)
    out = torch.empty_like(w)
    st = _lib.lexi_pack_weights(_dp(w), _dp(out), n, rows, K, _dtype_code(w.dtype), _stream_ptr(stream))
    if st != LEXI_OK:
        raise LexiError(st, "lexi_pack_weights")
    return out


class Layer:
    """Host-side lexi_layer_t plus references that keep its device tensors alive.

    The constructor takes expert weight matrices already in the packed layout; `from_tensors` takes row-major
    tensors and packs them with the library's own kernel."""

    def __init__(self, w_router, w_gate, w_up, w_down, router_bias=None, ws_gate=None, ws_up=None, ws_down=None,
                 w_shared_gate=None, shared_kind: Optional[int] = None):
        E, F, d = w_gate.shape
        self.d, self.E, self.F = int(d), int(E), int(F)
        self.F_shared = 0 if ws_gate is None else int(ws_gate.shape[0])
        if shared_kind is None:
            shared_kind = SHARED_NONE if ws_gate is None else (SHARED_SIGMOID if w_shared_gate is not None else SHARED_UNGATED)
        self.shared_kind = shared_kind
        self.dtype = w_gate.dtype
        self.tensors = dict(w_router=w_router, router_bias=router_bias, w_gate=w_gate, w_up=w_up, w_down=w_down,
                            ws_gate=ws_gate, ws_up=ws_up, ws_down=ws_down, w_shared_gate=w_shared_gate)
        for name, t in self.tensors.items():
            if t is not None and not (t.is_cuda and t.is_contiguous()):
                raise ValueError(f"{name}: contiguous CUDA tensor required")
        self.c = lexi_layer_t(self.d, self.E, self.F, self.F_shared, _dtype_code(self.dtype), shared_kind,
                              _dp(w_router), _dp(router_bias), _dp(w_gate), _dp(w_up), _dp(w_down), _dp(ws_gate),
                              _dp(ws_up), _dp(ws_down), _dp(w_shared_gate))

    @classmethod
    def from_tensors(cls, tensors: Dict[str, Optional[torch.Tensor]], shared_kind: Optional[int] = None) -> "Layer":
        """tensors: row-major w_gate/w_up [E][F][d], w_down [E][d][F], ws_gate/ws_up [Fs][d], ws_down [d][Fs], ..."""
        def pk(name):
            t = tensors.get(name)
            return None if t is None else lexi_pack_weights(t)
        return cls(tensors["w_router"], pk("w_gate"), pk("w_up"), pk("w_down"),
                   router_bias=tensors.get("router_bias"), ws_gate=pk("ws_gate"), ws_up=pk("ws_up"),
                   ws_down=pk("ws_down"), w_shared_gate=tensors.get("w_shared_gate"), shared_kind=shared_kind)


class RoutingOut:
    """Device arrays that receive the routing decision of one layer call."""

    def __init__(self, T: int, k: int, E: int, device="cuda:0", moe_input: Optional[torch.Tensor] = None):
        i32 = dict(dtype=torch.int32, device=device)
        self.moe_input = moe_input          # optional [T][d] tensor of the layer dtype
        self.topk_idx = torch.empty((T, k), **i32)
        self.gates = torch.empty((T, k), dtype=torch.float32, device=device)
        self.counts = torch.empty(E, **i32)
        self.offsets = torch.empty(E + 1, **i32)
        self.perm = torch.empty(T * k, **i32)
        self.inv_perm = torch.empty(T * k, **i32)
        self.c = lexi_routing_out_t(_dp(self.topk_idx), _dp(self.gates), _dp(self.counts), _dp(self.offsets),
                                    _dp(self.perm), _dp(self.inv_perm), _dp(moe_input))


def _layer_array(layers: Sequence[Layer]):
    arr = (lexi_layer_t * len(layers))()
    for i, ly in enumerate(layers):
        arr[i] = ly.c
    return arr


def lexi_moe_workspace_bytes(layers: Sequence[Layer], T_max: int, k_max: int) -> int:
    return int(_lib.lexi_moe_workspace_bytes(_layer_array(layers), len(layers), T_max, k_max))


def alloc_workspace(layers: Sequence[Layer], T_max: int, k_max: int, device="cuda:0") -> torch.Tensor:
    n = lexi_moe_workspace_bytes(layers, T_max, k_max)
    if n == 0:
        raise LexiError(-2, "lexi_moe_workspace_bytes")
    return torch.empty(n, dtype=torch.uint8, device=device)


def _check_io(where: str, x: torch.Tensor, y: Optional[torch.Tensor], d: int, dtype: torch.dtype) -> None:
    """The C ABI takes bare pointers: a tensor of another dtype, width or stride would be misread silently."""
    if not (x.is_cuda and x.dtype == dtype and int(x.shape[-1]) == d and x.stride(-1) == 1 and
            (x.dim() < 2 or x.stride(-2) == d)):
        raise ValueError(f"{where}: x must be a CUDA tensor [..., T, {d}] of {dtype} with contiguous rows")
    if y is not None and not (y.is_cuda and int(y.shape[-1]) == d and y.stride(-1) == 1 and
                              (y.dim() < 2 or y.stride(-2) == d) and int(y.shape[-2]) == int(x.shape[-2])):
        raise ValueError(f"{where}: y must be a CUDA tensor [..., T, {d}] with contiguous rows")


def lexi_moe_layer_forward(layer: Layer, x: torch.Tensor, y: torch.Tensor, k: int, workspace: torch.Tensor,
                           routing: Optional[RoutingOut] = None, stream: Optional[torch.cuda.Stream] = None) -> None:
    """y = f_moe(x; k) for one layer, enqueued on `stream` (default: torch's current stream)."""
    _check_io("lexi_moe_layer_forward", x, y, layer.d, layer.dtype)
    if x.dim() != 2 or y.dim() != 2:
        raise ValueError("lexi_moe_layer_forward: x and y are [T][d]")
    T = int(x.shape[0])
    st = _lib.lexi_moe_layer_forward(ctypes.byref(layer.c), _dp(x), _dp(y), _dtype_code(y.dtype), T, int(k),
                                     _dp(workspace), workspace.numel(), _stream_ptr(stream),
                                     ctypes.byref(routing.c) if routing is not None else None)
    if st != LEXI_OK:
        raise LexiError(st, "lexi_moe_layer_forward")


def lexi_moe_layer_forward_static(layer: Layer, x: torch.Tensor, y: torch.Tensor, k: int,
                                  routing: Optional[RoutingOut] = None, stream: Optional[torch.cuda.Stream] = None) -> None:
    """lexi_moe_layer_forward without a workspace argument: the library's static device scratch (64 MiB) is used."""
    _check_io("lexi_moe_layer_forward_static", x, y, layer.d, layer.dtype)
    if x.dim() != 2 or y.dim() != 2:
        raise ValueError("lexi_moe_layer_forward_static: x and y are [T][d]")
    st = _lib.lexi_moe_layer_forward_static(ctypes.byref(layer.c), _dp(x), _dp(y), _dtype_code(y.dtype), int(x.shape[0]),
                                            int(k), _stream_ptr(stream),
                                            ctypes.byref(routing.c) if routing is not None else None)
    if st != LEXI_OK:
        raise LexiError(st, "lexi_moe_layer_forward_static")


def lexi_moe_stack_forward(layers: Sequence[Layer], k_vec: Sequence[int], x: torch.Tensor, y: torch.Tensor,
                           workspace: torch.Tensor, routing: Optional[Sequence[RoutingOut]] = None,
                           stream: Optional[torch.cuda.Stream] = None, layer_array=None, stage_events=None,
                           chained: bool = False) -> None:
    """Stack of L layers with the per-layer k vector.  x: [T][d] (shared by all layers) or [L][T][d]; y: [L][T][d].
    chained=True: pre-norm residual blocks h_{l+1} = h_l + f_l(norm(h_l)); x [T][d], y fp32 [L][T][d] or [T][d].

    stage_events: None, or a StageEvents object; then the profiled entry point records its events."""
    L = len(layers)
    for ly in layers:
        _check_io("lexi_moe_stack_forward", x, y, ly.d, ly.dtype)
    if x.dim() not in (2, 3) or y.dim() not in (2, 3) or (x.dim() == 3 and int(x.shape[0]) < L) or \
            (y.dim() == 3 and int(y.shape[0]) < L):
        raise ValueError("lexi_moe_stack_forward: x is [T][d] or [L][T][d], y is [L][T][d] (or [T][d])")
    T = int(x.shape[-2])
    x_stride = 0 if x.dim() == 2 else int(x.stride(0))
    y_stride = int(y.stride(0)) if y.dim() == 3 else 0
    kv = (ctypes.c_int32 * L)(*[int(v) for v in k_vec])
    dbg = None
    if routing is not None:
        dbg = (lexi_routing_out_t * L)()
        for i, r in enumerate(routing):
            dbg[i] = r.c
    arr = layer_array if layer_array is not None else _layer_array(layers)
    if stage_events is not None:
        st = _lib.lexi_moe_stack_forward_profiled(arr, L, kv, _dp(x), x_stride, _dp(y), y_stride, _dtype_code(y.dtype),
                                                  T, int(chained), _dp(workspace), workspace.numel(), _stream_ptr(stream), dbg,
                                                  stage_events.c)
    else:
        st = _lib.lexi_moe_stack_forward(arr, L, kv, _dp(x), x_stride, _dp(y), y_stride, _dtype_code(y.dtype), T,
                                         int(chained), _dp(workspace), workspace.numel(), _stream_ptr(stream), dbg)
    if st != LEXI_OK:
        raise LexiError(st, "lexi_moe_stack_forward")


def lexi_moe_profile_layer(layer: Layer, x: torch.Tensor, k_base: int, k_list: Sequence[int],
                           workspace: Optional[torch.Tensor] = None, stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """Delta_k = ||f_moe(x; k) - f_moe(x; k_base)||_F for every k of k_list (Algorithm 1, one iteration), as a device
    float tensor [len(k_list)].  The workspace is allocated here when none is given."""
    _check_io("lexi_moe_profile_layer", x, None, layer.d, layer.dtype)
    if x.dim() != 2:
        raise ValueError("lexi_moe_profile_layer: x is [T][d]")
    T, n = int(x.shape[0]), len(k_list)
    need = int(_lib.lexi_moe_profile_workspace_bytes(ctypes.byref(layer.c), T, int(k_base), n))
    if need == 0:
        raise LexiError(-2, "lexi_moe_profile_workspace_bytes")
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
    delta = torch.empty(n, dtype=torch.float32, device=x.device)
    kl = (ctypes.c_int32 * n)(*[int(k) for k in k_list])
    st = _lib.lexi_moe_profile_layer(ctypes.byref(layer.c), _dp(x), T, int(k_base), kl, n, _dp(delta), _dp(workspace),
                                     workspace.numel(), _stream_ptr(stream))
    if st != LEXI_OK:
        raise LexiError(st, "lexi_moe_profile_layer")
    return delta


def lexi_allocate_topk(D, B: int, k_min: int, k_max: int, n_pop: int = 32, g_max: int = 500, eta_mut: float = 0.1,
                       seed: int = 0):
    """Stage 2 (Algorithm 2) on the host: D [L][k_max+1] losses -> (k* as a list of ints, phi(k*))."""
    import numpy as np
    D = np.ascontiguousarray(D, dtype=np.float64)
    if D.ndim != 2 or D.shape[1] != k_max + 1:
        raise ValueError("D must be [L][k_max + 1]")
    L = int(D.shape[0])
    out = (ctypes.c_int32 * L)()
    phi = ctypes.c_double()
    st = _lib.lexi_allocate_topk(D.ctypes.data_as(ctypes.POINTER(ctypes.c_double)), L, int(B), int(k_min), int(k_max),
                                 int(n_pop), int(g_max), float(eta_mut), int(seed), out, ctypes.byref(phi))
    if st != LEXI_OK:
        raise LexiError(st, "lexi_allocate_topk")
    return list(out), phi.value


def lexi_moe_down_plan(layer: Layer, T: int, k: int, shared: bool = False) -> int:
    """Schedule of the (routed or shared) down GEMM of a call: 0 streaming, 1 tiles, 2 tiles with the reduction cut in
    two, 3 tiles storing the output rows directly, 4 streaming with the combine in the same launch; -1 if there is no
    such GEMM."""
    return int(_lib.lexi_moe_down_plan(ctypes.byref(layer.c), int(T), int(k), 1 if shared else 0))


def lexi_probe_mfma_bf16(operands: torch.Tensor, sink: torch.Tensor, iters: int, workgroups: int,
                         stream: Optional[torch.cuda.Stream] = None) -> float:
    """Enqueue the matrix-core probe; returns the flops it executes (time it with events)."""
    st = _lib.lexi_probe_mfma_bf16(_dp(operands), _dp(sink), int(iters), int(workgroups), _stream_ptr(stream))
    if st != LEXI_OK:
        raise LexiError(st, "lexi_probe_mfma_bf16")
    return float(workgroups) * 4 * iters * 16 * 32768


def lexi_probe_hbm_read(src: torch.Tensor, sink: torch.Tensor, stream: Optional[torch.cuda.Stream] = None) -> float:
    """Enqueue one streaming read of `src`; returns the bytes read (time it with events)."""
    nbytes = src.numel() * src.element_size()
    st = _lib.lexi_probe_hbm_read(_dp(src), nbytes, _dp(sink), _stream_ptr(stream))
    if st != LEXI_OK:
        raise LexiError(st, "lexi_probe_hbm_read")
    return float(nbytes)


class StageEvents:
    """L x 6 HIP events (created through torch) that the profiled stack entry point records between stages."""

    def __init__(self, L: int):
        self.L = L
        self.events = [[torch.cuda.Event(enable_timing=True) for _ in range(N_STAGE_EVENTS)] for _ in range(L)]
        for row in self.events:          # torch creates the underlying hipEvent_t on the first record
            for e in row:
                e.record()
        torch.cuda.synchronize()
        self.c = (lexi_stage_events_t * L)()
        for l, row in enumerate(self.events):
            for i, e in enumerate(row):
                self.c[l].ev[i] = e.cuda_event

    def stage_ms(self):
        """After a synchronize: per-layer list of the 5 stage durations in milliseconds (routing, gate/up, down, shared,
        combine).  Where the library recorded "shared expert done" before "down done" (down projection and combine in
        one launch), the wait for the shared expert is the shared stage and the launch is the down stage."""
        out = []
        for row in self.events:
            t = [row[0].elapsed_time(e) for e in row]
            if t[4] < t[3]:
                out.append([t[1], t[2] - t[1], t[3] - t[4], t[4] - t[2], t[5] - t[3]])
            else:
                out.append([t[i + 1] - t[i] for i in range(N_STAGE_EVENTS - 1)])
        return out
