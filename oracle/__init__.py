"""Python face of the CPU oracle (``lexi_oracle.c``).  TEST INFRASTRUCTURE ONLY.

Only ``tests/``, ``__graft_entry__.smoke()`` and the benchmark's CPU-baseline
leg may import this package.  It imports nothing from the HIP package and the
HIP package imports nothing from here.

Arrays are numpy: fp32 tensors as float32, bf16 tensors as uint16 bit patterns.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Dict, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# LEXI_ORACLE_LIB: load this build of lexi_oracle.c instead (the sanitizer test points it at an instrumented one)
LIB = os.environ.get("LEXI_ORACLE_LIB") or os.path.join(_HERE, "liblexi_oracle.so")
# -ffp-contract=off: the router's fused multiply-adds are the explicit fmaf() calls and nothing else.
CFLAGS = ["-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared"]


def build() -> None:
    subprocess.check_call(["gcc", *CFLAGS, "-o", LIB, os.path.join(_HERE, "lexi_oracle.c"), "-lm"])


class _Layer(ctypes.Structure):
    _fields_ = [("d", ctypes.c_int32), ("E", ctypes.c_int32), ("F", ctypes.c_int32), ("F_shared", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("shared_kind", ctypes.c_int32),
                ("w_router", ctypes.c_void_p), ("router_bias", ctypes.c_void_p),
                ("w_gate", ctypes.c_void_p), ("w_up", ctypes.c_void_p), ("w_down", ctypes.c_void_p),
                ("ws_gate", ctypes.c_void_p), ("ws_up", ctypes.c_void_p), ("ws_down", ctypes.c_void_p),
                ("w_shared_gate", ctypes.c_void_p)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB):
            build()
        L = ctypes.CDLL(LIB)
        vp, i32 = ctypes.c_void_p, ctypes.c_int32
        L.lexi_oracle_num_threads.restype = ctypes.c_int
        L.lexi_oracle_router_logits.argtypes = [ctypes.POINTER(_Layer), vp, i32, vp]
        L.lexi_oracle_topk.argtypes = [vp, i32, i32, i32, vp]
        L.lexi_oracle_gates.argtypes = [vp, vp, i32, i32, i32, vp]
        L.lexi_oracle_permutation.argtypes = [vp, i32, i32, i32, vp, vp, vp, vp]
        L.lexi_oracle_expert_ffn.argtypes = [ctypes.POINTER(_Layer), i32, vp, i32, i32, vp]
        L.lexi_oracle_shared_coeff.argtypes = [ctypes.POINTER(_Layer), vp, i32]
        L.lexi_oracle_shared_coeff.restype = ctypes.c_double
        L.lexi_oracle_moe_layer.argtypes = [ctypes.POINTER(_Layer), vp, i32, i32, vp, i32, i32, i32, vp, vp, vp, vp,
                                            vp, vp, vp, vp]
        _lib = L
    return _lib


def num_threads() -> int:
    return int(lib().lexi_oracle_num_threads())


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data


class Layer:
    """One MoE layer's weights (numpy arrays kept alive here) in the oracle's struct."""

    def __init__(self, d: int, E: int, F: int, dtype: str, w_router, w_gate, w_up, w_down, router_bias=None,
                 F_shared: int = 0, shared_kind: int = 0, ws_gate=None, ws_up=None, ws_down=None,
                 w_shared_gate=None):
        wd = np.float32 if dtype == "f32" else np.uint16
        self.d, self.E, self.F, self.F_shared, self.dtype, self.shared_kind = d, E, F, F_shared, dtype, shared_kind

        def chk(a, shape, dt):
            if a is None:
                return None
            a = np.ascontiguousarray(a, dtype=dt)
            assert a.shape == tuple(shape), (a.shape, shape)
            return a

        self.w_router = chk(w_router, (d, E), np.float32)
        self.router_bias = chk(router_bias, (E,), np.float32)
        self.w_gate = chk(w_gate, (E, F, d), wd)
        self.w_up = chk(w_up, (E, F, d), wd)
        self.w_down = chk(w_down, (E, d, F), wd)
        self.ws_gate = chk(ws_gate, (F_shared, d), wd)
        self.ws_up = chk(ws_up, (F_shared, d), wd)
        self.ws_down = chk(ws_down, (d, F_shared), wd)
        self.w_shared_gate = chk(w_shared_gate, (d,), wd)
        self.c = _Layer(d, E, F, F_shared, 0 if dtype == "f32" else 1, shared_kind, _ptr(self.w_router),
                        _ptr(self.router_bias), _ptr(self.w_gate), _ptr(self.w_up), _ptr(self.w_down),
                        _ptr(self.ws_gate), _ptr(self.ws_up), _ptr(self.ws_down), _ptr(self.w_shared_gate))

    @classmethod
    def from_tensors(cls, cfg, tensors: Dict[str, Optional[np.ndarray]]) -> "Layer":
        """cfg: any object with d, E, F, F_shared, dtype, shared_kind; tensors: name -> array."""
        return cls(cfg.d, cfg.E, cfg.F, cfg.dtype, tensors["w_router"], tensors["w_gate"], tensors["w_up"],
                   tensors["w_down"], router_bias=tensors.get("router_bias"), F_shared=cfg.F_shared,
                   shared_kind=cfg.shared_kind, ws_gate=tensors.get("ws_gate"), ws_up=tensors.get("ws_up"),
                   ws_down=tensors.get("ws_down"), w_shared_gate=tensors.get("w_shared_gate"))

    def x_array(self, x) -> np.ndarray:
        x = np.ascontiguousarray(x, dtype=np.float32 if self.dtype == "f32" else np.uint16)
        assert x.ndim == 2 and x.shape[1] == self.d
        return x


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise RuntimeError(f"oracle {what} failed with code {rc}")


def router_logits(layer: Layer, x) -> np.ndarray:
    x = layer.x_array(x)
    out = np.empty((x.shape[0], layer.E), dtype=np.float32)
    _check(lib().lexi_oracle_router_logits(ctypes.byref(layer.c), x.ctypes.data, x.shape[0], out.ctypes.data), "router_logits")
    return out


def topk(logits: np.ndarray, k: int) -> np.ndarray:
    logits = np.ascontiguousarray(logits, dtype=np.float32)
    T, E = logits.shape
    out = np.empty((T, k), dtype=np.int32)
    _check(lib().lexi_oracle_topk(logits.ctypes.data, T, E, k, out.ctypes.data), "topk")
    return out


def gates(logits: np.ndarray, topk_idx: np.ndarray) -> np.ndarray:
    logits = np.ascontiguousarray(logits, dtype=np.float32)
    topk_idx = np.ascontiguousarray(topk_idx, dtype=np.int32)
    T, E = logits.shape
    k = topk_idx.shape[1]
    out = np.empty((T, k), dtype=np.float32)
    _check(lib().lexi_oracle_gates(logits.ctypes.data, topk_idx.ctypes.data, T, E, k, out.ctypes.data), "gates")
    return out


@dataclass
class Permutation:
    counts: np.ndarray
    offsets: np.ndarray
    perm: np.ndarray
    inv_perm: np.ndarray


def permutation(topk_idx: np.ndarray, E: int) -> Permutation:
    topk_idx = np.ascontiguousarray(topk_idx, dtype=np.int32)
    T, k = topk_idx.shape
    p = Permutation(np.empty(E, np.int32), np.empty(E + 1, np.int32), np.empty(T * k, np.int32), np.empty(T * k, np.int32))
    _check(lib().lexi_oracle_permutation(topk_idx.ctypes.data, T, E, k, p.counts.ctypes.data, p.offsets.ctypes.data,
                                         p.perm.ctypes.data, p.inv_perm.ctypes.data), "permutation")
    return p


def expert_ffn(layer: Layer, e: int, x, t: int, round_act: bool = False) -> np.ndarray:
    """fp64 output [d] of routed expert e (or the shared expert, e = -1, unscaled) on token row t."""
    x = layer.x_array(x)
    y = np.empty(layer.d, dtype=np.float64)
    _check(lib().lexi_oracle_expert_ffn(ctypes.byref(layer.c), e, x.ctypes.data, t, int(round_act), y.ctypes.data), "expert_ffn")
    return y


def shared_coeff(layer: Layer, x, t: int) -> float:
    x = layer.x_array(x)
    return float(lib().lexi_oracle_shared_coeff(ctypes.byref(layer.c), x.ctypes.data, t))


@dataclass
class LayerResult:
    out: Optional[np.ndarray]        # [n_tokens][d] fp64 (None when routing_only)
    logits: np.ndarray               # [T][E] fp32
    topk_idx: np.ndarray             # [T][k] int32
    gates: np.ndarray                # [T][k] fp32
    counts: np.ndarray
    offsets: np.ndarray
    perm: np.ndarray
    inv_perm: np.ndarray


def moe_layer(layer: Layer, x, k: int, tokens=None, round_act: bool = False, routing_only: bool = False) -> LayerResult:
    """f_moe(X; k) for one layer.  `tokens`: indices whose outputs are wanted (default all)."""
    x = layer.x_array(x)
    T, d, E = x.shape[0], layer.d, layer.E
    if not 1 <= k <= E:
        raise RuntimeError(f"oracle moe_layer: k={k} outside 1..E={E}")
    if tokens is None:
        tl, n = None, T
    else:
        tl = np.ascontiguousarray(tokens, dtype=np.int32)
        n = tl.shape[0]
    out = None if routing_only else np.empty((n, d), dtype=np.float64)
    r = LayerResult(out, np.empty((T, E), np.float32), np.empty((T, k), np.int32), np.empty((T, k), np.float32),
                    np.empty(E, np.int32), np.empty(E + 1, np.int32), np.empty(T * k, np.int32),
                    np.empty(T * k, np.int32))
    _check(lib().lexi_oracle_moe_layer(ctypes.byref(layer.c), x.ctypes.data, T, k, _ptr(tl), n, int(round_act),
                                       int(routing_only), _ptr(out), r.logits.ctypes.data, r.topk_idx.ctypes.data,
                                       r.gates.ctypes.data, r.counts.ctypes.data, r.offsets.ctypes.data,
                                       r.perm.ctypes.data, r.inv_perm.ctypes.data), "moe_layer")
    return r


def moe_stack(layers, xs, k_vec, tokens=None, round_act: bool = False, routing_only: bool = False):
    """Independent-input stack: layer l reads xs[l] (or the one x given) with k_vec[l]; returns a list of LayerResult."""
    res = []
    for l, ly in enumerate(layers):
        x = xs[l] if isinstance(xs, (list, tuple)) else xs
        res.append(moe_layer(ly, x, int(k_vec[l]), tokens=tokens, round_act=round_act, routing_only=routing_only))
    return res


def profile_layer(layer: Layer, x, k_base: int, k_list, round_act: bool = False) -> np.ndarray:
    """One iteration of the Stage-1 top-k perturbation profiling (paper Algorithm 1) on one input X:
    Y_base = f_moe(X; k_base), then for every k of the list Delta_k = || f_moe(X; k) - Y_base ||_F  (fp64).
    Taken in the algorithm's own order: the baseline pass first, then one full pass per target k; the average over
    iterations that the algorithm ends with is left to the caller."""
    y_base = moe_layer(layer, x, int(k_base), round_act=round_act).out
    deltas = np.empty(len(k_list), dtype=np.float64)
    for i, k in enumerate(k_list):
        y_k = moe_layer(layer, x, int(k), round_act=round_act).out
        deltas[i] = np.sqrt(np.sum((y_k - y_base) ** 2))
    return deltas


# ---------------------------------------------------------------- chained residual stack (pre-norm MoE blocks)
RMS_EPS = 1e-6


def bf16_rne(a: np.ndarray) -> np.ndarray:
    """Nearest-even rounding of float values to bf16, returned as uint16 bit patterns (finite inputs)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    u = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (u >> np.uint32(16)).astype(np.uint16)


def bf16_to_f64(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def rms_norm(h: np.ndarray) -> np.ndarray:
    """u = h / sqrt(mean_j(h_j^2) + eps) per token, fp64 (no learned scale)."""
    h = np.asarray(h, dtype=np.float64)
    return h / np.sqrt(np.mean(h * h, axis=1, keepdims=True) + RMS_EPS)


def chained_layer(layer: Layer, h, k: int, u_forced=None, round_act: bool = True):
    """One block of the chained stack: u = round_to_layer_dtype(rms_norm(h)), h' = h + f_moe(u; k).
    h: [T][d] fp64/fp32 hidden state.  u_forced: if given (bf16 bit patterns or fp32 values), it is used as the MoE
    input instead of the rounded normalisation (teacher forcing: lets a second implementation be checked block by
    block on bit-identical MoE inputs).  Returns (h', u, LayerResult)."""
    h = np.asarray(h, dtype=np.float64)
    if u_forced is not None:
        u = u_forced
    elif layer.dtype == "bf16":
        u = bf16_rne(rms_norm(h))
    else:
        u = rms_norm(h).astype(np.float32)
    res = moe_layer(layer, u, k, round_act=round_act and layer.dtype == "bf16")
    return h + res.out, u, res


def chained_stack(layers, x, k_vec, round_act: bool = True):
    """h_0 = x (widened exactly); h_{l+1} = h_l + f_moe_l(norm(h_l); k_l).  Returns the list [h_1 .. h_L] (fp64)."""
    h = bf16_to_f64(x) if layers[0].dtype == "bf16" else np.asarray(x, dtype=np.float64)
    hs = []
    for l, ly in enumerate(layers):
        h, _, _ = chained_layer(ly, h, int(k_vec[l]), round_act=round_act)
        hs.append(h)
    return hs
