"""Seeded synthetic inputs for the MoE-layer workloads (no MoE arithmetic in here).

Three bit-identical implementations of one counter-based generator:
``generator`` (numpy, the readable definition), ``csrc/synth_host.c`` (fast
host fill, OpenMP) and ``csrc/synth_device.hip`` (fill directly in HBM).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Dict, Optional

import numpy as np

from . import generator
from .configs import (C1, C2, C3, C4, C5, C6, C7, CONFIGS, SHARED_NONE, SHARED_SIGMOID, SHARED_UNGATED, MoEConfig, mini, pruned)
from .generator import (KIND_W_DOWN, KIND_W_GATE, KIND_W_ROUTER, KIND_W_SHARED_GATE, KIND_W_UP, KIND_WS_DOWN,
                        KIND_WS_GATE, KIND_WS_UP, KIND_X, tensor_id, zipf_router_bias)

_HERE = os.path.dirname(os.path.abspath(__file__))
HOST_LIB = os.path.join(_HERE, "libsynth_host.so")
DEVICE_LIB = os.path.join(_HERE, "libsynth_device.so")
HIP_FLAGS = ["--offload-arch=gfx950", "-O3", "-fPIC", "-shared", "-Xclang", "-target-feature", "-Xclang",
             "-packed-fp32-ops"]


def build(device: bool = True) -> None:
    """Compile the host (gcc) and device (hipcc, gfx950) generator libraries in-tree."""
    subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-o", HOST_LIB,
                           os.path.join(_HERE, "csrc", "synth_host.c")])
    if device:
        subprocess.check_call(["hipcc", *HIP_FLAGS, "-o", DEVICE_LIB, os.path.join(_HERE, "csrc", "synth_device.hip")])


_host = None
_device = None


def _host_lib():
    global _host
    if _host is None:
        if not os.path.exists(HOST_LIB):
            build(device=False)
        lib = ctypes.CDLL(HOST_LIB)
        lib.lexi_synth_fill_host.restype = ctypes.c_int
        lib.lexi_synth_fill_host.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_uint64, ctypes.c_uint64,
                                             ctypes.c_uint64, ctypes.c_uint64, ctypes.c_double]
        _host = lib
    return _host


def _device_lib():
    global _device
    if _device is None:
        if not os.path.exists(DEVICE_LIB):
            raise RuntimeError(f"{DEVICE_LIB} is not built; run lexi_synth.build()")
        lib = ctypes.CDLL(DEVICE_LIB)
        lib.lexi_synth_fill_device.restype = ctypes.c_int
        lib.lexi_synth_fill_device.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_uint64, ctypes.c_uint64,
                                               ctypes.c_uint64, ctypes.c_uint64, ctypes.c_double, ctypes.c_void_p]
        _device = lib
    return _device


def fill_host(seed: int, tid: int, count: int, sigma: float, dtype: str, start: int = 0) -> np.ndarray:
    """Fast host fill: float32 array ('f32') or uint16 bf16 bit patterns ('bf16')."""
    out = np.empty(count, dtype=np.float32 if dtype == "f32" else np.uint16)
    rc = _host_lib().lexi_synth_fill_host(out.ctypes.data, 0 if dtype == "f32" else 1, seed, tid, start, count,
                                          float(sigma))
    if rc != 0:
        raise RuntimeError("lexi_synth_fill_host failed")
    return out


def fill_device(tensor, seed: int, tid: int, sigma: float, start: int = 0) -> None:
    """Fill a contiguous torch CUDA tensor (float32 or bfloat16) in place on the current stream."""
    import torch
    assert tensor.is_cuda and tensor.is_contiguous()
    if tensor.dtype == torch.float32:
        dt = 0
    elif tensor.dtype == torch.bfloat16:
        dt = 1
    else:
        raise ValueError("fill_device: float32 or bfloat16 only")
    stream = torch.cuda.current_stream(tensor.device).cuda_stream
    rc = _device_lib().lexi_synth_fill_device(tensor.data_ptr(), dt, seed, tid, start, tensor.numel(), float(sigma),
                                              ctypes.c_void_p(stream))
    if rc != 0:
        raise RuntimeError(f"lexi_synth_fill_device failed ({rc})")


# ---------------------------------------------------------------------------
# Tensor sets.  Layouts (row-major, last index contiguous):
#   x [T][d];  w_router [d][E] fp32;  router_bias [E] fp32 or None
#   w_gate, w_up [E][F][d];  w_down [E][d][F]      (one row = one output feature's input weights)
#   ws_gate, ws_up [Fs][d];  ws_down [d][Fs];  w_shared_gate [d]
# ---------------------------------------------------------------------------

def layer_shapes(cfg: MoEConfig) -> Dict[str, tuple]:
    shp = {
        "w_router": (KIND_W_ROUTER, (cfg.d, cfg.E), "f32"),
        "w_gate": (KIND_W_GATE, (cfg.E, cfg.F, cfg.d), cfg.dtype),
        "w_up": (KIND_W_UP, (cfg.E, cfg.F, cfg.d), cfg.dtype),
        "w_down": (KIND_W_DOWN, (cfg.E, cfg.d, cfg.F), cfg.dtype),
    }
    if cfg.F_shared:
        shp["ws_gate"] = (KIND_WS_GATE, (cfg.F_shared, cfg.d), cfg.dtype)
        shp["ws_up"] = (KIND_WS_UP, (cfg.F_shared, cfg.d), cfg.dtype)
        shp["ws_down"] = (KIND_WS_DOWN, (cfg.d, cfg.F_shared), cfg.dtype)
        if cfg.shared_kind == SHARED_SIGMOID:
            shp["w_shared_gate"] = (KIND_W_SHARED_GATE, (cfg.d,), cfg.dtype)
    return shp


def host_layer(cfg: MoEConfig, layer: int) -> Dict[str, Optional[np.ndarray]]:
    """All weight tensors of one layer as numpy arrays (bf16 as uint16 bit patterns)."""
    out: Dict[str, Optional[np.ndarray]] = {}
    for name, (kind, shape, dt) in layer_shapes(cfg).items():
        n = int(np.prod(shape))
        out[name] = fill_host(cfg.seed, tensor_id(layer, kind), n, cfg.sigma_w, dt).reshape(shape)
    out["router_bias"] = zipf_router_bias(cfg.seed, layer, cfg.E, cfg.zipf_s) if cfg.zipf_s > 0 else None
    return out


def host_x(cfg: MoEConfig, layer: int, T: int) -> np.ndarray:
    return fill_host(cfg.seed, tensor_id(layer, KIND_X), T * cfg.d, cfg.sigma_x, cfg.dtype).reshape(T, cfg.d)


def device_layer(cfg: MoEConfig, layer: int, device="cuda:0"):
    """Same tensors as host_layer, generated directly in HBM as torch tensors."""
    import torch
    out = {}
    for name, (kind, shape, dt) in layer_shapes(cfg).items():
        t = torch.empty(shape, dtype=torch.float32 if dt == "f32" else torch.bfloat16, device=device)
        fill_device(t, cfg.seed, tensor_id(layer, kind), cfg.sigma_w)
        out[name] = t
    out["router_bias"] = (torch.from_numpy(zipf_router_bias(cfg.seed, layer, cfg.E, cfg.zipf_s)).to(device)
                          if cfg.zipf_s > 0 else None)
    return out


def device_x(cfg: MoEConfig, layer: int, T: int, device="cuda:0"):
    import torch
    t = torch.empty((T, cfg.d), dtype=torch.float32 if cfg.dtype == "f32" else torch.bfloat16, device=device)
    fill_device(t, cfg.seed, tensor_id(layer, KIND_X), cfg.sigma_x)
    return t
