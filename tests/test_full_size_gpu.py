"""Full-size workloads in the launch configuration the benchmark times: the whole L-layer stack at the workload's
real shapes and token counts through lexi_moe_stack_forward with its per-layer k vector.

Routing (selected experts, gates, counts, offsets, permutation) is compared with the oracle for EVERY token of EVERY
layer run.  Outputs are compared on sampled tokens, which the oracle computes one by one, on three layers (first,
middle, last); those layers' weights are regenerated on the host from the same seeded streams.
"""
import numpy as np
import pytest

import lexi_synth as S
import oracle as O
from helpers import TOL_BF16, check_routing, rel_err

pytestmark = pytest.mark.gpu

N_SAMPLE = 20   # tokens per checked layer whose outputs the oracle computes


def _sample_tokens(T, seed):
    rng = np.random.default_rng(seed)
    fixed = [0, T - 1, T // 2]
    extra = rng.choice(T, size=min(T, N_SAMPLE), replace=False).tolist()
    return np.array(sorted(set(fixed + extra)), dtype=np.int32)


_STACK = {}   # name -> (layer ids, device layers, host layers of the output-checked ones): one workload resident at a time


def _progress(msg):
    """Progress lines for long runs: printed (visible with -s) and appended to gpurun_out/ when that folder exists."""
    import os
    print(msg, flush=True)
    d = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "gpurun_out")
    if os.path.isdir(d):
        with open(os.path.join(d, "test_full_size_progress.log"), "a") as f:
            f.write(msg + "\n")


def _stack(cfg, layer_ids):
    import torch
    import paper_2509_02753_amd as P
    key = (cfg.name, tuple(layer_ids))
    if key not in _STACK:
        _STACK.clear()
        torch.cuda.empty_cache()
        layers = []
        for i, l in enumerate(layer_ids):
            if i % 4 == 0:
                _progress(f"[full-size] {cfg.name}: device weights of layer {l} ({i + 1}/{len(layer_ids)})")
            rm = S.device_layer(cfg, l, "cuda:0")
            layers.append(P.Layer.from_tensors(rm, shared_kind=cfg.shared_kind))
            del rm
        torch.cuda.synchronize()
        ffn_pos = sorted({0, len(layer_ids) // 2, len(layer_ids) - 1})
        host = {}
        for i in ffn_pos:
            _progress(f"[full-size] {cfg.name}: host weights of layer {layer_ids[i]}")
            host[i] = O.Layer.from_tensors(cfg, S.host_layer(cfg, layer_ids[i]))
        _STACK[key] = (layers, host)
    return _STACK[key]


def _check_stack(cfg, T, layer_ids=None):
    import torch
    import paper_2509_02753_amd as P
    layer_ids = list(range(cfg.L)) if layer_ids is None else list(layer_ids)
    kfull = cfg.k_lexi()
    assert kfull.shape == (cfg.L,) and int(kfull.sum()) == cfg.budget
    kvec = kfull[layer_ids].copy()
    layers, host = _stack(cfg, layer_ids)
    n = len(layer_ids)
    x = torch.empty((n, T, cfg.d), dtype=torch.bfloat16, device="cuda:0")
    for i, l in enumerate(layer_ids):
        S.fill_device(x[i], cfg.seed, S.tensor_id(l, S.KIND_X), cfg.sigma_x)
    y = torch.empty((n, T, cfg.d), dtype=torch.float32, device="cuda:0")
    ws = P.alloc_workspace(layers, T, int(kvec.max()))
    routs = [P.RoutingOut(T, int(kvec[i]), cfg.E) for i in range(n)]
    ws.fill_(0x7F)
    P.lexi_moe_stack_forward(layers, kvec, x, y, ws, routing=routs)
    torch.cuda.synchronize()
    # a second pass without the routing outputs (the timed configuration) must reproduce the first bit for bit
    y2 = torch.empty_like(y)
    P.lexi_moe_stack_forward(layers, kvec, x, y2, ws)
    torch.cuda.synchronize()
    assert torch.equal(y, y2), "two passes over the same inputs differ"
    del y2
    worst = 0.0
    for i, l in enumerate(layer_ids):
        xh = S.host_x(cfg, l, T)
        k = int(kvec[i])
        if i in host:
            tok = _sample_tokens(T, 1000 * cfg.number + l)
            ref = O.moe_layer(host[i], xh, k, tokens=tok, round_act=True)
            check_routing(routs[i], ref)
            err = rel_err(y[i].cpu().numpy()[tok], ref.out)
            worst = max(worst, err)
            assert err <= TOL_BF16, f"layer {l}: output error {err:.3e}"
        else:
            # routing needs only the router weights and the bias: a layer object with empty expert tensors
            check_routing(routs[i], O.moe_layer(_routing_only_layer(cfg, l), xh, k, routing_only=True))
    _progress(f"[full-size] {cfg.name} T={T}: routing exact on {n} layers, worst sampled output error {worst:.2e}")


class _RoutingCfg:
    """Shape record for an oracle layer that is only asked for routing: one tiny expert row keeps the arrays valid."""
    def __init__(self, cfg):
        self.d, self.E, self.F, self.F_shared, self.dtype, self.shared_kind = cfg.d, cfg.E, 1, 0, cfg.dtype, 0


def _routing_only_layer(cfg, l):
    z = np.zeros((cfg.E, 1, cfg.d), dtype=np.uint16)
    tensors = {
        "w_router": S.fill_host(cfg.seed, S.tensor_id(l, S.KIND_W_ROUTER), cfg.d * cfg.E, cfg.sigma_w, "f32").reshape(cfg.d, cfg.E),
        "router_bias": S.zipf_router_bias(cfg.seed, l, cfg.E, cfg.zipf_s) if cfg.zipf_s > 0 else None,
        "w_gate": z, "w_up": z, "w_down": np.zeros((cfg.E, cfg.d, 1), dtype=np.uint16),
    }
    return O.Layer.from_tensors(_RoutingCfg(cfg), tensors)


def test_c2_olmoe_prefill_full_stack():
    _check_stack(S.C2, 4096)


@pytest.mark.parametrize("T", [8192, 64])
def test_c3_qwen15_full_stack(T):
    _check_stack(S.C3, T)


@pytest.mark.parametrize("T", [4096, 32])
def test_c4_mixtral_full_stack(T):
    """All 32 layers, 90 GB of expert weights resident in HBM."""
    _check_stack(S.C4, T)


@pytest.mark.parametrize("T", [1, 16, 64, 256])
def test_c5_dsv2lite_decode_full_stack(T):
    _check_stack(S.C5, T)
