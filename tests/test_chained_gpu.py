"""Chained residual stack (pre-norm MoE blocks, hidden state in fp32) on the GPU against the oracle.

A chain amplifies the one legitimate difference between two implementations: the normalised input is rounded to bf16,
so a last-bit difference in the fp32 normalisation can flip a rounding, and a flipped rounding can flip a near-tied
routing decision further down.  The tests therefore check each block on the inputs the GPU really used (teacher
forcing: the oracle block is fed the GPU's hidden state and the GPU's rounded normalisation), which keeps routing
comparable bit for bit, and check the normalisation itself separately against its definition.
"""
from dataclasses import replace

import numpy as np
import pytest

import lexi_synth as S
import oracle as O
from helpers import TOL_BF16, TOL_F32, check_routing, device_and_host_layer, rel_err, to_numpy

pytestmark = pytest.mark.gpu


def _run_chain(cfg, T, kv, per_layer=True, with_inputs=True):
    import torch
    import paper_2509_02753_amd as P
    pairs = [device_and_host_layer(cfg, l) for l in range(cfg.L)]
    dls = [p[0] for p in pairs]
    x = S.device_x(cfg, 0, T)
    tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    y = torch.empty((cfg.L, T, cfg.d) if per_layer else (T, cfg.d), dtype=torch.float32, device="cuda:0")
    ws = P.alloc_workspace(dls, T, int(kv.max()))
    ws.fill_(0x7F)
    routs = None
    if with_inputs:
        routs = [P.RoutingOut(T, int(kv[l]), cfg.E,
                              moe_input=torch.empty((T, cfg.d), dtype=tdt, device="cuda:0")) for l in range(cfg.L)]
    P.lexi_moe_stack_forward(dls, kv, x, y, ws, routing=routs, chained=True)
    torch.cuda.synchronize()
    return pairs, x, y, routs


def _check_blocks(cfg, T, kv):
    pairs, x, y, routs = _run_chain(cfg, T, kv)
    bf = cfg.dtype == "bf16"
    h_in = O.bf16_to_f64(to_numpy(x)) if bf else to_numpy(x).astype(np.float64)
    worst = 0.0
    for l in range(cfg.L):
        u_gpu = to_numpy(routs[l].moe_input)
        # the normalisation against its definition, computed from the hidden state the GPU block read
        if bf:
            u_def = O.bf16_rne(O.rms_norm(h_in))
            diff = np.abs(u_gpu.astype(np.int32) - u_def.astype(np.int32))   # same sign unless 0: adjacent patterns
            assert diff.max() <= 1, f"layer {l}: normalised input off by more than one bf16 step"
            assert np.mean(diff != 0) <= 0.01, f"layer {l}: {np.mean(diff != 0):.3%} of the roundings differ"
        else:
            assert rel_err(u_gpu, O.rms_norm(h_in)) <= 1e-6
        # the block itself on bit-identical inputs
        h_ref, _, res = O.chained_layer(pairs[l][1], h_in, int(kv[l]), u_forced=u_gpu)
        check_routing(routs[l], res)
        h_out = y[l].cpu().numpy().astype(np.float64)
        # the residual add is one fp32 addition (at most half an ulp of the result away from the exact sum); the rest
        # of the difference is the block's own error, measured against the RMS of the block's output as elsewhere
        rms = float(np.sqrt(np.mean(res.out ** 2)))
        err = max(0.0, float(np.abs(h_out - h_ref).max()) - 2.0 ** -24 * float(np.abs(h_ref).max())) / rms
        worst = max(worst, err)
        tol = TOL_BF16 if bf else TOL_F32
        assert err <= tol, f"layer {l}: block output error {err:.3e}"
        h_in = h_out
    return worst


@pytest.mark.parametrize("base,T", [("C2", 150), ("C3", 200), ("C5", 150), ("C5", 1), ("C4", 300)])
def test_each_block_matches_the_oracle_on_the_inputs_it_used(base, T):
    cfg = S.mini(getattr(S, base), L=4, d=256, F=384)
    _check_blocks(cfg, T, cfg.k_lexi())


def test_fp32_chain_matches_the_free_running_oracle():
    """fp32 layers have no rounding of the normalised input to flip: the whole chain agrees with the oracle's own."""
    cfg = replace(S.C1, name="c1_chain", L=3, budget=6)
    T = 97
    kv = cfg.k_lexi()
    _check_blocks(cfg, T, kv)
    pairs, x, y, _ = _run_chain(cfg, T, kv, with_inputs=False)
    hs = O.chained_stack([p[1] for p in pairs], to_numpy(x), kv)
    for l in range(cfg.L):
        assert rel_err(y[l].cpu().numpy(), hs[l]) <= 1e-5


def test_bf16_chain_stays_close_to_the_free_running_oracle():
    """Free-running comparison over 4 bf16 blocks: differences come only from rounding flips of the normalised input
    (and what they do to near-tied routing), so almost every token stays within the single-block tolerance."""
    cfg = S.mini(S.C2, L=4, d=256, F=384)
    T = 256
    kv = cfg.k_lexi()
    pairs, x, y, _ = _run_chain(cfg, T, kv, with_inputs=False)
    hs = O.chained_stack([p[1] for p in pairs], to_numpy(x), kv)
    ref = hs[-1]
    got = y[-1].cpu().numpy().astype(np.float64)
    per_token = np.abs(got - ref).max(axis=1) / np.sqrt(np.mean(ref * ref))
    assert np.median(per_token) <= TOL_BF16
    assert np.mean(per_token > 2 * TOL_BF16) <= 0.05, f"{np.mean(per_token > 2 * TOL_BF16):.2%} of tokens drifted"


def test_in_place_chain_and_reported_inputs():
    import torch
    import paper_2509_02753_amd as P
    cfg = S.mini(S.C5, L=3, d=256, F=384)
    T = 70
    kv = cfg.k_lexi()
    pairs, x, y, routs = _run_chain(cfg, T, kv)
    # stride 0: every block updates the one hidden-state buffer in place; the result is the last per-layer state
    _, _, y1, _ = _run_chain(cfg, T, kv, per_layer=False, with_inputs=False)
    assert torch.equal(y1, y[-1])
    # without the debugging outputs the normalised input lives in the workspace: same result
    _, _, y2, _ = _run_chain(cfg, T, kv, with_inputs=False)
    assert torch.equal(y2, y)
    # independent mode reports the input it was given
    dl = pairs[0][0]
    ws = P.alloc_workspace([dl], T, int(kv[0]))
    r = P.RoutingOut(T, int(kv[0]), cfg.E, moe_input=torch.zeros_like(x))
    yo = torch.empty((T, cfg.d), dtype=torch.float32, device="cuda:0")
    P.lexi_moe_layer_forward(dl, x, yo, int(kv[0]), ws, routing=r)
    torch.cuda.synchronize()
    assert torch.equal(r.moe_input, x)


def test_chained_mode_rejects_what_it_cannot_run():
    import torch
    import paper_2509_02753_amd as P
    cfg = S.mini(S.C5, L=2, d=256, F=384)
    T = 8
    kv = cfg.k_lexi()
    dls = [device_and_host_layer(cfg, l)[0] for l in range(cfg.L)]
    ws = P.alloc_workspace(dls, T, int(kv.max()))
    x = S.device_x(cfg, 0, T)
    with pytest.raises(RuntimeError):      # bf16 hidden state
        P.lexi_moe_stack_forward(dls, kv, x, torch.empty((cfg.L, T, cfg.d), dtype=torch.bfloat16, device="cuda:0"), ws,
                                 chained=True)
    with pytest.raises(RuntimeError):      # one input per layer
        P.lexi_moe_stack_forward(dls, kv, torch.stack([x, x]),
                                 torch.empty((cfg.L, T, cfg.d), dtype=torch.float32, device="cuda:0"), ws, chained=True)


def test_chained_stack_replayed_from_a_hip_graph_matches_eager():
    """The whole chain (normalisation, routing, expert GEMMs, shared expert on its side stream, combine + residual of
    every block) captured once and replayed: every replay equals the eager result, with eager work in between."""
    import torch
    import paper_2509_02753_amd as P
    cfg = S.mini(S.C5, L=4, d=256, F=384)
    T = 12
    kv = cfg.k_lexi()
    dls = [device_and_host_layer(cfg, l)[0] for l in range(cfg.L)]
    x = S.device_x(cfg, 0, T)
    y_eager = torch.empty((T, cfg.d), dtype=torch.float32, device="cuda:0")
    y_graph = torch.empty_like(y_eager)
    ws = P.alloc_workspace(dls, T, int(kv.max()))
    ws2 = P.alloc_workspace(dls, T, int(kv.max()))
    P.lexi_moe_stack_forward(dls, kv, x, y_eager, ws, chained=True)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        P.lexi_moe_stack_forward(dls, kv, x, y_graph, ws2, chained=True)
    for i in range(4):
        y_graph.fill_(float("nan"))
        ws2.fill_(0xFF)
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(y_graph, y_eager), f"replay {i} differs from the eager result"
        y_other = torch.empty_like(y_eager)
        P.lexi_moe_stack_forward(dls, kv, x, y_other, ws, chained=True)
        torch.cuda.synchronize()
        assert torch.equal(y_other, y_eager)


def test_chain_of_blocks_with_different_shapes():
    """Blocks that share only the hidden size and dtype (different expert counts, widths, shared-expert kinds, k): the
    normalised input handed from one block's combine to the next block must not depend on either block's layout."""
    import torch
    import paper_2509_02753_amd as P
    T, d = 75, 256
    shapes = [dict(E=64, F=320, F_shared=0, shared_kind=0, k=6, zipf_s=0.0),
              dict(E=5, F=64, F_shared=192, shared_kind=2, k=5, zipf_s=0.0),
              dict(E=40, F=576, F_shared=64, shared_kind=1, k=1, zipf_s=1.1)]
    cfgs = [replace(S.C2, name=f"hetc{i}", number=300 + i, L=len(shapes), d=d, E=s["E"], F=s["F"], F_shared=s["F_shared"],
                    shared_kind=s["shared_kind"], zipf_s=s["zipf_s"], k_base=s["k"], k_min=1, k_max=s["E"], budget=s["k"],
                    fixed_kvec=None) for i, s in enumerate(shapes)]
    kv = np.array([s["k"] for s in shapes], dtype=np.int32)
    pairs = [device_and_host_layer(cfgs[i], i) for i in range(len(shapes))]
    dls = [p[0] for p in pairs]
    x = S.device_x(cfgs[0], 0, T)
    ws = P.alloc_workspace(dls, T, int(kv.max()))
    ws.fill_(0x7F)
    y = torch.empty((len(shapes), T, d), dtype=torch.float32, device="cuda:0")
    routs = [P.RoutingOut(T, int(kv[i]), shapes[i]["E"],
                          moe_input=torch.empty((T, d), dtype=torch.bfloat16, device="cuda:0")) for i in range(len(shapes))]
    P.lexi_moe_stack_forward(dls, kv, x, y, ws, routing=routs, chained=True)
    torch.cuda.synchronize()
    h_in = O.bf16_to_f64(to_numpy(x))
    for i in range(len(shapes)):
        u_gpu = to_numpy(routs[i].moe_input)
        diff = np.abs(u_gpu.astype(np.int32) - O.bf16_rne(O.rms_norm(h_in)).astype(np.int32))
        assert diff.max() <= 1 and np.mean(diff != 0) <= 0.01
        h_ref, _, res = O.chained_layer(pairs[i][1], h_in, int(kv[i]), u_forced=u_gpu)
        check_routing(routs[i], res)
        h_out = y[i].cpu().numpy().astype(np.float64)
        rms = float(np.sqrt(np.mean(res.out ** 2)))
        assert (float(np.abs(h_out - h_ref).max()) - 2.0 ** -24 * float(np.abs(h_ref).max())) / rms <= TOL_BF16
        h_in = h_out
    # the same chain without the debugging outputs (normalised input in the workspace) and in place
    y2 = torch.empty((T, d), dtype=torch.float32, device="cuda:0")
    P.lexi_moe_stack_forward(dls, kv, x, y2, ws, chained=True)
    torch.cuda.synchronize()
    assert torch.equal(y2, y[-1])
