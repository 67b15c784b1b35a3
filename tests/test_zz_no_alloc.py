"""The entry point that allocates nothing (scratch in a static device array inside the library) against the entry point
that takes a caller-provided workspace: same kernels, so the outputs and the routing must agree bit for bit.  Two calls
in a row, the second on a smaller input, so stale scratch contents of the first call are exercised."""
import ctypes

import numpy as np
import pytest

import lexi_synth as S
from helpers import device_and_host_layer, to_numpy

pytestmark = pytest.mark.gpu


def _both(cfg, dl, T, k, y_dtype):
    import torch
    import paper_2509_02753_amd as P
    x = S.device_x(cfg, 0, T)
    y_ws = torch.empty((T, cfg.d), dtype=y_dtype, device="cuda:0")
    r_ws = P.RoutingOut(T, k, cfg.E)
    P.lexi_moe_layer_forward(dl, x, y_ws, k, P.alloc_workspace([dl], T, k), routing=r_ws)
    y_st = torch.full((T, cfg.d), 7.0, dtype=y_dtype, device="cuda:0")
    r_st = P.RoutingOut(T, k, cfg.E)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    P.lexi_moe_layer_forward_static(dl, x, y_st, k, routing=r_st)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    assert torch.equal(y_ws, y_st), f"T={T} k={k}: outputs differ"
    for name in ("topk_idx", "gates", "counts", "offsets", "perm", "inv_perm"):
        assert np.array_equal(to_numpy(getattr(r_ws, name)), to_numpy(getattr(r_st, name))), name


@pytest.mark.parametrize("name", ["c5_dsv2lite", "c3_qwen15", "c2_olmoe"])
def test_static_scratch_entry_point_matches_the_workspace_entry_point(name):
    import torch
    cfg = S.mini(S.CONFIGS[name], L=1, d=256, F=384)
    dl, _ = device_and_host_layer(cfg, 0)
    for T, k in ((300, 4), (33, 2), (1, 3), (700, 1)):      # a larger call, then smaller ones, then a larger one again
        _both(cfg, dl, T, k, torch.float32)
    _both(cfg, dl, 64, 4, torch.bfloat16)


def test_static_scratch_entry_point_against_the_oracle():
    import torch
    import oracle as O
    import paper_2509_02753_amd as P
    from helpers import TOL_BF16, check_routing, rel_err
    cfg = S.mini(S.C5, L=1, d=256, F=384)
    dl, hl = device_and_host_layer(cfg, 0)
    for T, k in ((256, 6), (16, 4)):
        y = torch.empty((T, cfg.d), dtype=torch.float32, device="cuda:0")
        rout = P.RoutingOut(T, k, cfg.E)
        P.lexi_moe_layer_forward_static(dl, S.device_x(cfg, 0, T), y, k, routing=rout)
        torch.cuda.synchronize()
        ref = O.moe_layer(hl, S.host_x(cfg, 0, T), k, round_act=True)
        check_routing(rout, ref)
        assert rel_err(y.cpu().numpy(), ref.out) <= TOL_BF16


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    """A prefill-sized call needs more than the 64 MiB array: LEXI_ERR_WORKSPACE, nothing launched, y untouched."""
    import torch
    import paper_2509_02753_amd as P
    cfg = S.mini(S.C2, L=1, d=2048, F=1024)
    dl, _ = device_and_host_layer(cfg, 0)
    T, k = 4096, 8
    assert P.lexi_moe_workspace_bytes([dl], T, k) > (64 << 20)
    x = S.device_x(cfg, 0, T)
    y = torch.full((T, cfg.d), 3.0, dtype=torch.float32, device="cuda:0")
    with pytest.raises(P.LexiError) as ei:
        P.lexi_moe_layer_forward_static(dl, x, y, k)
    assert ei.value.status == -5
    torch.cuda.synchronize()
    assert bool((y == 3.0).all())
    # the same layer at a decode-sized batch fits and still works after the rejected call
    T = 32
    ya = torch.empty((T, cfg.d), dtype=torch.float32, device="cuda:0")
    yb = torch.empty_like(ya)
    xs = S.device_x(cfg, 0, T)
    P.lexi_moe_layer_forward(dl, xs, ya, k, P.alloc_workspace([dl], T, k))
    P.lexi_moe_layer_forward_static(dl, xs, yb, k)
    torch.cuda.synchronize()
    assert torch.equal(ya, yb)
