"""Shared pieces of the GPU parity tests: build the same seeded layer on host (oracle) and device (HIP path)."""
import numpy as np

import lexi_synth as S
import oracle as O

TOL_BF16 = 1e-2   # max|err| / RMS(ref), bf16 operands with fp32 accumulation
TOL_F32 = 1e-5    # fp32 layers
TOL_GATE = 1e-6   # absolute, gates are in [0, 1]


def to_numpy(t):
    import torch
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def device_and_host_layer(cfg, layer):
    """The HIP-side Layer, the oracle-side Layer, built from the same generator streams."""
    import paper_2509_02753_amd as P
    dev = S.device_layer(cfg, layer)
    host = S.host_layer(cfg, layer)
    return P.Layer.from_tensors(dev, shared_kind=cfg.shared_kind), O.Layer.from_tensors(cfg, host)


def rel_err(got, ref):
    """max |got - ref| / RMS(ref) over the whole array (fp64)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    rms = float(np.sqrt(np.mean(ref * ref)))
    return float(np.abs(got - ref).max()) / rms


def check_routing(r_gpu, r_ref):
    """Routing must agree bit for bit; gates to 1e-6."""
    assert np.array_equal(to_numpy(r_gpu.topk_idx), r_ref.topk_idx), "topk_idx differs"
    assert np.array_equal(to_numpy(r_gpu.counts), r_ref.counts), "counts differ"
    assert np.array_equal(to_numpy(r_gpu.offsets), r_ref.offsets), "offsets differ"
    assert np.array_equal(to_numpy(r_gpu.perm), r_ref.perm), "perm differs"
    assert np.array_equal(to_numpy(r_gpu.inv_perm), r_ref.inv_perm), "inv_perm differs"
    g = to_numpy(r_gpu.gates)
    assert np.abs(g - r_ref.gates).max() <= TOL_GATE, "gates differ"
    assert np.abs(g.astype(np.float64).sum(1) - 1.0).max() <= 1e-5


def run_and_check_layer(cfg, layer, T, k, tokens=None, check_bf16_out=True):
    """One layer on the GPU through the C ABI vs the oracle.  Returns the output error."""
    import torch
    import paper_2509_02753_amd as P
    dl, hl = device_and_host_layer(cfg, layer)
    xd = S.device_x(cfg, layer, T)
    xh = S.host_x(cfg, layer, T)
    ws = P.alloc_workspace([dl], T, k)
    y = torch.empty((T, cfg.d), dtype=torch.float32, device="cuda:0")
    rout = P.RoutingOut(T, k, cfg.E)
    P.lexi_moe_layer_forward(dl, xd, y, k, ws, routing=rout)
    torch.cuda.synchronize()
    ref = O.moe_layer(hl, xh, k, tokens=tokens, round_act=True)
    check_routing(rout, ref)
    yg = y.cpu().numpy()
    if tokens is not None:
        yg = yg[np.asarray(tokens)]
    err = rel_err(yg, ref.out)
    tol = TOL_F32 if cfg.dtype == "f32" else TOL_BF16
    assert err <= tol, f"output error {err:.3e} > {tol:.0e}"
    if check_bf16_out:
        yb = torch.empty((T, cfg.d), dtype=torch.bfloat16, device="cuda:0")
        P.lexi_moe_layer_forward(dl, xd, yb, k, ws)
        torch.cuda.synchronize()
        assert torch.equal(yb, y.to(torch.bfloat16)), "bf16 output is not the nearest-even rounding of the fp32 output"
    return err
