"""The synthetic input generators: three implementations, one definition; workload table vs the paper's Table 1."""
import os

import numpy as np
import pytest

import lexi_synth as S
from lexi_synth import generator as G


def test_mix64_is_splitmix64():
    # SplitMix64 seeded with 0: the first outputs of the published generator (state += GOLDEN, then mix).
    state = np.uint64(0)
    outs = []
    with np.errstate(over="ignore"):
        for _ in range(3):
            state = state + G.GOLDEN
            outs.append(int(G.mix64(state)))
    assert outs == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]


@pytest.mark.parametrize("dtype,sigma", [("f32", 1.0), ("bf16", 0.02), ("bf16", 1.0)])
def test_host_c_equals_numpy(dtype, sigma):
    a = G.fill(S.C2.seed, 37, 50_000, sigma, dtype, start=12345)
    b = S.fill_host(S.C2.seed, 37, 50_000, sigma, dtype, start=12345)
    assert a.dtype == b.dtype and np.array_equal(a, b)


def test_counter_based_any_element_alone():
    full = S.fill_host(7, 3, 1000, 0.02, "bf16")
    for i in (0, 1, 511, 999):
        assert S.fill_host(7, 3, 1, 0.02, "bf16", start=i)[0] == full[i]


def test_distribution_moments():
    z = G.normal_f64(S.BASE_SEED if hasattr(S, "BASE_SEED") else G.BASE_SEED, 1, 0, 400_000)
    assert abs(z.mean()) < 0.01 and abs(z.std() - 1.0) < 0.01 and np.abs(z).max() < 6.0
    # Irwin-Hall(12) kurtosis is 3 - 0.1
    kurt = ((z - z.mean()) ** 4).mean() / z.var() ** 2
    assert abs(kurt - 2.9) < 0.05
    # distinct tensors are uncorrelated
    z2 = G.normal_f64(G.BASE_SEED, 2, 0, 400_000)
    assert abs(np.corrcoef(z, z2)[0, 1]) < 0.01


def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.00390625, 1.01171875, -1.00390625, 3.140625, 1e-3], dtype=np.float32)
    b = G.bf16_bits_to_f32(G.f32_to_bf16_bits(x))
    # 1 + 2^-8 is a tie between 1 and 1+2^-7 -> even (1.0); 1 + 3*2^-8 ties to 1+2^-6... (even mantissa)
    assert b[0] == 1.0 and b[1] == 1.0 and b[2] == 1.015625 and b[3] == -1.0
    assert np.all(np.abs(b - x) <= np.abs(x) * 2.0 ** -8)


def test_k_vectors_respect_budget_and_bounds():
    for cfg in (S.C2, S.C3, S.C4, S.C5):
        k = cfg.k_lexi()
        assert k.shape == (cfg.L,) and int(k.sum()) == cfg.budget
        assert k.min() >= cfg.k_min and k.max() <= cfg.k_max
        assert np.array_equal(k, cfg.k_lexi())  # seeded: same every call
        assert int(cfg.k_uniform().sum()) == cfg.L * cfg.k_base
    assert list(S.C4.k_lexi()) == [1] * 16 + [2] * 16
    assert len(set(S.C2.k_lexi().tolist())) > 2  # really layer-adaptive, not flat


def test_zipf_bias():
    b = S.zipf_router_bias(S.C5.seed, 0, 64, 1.1)
    assert b.dtype == np.float32 and b.shape == (64,)
    expect = np.sort(-1.1 * np.log(np.arange(1, 65)))
    assert np.allclose(np.sort(b), expect, rtol=1e-6)
    assert not np.array_equal(b, S.zipf_router_bias(S.C5.seed, 1, 64, 1.1))


def test_workloads_match_paper_table1():
    rows = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "table1_models.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            name, _p, layers, experts, topk, ffn, budgets = [s.strip() for s in line.split("|")]
            rows[name] = (int(layers), int(experts), int(topk), int(ffn), [int(b) for b in budgets.split()])
    olmoe, qwen, dsv2, mixtral = (rows["OLMoE-1B-7B-0125-Instruct"], rows["Qwen1.5-MoE-A2.7B-Chat"],
                                  rows["DeepSeek-V2-Lite-Chat"], rows["Mixtral-8x7B-Instruct-v0.1"])
    assert (S.C2.L, S.C2.E, S.C2.k_base, S.C2.F) == olmoe[:4]
    assert (S.C3.L, S.C3.E, S.C3.k_base, S.C3.F) == qwen[:4] and S.C3.budget in qwen[4]
    assert (S.C4.L, S.C4.E, S.C4.k_base, S.C4.F) == mixtral[:4] and S.C4.budget in mixtral[4]
    # DeepSeek-V2-Lite: 27 layers of which the first is dense -> 26 MoE layers (its budgets are multiples of 26)
    assert (S.C5.L + 1, S.C5.E, S.C5.k_base, S.C5.F) == dsv2[:4] and S.C5.budget in dsv2[4]
    assert all(b % 26 == 0 for b in dsv2[4])


def test_layer_tensor_shapes():
    cfg = S.mini(S.C3, L=1, d=128, F=64)
    t = S.host_layer(cfg, 0)
    assert t["w_router"].shape == (128, 60) and t["w_router"].dtype == np.float32
    assert t["w_gate"].shape == (60, 64, 128) and t["w_gate"].dtype == np.uint16
    assert t["w_down"].shape == (60, 128, 64)
    assert t["ws_gate"].shape == (128, 128) and t["ws_down"].shape == (128, 128) and t["w_shared_gate"].shape == (128,)
    assert t["router_bias"] is None
    assert S.host_x(cfg, 0, 5).shape == (5, 128)


@pytest.mark.gpu
def test_device_fill_equals_host():
    import torch
    for dtype, tdt in (("f32", torch.float32), ("bf16", torch.bfloat16)):
        n = 1_000_003
        t = torch.empty(n, dtype=tdt, device="cuda:0")
        S.fill_device(t, S.C4.seed, 99, 0.02, start=5)
        torch.cuda.synchronize()
        h = S.fill_host(S.C4.seed, 99, n, 0.02, dtype, start=5)
        if dtype == "f32":
            assert np.array_equal(t.cpu().numpy(), h)
        else:
            assert np.array_equal(t.view(torch.int16).cpu().numpy().view(np.uint16), h)
