"""HIP path vs CPU oracle, element by element, through the C ABI (needs an MI355X)."""
import numpy as np
import pytest

import lexi_synth as S
import oracle as O
from helpers import TOL_BF16, check_routing, device_and_host_layer, rel_err, run_and_check_layer, to_numpy

pytestmark = pytest.mark.gpu


def test_c1_plumbing_fp32_full_size():
    """Config 1 at its real size: T=64, d=128, E=8, F=256, k=2, everything fp32."""
    err = run_and_check_layer(S.C1, 0, 64, 2)
    assert err <= 1e-5


@pytest.mark.parametrize("name,T,k", [
    ("c2_olmoe", 300, 8), ("c2_olmoe", 300, 2), ("c2_olmoe", 1, 5), ("c2_olmoe", 129, 64),
    ("c3_qwen15", 700, 4), ("c3_qwen15", 64, 1), ("c3_qwen15", 37, 60),
    ("c4_mixtral", 700, 2), ("c4_mixtral", 32, 1), ("c4_mixtral", 513, 8),
    ("c5_dsv2lite", 1, 6), ("c5_dsv2lite", 16, 4), ("c5_dsv2lite", 256, 6), ("c5_dsv2lite", 1000, 2),
    # around the batch sizes where the routing path switches kernels
    ("c5_dsv2lite", 5, 6), ("c2_olmoe", 16, 64), ("c3_qwen15", 17, 4), ("c5_dsv2lite", 128, 3), ("c2_olmoe", 2047, 5),
    ("c2_olmoe", 2100, 3),
])
def test_mini_layers_all_tokens(name, T, k):
    """Scaled-down shapes (same E, k range, shared expert and bias as the workload), every token compared.
    Sizes span several token tiles, ragged tails, empty experts (Zipf bias) and k = 1 / k = E."""
    cfg = S.mini(S.CONFIGS[name], L=1, d=256, F=384)
    run_and_check_layer(cfg, 0, T, k)


@pytest.mark.parametrize("name,inter,intra,T,k", [
    ("c2_olmoe", 0.125, 0.0, 260, 8), ("c2_olmoe", 0.5, 0.0, 131, 3), ("c3_qwen15", 0.25, 0.0, 200, 4),
    ("c2_olmoe", 0.0, 0.125, 260, 8), ("c3_qwen15", 0.0, 0.5, 150, 2), ("c5_dsv2lite", 0.25, 0.25, 64, 6),
])
def test_pruned_shapes(name, inter, intra, T, k):
    """Shapes of the paper's comparison methods (Sec. 3): fewer experts (E not a power of two: 56, 45, 32, 48) and
    narrower expert FFNs (widths that are odd multiples of 64), every token compared."""
    base = S.mini(S.CONFIGS[name], L=1, d=256, F=512)
    cfg = S.pruned(base, inter=inter, intra=intra)
    assert (cfg.E, cfg.F) != (base.E, base.F)
    run_and_check_layer(cfg, 0, T, k)


@pytest.mark.parametrize("name,T,k", [("c6_minicpm", 160, 2), ("c6_minicpm", 20, 1), ("c7_vl2tiny", 300, 6), ("c7_vl2tiny", 9, 3)])
def test_remaining_table1_shapes_one_full_layer(name, T, k):
    """The two Table 1 shapes that are not benchmark workloads, at their real widths (hidden sizes that are not powers
    of two: 18 and 10 router segments, 9 and 5 down-GEMM column blocks), one layer, every token compared."""
    run_and_check_layer(S.CONFIGS[name], 0, T, k)


def test_repeated_calls_and_k_changes_leave_no_state():
    """UpdateTopk changes k only: k=2, then k=8, then k=2 again reproduces the first result bit for bit."""
    import torch
    import paper_2509_02753_amd as P
    cfg = S.mini(S.C2, L=1, d=256, F=384)
    dl, _ = device_and_host_layer(cfg, 0)
    x = S.device_x(cfg, 0, 333)
    ws = P.alloc_workspace([dl], 333, 8)
    ys = []
    for k in (2, 8, 2, 8):
        y = torch.empty((333, cfg.d), dtype=torch.float32, device="cuda:0")
        ws.fill_(0xFF)  # stale workspace contents must not matter
        P.lexi_moe_layer_forward(dl, x, y, k, ws)
        ys.append(y)
    torch.cuda.synchronize()
    assert torch.equal(ys[0], ys[2]) and torch.equal(ys[1], ys[3]) and not torch.equal(ys[0], ys[1])


def test_ties_go_to_the_lower_expert_on_device():
    """Duplicate router columns give bit-identical logits; the lower index must win on the GPU as in the oracle."""
    import torch
    import paper_2509_02753_amd as P
    cfg = S.mini(S.C2, L=1, d=256, F=128)
    dev, host = S.device_layer(cfg, 0), S.host_layer(cfg, 0)
    for a, b in ((7, 3), (40, 3), (63, 62)):
        host["w_router"][:, a] = host["w_router"][:, b]
    dev["w_router"] = torch.from_numpy(host["w_router"]).cuda()
    dl, hl = P.Layer.from_tensors(dev), O.Layer.from_tensors(cfg, host)
    T = 200
    xd, xh = S.device_x(cfg, 0, T), S.host_x(cfg, 0, T)
    for k in (1, 3, 8):
        rout = P.RoutingOut(T, k, cfg.E)
        y = torch.empty((T, cfg.d), dtype=torch.float32, device="cuda:0")
        P.lexi_moe_layer_forward(dl, xd, y, k, P.alloc_workspace([dl], T, k), routing=rout)
        torch.cuda.synchronize()
        check_routing(rout, O.moe_layer(hl, xh, k, routing_only=True))


def test_stack_with_per_layer_k_vector():
    """lexi_moe_stack_forward with k* = (k_1..k_L): each layer equals the oracle with its own k and its own X."""
    import torch
    import paper_2509_02753_amd as P
    cfg = S.mini(S.C5, L=4, d=256, F=384)
    T = 150
    kv = cfg.k_lexi()
    assert len(set(kv.tolist())) > 1
    pairs = [device_and_host_layer(cfg, l) for l in range(cfg.L)]
    dls = [p[0] for p in pairs]
    x = torch.stack([S.device_x(cfg, l, T) for l in range(cfg.L)])
    y = torch.empty((cfg.L, T, cfg.d), dtype=torch.float32, device="cuda:0")
    ws = P.alloc_workspace(dls, T, int(kv.max()))
    routs = [P.RoutingOut(T, int(kv[l]), cfg.E) for l in range(cfg.L)]
    P.lexi_moe_stack_forward(dls, kv, x, y, ws, routing=routs)
    torch.cuda.synchronize()
    for l in range(cfg.L):
        ref = O.moe_layer(pairs[l][1], S.host_x(cfg, l, T), int(kv[l]), round_act=True)
        check_routing(routs[l], ref)
        assert rel_err(y[l].cpu().numpy(), ref.out) <= TOL_BF16
    # same X for every layer (stride 0), as in per-layer profiling on one random input
    y2 = torch.empty_like(y)
    P.lexi_moe_stack_forward(dls, kv, x[0].contiguous(), y2, ws)
    y3 = torch.empty((T, cfg.d), dtype=torch.float32, device="cuda:0")
    P.lexi_moe_layer_forward(dls[2], x[0].contiguous(), y3, int(kv[2]), ws)
    torch.cuda.synchronize()
    assert torch.equal(y2[0], y[0]) and torch.equal(y2[2], y3)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_pack_weights_matches_the_documented_index(dtype):
    """lexi_pack_weights against the layout formula printed in the header, on matrices of distinct values."""
    import torch
    import paper_2509_02753_amd as P
    n, R, K = 3, 48, 96
    src = torch.arange(n * R * K, dtype=torch.float32).reshape(n, R, K) % 251   # exact in bf16
    src = src.to(torch.bfloat16 if dtype == "bf16" else torch.float32).cuda().contiguous()
    packed = P.lexi_pack_weights(src).float().cpu().numpy().reshape(n, R * K)
    ref = src.float().cpu().numpy()
    r, k = np.meshgrid(np.arange(R), np.arange(K), indexing="ij")
    idx = ((((r // 16) * (K // 32) + k // 32) * 64 + ((k % 32) // 8) * 16 + r % 16) * 8 + k % 8)
    assert np.array_equal(np.sort(idx.reshape(-1)), np.arange(R * K))           # the formula is a permutation
    for m in range(n):
        assert np.array_equal(packed[m][idx], ref[m])
    with pytest.raises(P.LexiError):
        P.lexi_pack_weights(torch.zeros((40, 96), dtype=torch.bfloat16, device="cuda"))   # rows % 16 != 0


@pytest.mark.parametrize("name,T", [
    ("c3_qwen15", 40),     # sigmoid-gated shared expert: the side stream is in the capture, joined before the combine
    ("c5_dsv2lite", 4),    # ungated shared expert, a handful of tokens: joined before the launch that holds down + combine
])
def test_stack_replayed_from_a_hip_graph_matches_eager(name, T):
    """A captured stack call (side-stream fork/join of the shared expert included) replays to the eager result,
    every time, with eager work and synchronisations between the replays."""
    import torch
    import paper_2509_02753_amd as P
    cfg = S.mini(S.CONFIGS[name], L=3, d=256, F=384)
    kv = cfg.k_lexi()
    dls = [device_and_host_layer(cfg, l)[0] for l in range(cfg.L)]
    x = torch.stack([S.device_x(cfg, l, T) for l in range(cfg.L)])
    y_eager = torch.empty((cfg.L, T, cfg.d), dtype=torch.float32, device="cuda:0")
    y_graph = torch.empty_like(y_eager)
    ws = P.alloc_workspace(dls, T, int(kv.max()))
    ws2 = P.alloc_workspace(dls, T, int(kv.max()))
    P.lexi_moe_stack_forward(dls, kv, x, y_eager, ws)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        P.lexi_moe_stack_forward(dls, kv, x, y_graph, ws2)
    for i in range(4):
        y_graph.fill_(float("nan"))
        ws2.fill_(0xFF)
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(y_graph, y_eager), f"replay {i} differs from the eager result"
        y_other = torch.empty_like(y_eager)
        P.lexi_moe_stack_forward(dls, kv, x, y_other, ws)     # eager work between the replays
        torch.cuda.synchronize()
        assert torch.equal(y_other, y_eager)


def _random_shape_cases(n, seed):
    """Seeded shapes inside the documented limits: d a multiple of 128, F and F_shared multiples of 64, 1 <= E <= 64,
    1 <= k <= E, any T; every routing path (T <= 16, <= 128, <= 1024, above) and every shared-expert kind appears."""
    rng = np.random.default_rng(seed)
    cases = []
    t_pool = [1, 2, 3, 7, 15, 16, 17, 31, 33, 64, 100, 127, 128, 129, 200, 257, 511, 700, 1023, 1024, 1025, 1500, 2049]
    for i in range(n):
        E = int(rng.choice([1, 2, 3, 5, 8, 13, 31, 32, 33, 48, 60, 63, 64]))
        d = 128 * int(rng.integers(1, 7))
        F = 64 * int(rng.integers(1, 9))
        kind = int(rng.integers(0, 3))
        Fs = 64 * int(rng.integers(1, 7)) if kind else 0
        T = int(t_pool[i % len(t_pool)])
        k = int(rng.integers(1, E + 1)) if i % 3 else min(E, int(rng.choice([1, 2, E])))
        zipf = 1.1 if rng.random() < 0.3 else 0.0
        dtype = "f32" if i % 7 == 6 else "bf16"
        cases.append((i, E, d, F, Fs, kind, T, k, zipf, dtype))
    return cases


@pytest.mark.parametrize("case", _random_shape_cases(46, 20250902), ids=lambda c: f"{c[0]}-E{c[1]}d{c[2]}F{c[3]}s{c[4]}T{c[6]}k{c[7]}{c[9]}")
def test_random_shapes_inside_the_limits(case):
    """Every token of one layer against the oracle on seeded random shapes: ragged column blocks (F, d not multiples
    of the 128/256-wide workgroup tiles), expert counts that are not powers of two, k anywhere in 1..E, empty experts
    under a Zipf bias, fp32 and bf16 layers, all three shared-expert kinds."""
    from dataclasses import replace
    i, E, d, F, Fs, kind, T, k, zipf, dtype = case
    cfg = replace(S.C2, name=f"rand{i}", number=100 + i, L=1, d=d, E=E, F=F, dtype=dtype, k_base=k, k_min=1, k_max=E,
                  budget=k, F_shared=Fs, shared_kind=kind, zipf_s=zipf, fixed_kvec=None)
    if T * k * F * 3 * d > 3e10:      # keep the fp64 oracle of one case to a few seconds
        T = max(1, int(3e10 / (k * F * 3 * d)))
    run_and_check_layer(cfg, 0, T, k, check_bf16_out=(i % 4 == 0))


def test_stack_of_layers_with_different_shapes():
    """One stack call over layers that share only the hidden size: different expert counts, FFN widths, shared-expert
    kinds and k; each layer must equal its own single-layer oracle result, and the workspace is sized for the largest."""
    import torch
    import paper_2509_02753_amd as P
    from dataclasses import replace
    T, d = 190, 384
    shapes = [dict(E=64, F=448, F_shared=0, shared_kind=0, k=7, zipf_s=0.0),
              dict(E=9, F=64, F_shared=320, shared_kind=2, k=9, zipf_s=0.0),
              dict(E=33, F=704, F_shared=128, shared_kind=1, k=1, zipf_s=1.1),
              dict(E=1, F=192, F_shared=0, shared_kind=0, k=1, zipf_s=0.0)]
    cfgs = [replace(S.C2, name=f"het{i}", number=200 + i, L=len(shapes), d=d, E=s["E"], F=s["F"], F_shared=s["F_shared"],
                    shared_kind=s["shared_kind"], zipf_s=s["zipf_s"], k_base=s["k"], k_min=1, k_max=s["E"], budget=s["k"],
                    fixed_kvec=None) for i, s in enumerate(shapes)]
    kv = np.array([s["k"] for s in shapes], dtype=np.int32)
    pairs = [device_and_host_layer(cfgs[i], i) for i in range(len(shapes))]
    dls = [p[0] for p in pairs]
    x = torch.stack([S.device_x(cfgs[i], i, T) for i in range(len(shapes))])
    y = torch.empty((len(shapes), T, d), dtype=torch.float32, device="cuda:0")
    ws = P.alloc_workspace(dls, T, int(kv.max()))
    assert ws.numel() >= max(P.lexi_moe_workspace_bytes([dl], T, int(k)) for dl, k in zip(dls, kv))
    routs = [P.RoutingOut(T, int(kv[i]), shapes[i]["E"]) for i in range(len(shapes))]
    ws.fill_(0x7F)
    P.lexi_moe_stack_forward(dls, kv, x, y, ws, routing=routs)
    torch.cuda.synchronize()
    for i in range(len(shapes)):
        ref = O.moe_layer(pairs[i][1], S.host_x(cfgs[i], i, T), int(kv[i]), round_act=True)
        check_routing(routs[i], ref)
        assert rel_err(y[i].cpu().numpy(), ref.out) <= TOL_BF16, f"layer {i}"


def test_two_host_threads_on_two_streams():
    """Two host threads drive the same layers on their own streams, workspaces and outputs (the shared expert's side
    stream and its events are shared by all callers of a device): every result equals the single-threaded one."""
    import threading
    import torch
    import paper_2509_02753_amd as P
    cfg = S.mini(S.C3, L=3, d=256, F=384)    # sigmoid-gated shared expert -> side stream in every layer
    T = 48
    kv = cfg.k_lexi()
    dls = [device_and_host_layer(cfg, l)[0] for l in range(cfg.L)]
    x = torch.stack([S.device_x(cfg, l, T) for l in range(cfg.L)])
    y_ref = torch.empty((cfg.L, T, cfg.d), dtype=torch.float32, device="cuda:0")
    P.lexi_moe_stack_forward(dls, kv, x, y_ref, P.alloc_workspace(dls, T, int(kv.max())))
    torch.cuda.synchronize()
    errors = []

    def worker(idx):
        try:
            stream = torch.cuda.Stream()
            ws = P.alloc_workspace(dls, T, int(kv.max()))
            ys = [torch.empty_like(y_ref) for _ in range(12)]
            with torch.cuda.stream(stream):
                for y in ys:
                    P.lexi_moe_stack_forward(dls, kv, x, y, ws, stream=stream)
            stream.synchronize()
            for i, y in enumerate(ys):
                if not torch.equal(y, y_ref):
                    errors.append(f"thread {idx}, call {i}: result differs")
        except Exception as e:  # noqa: BLE001  (reported through the list: exceptions do not cross threads)
            errors.append(f"thread {idx}: {e!r}")

    threads = [threading.Thread(target=worker, args=(i,)) for i in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join(timeout=100)
    assert not any(t.is_alive() for t in threads), "a worker did not finish"
    assert not errors, errors


def test_a_nan_activation_is_routed_safely():
    """Inputs are finite by contract; a NaN activation must nevertheless produce a valid routing (every index in
    range, perm a permutation) and NaN for that token only.  A row of NaN logits ranks every expert equal, so both
    sides select experts 0..k-1 for it; every other token matches the oracle as usual."""
    import torch
    import paper_2509_02753_amd as P
    cfg = S.mini(S.C2, L=1, d=256, F=128)
    dl, hl = device_and_host_layer(cfg, 0)
    for T, k, bad in ((200, 4, 17), (9, 3, 8), (2100, 2, 2099)):
        xh = S.host_x(cfg, 0, T).copy()
        xh[bad, 5] = 0x7FC0                      # bf16 quiet NaN
        xd = torch.from_numpy(xh.view(np.int16)).cuda().view(torch.bfloat16)
        y = torch.empty((T, cfg.d), dtype=torch.float32, device="cuda:0")
        rout = P.RoutingOut(T, k, cfg.E)
        P.lexi_moe_layer_forward(dl, xd, y, k, P.alloc_workspace([dl], T, k), routing=rout)
        torch.cuda.synchronize()
        idx, perm = to_numpy(rout.topk_idx), to_numpy(rout.perm)
        assert idx.min() >= 0 and idx.max() < cfg.E
        assert idx[bad].tolist() == list(range(k))
        assert np.array_equal(np.sort(perm), np.arange(T * k))
        ref = O.moe_layer(hl, xh, k, round_act=True)
        assert np.array_equal(idx, ref.topk_idx) and np.array_equal(perm, ref.perm)
        yg = y.cpu().numpy()
        assert np.isnan(yg[bad]).all()
        keep = np.arange(T) != bad
        assert np.isfinite(yg[keep]).all() and rel_err(yg[keep], ref.out[keep]) <= TOL_BF16


@pytest.mark.parametrize("name,d,F,F_shared,T,k,want_routed,want_shared", [
    ("c2_olmoe", 1024, 2048, 0, 1300, 2, 2, None),      # routed down GEMM on the tile schedule, reduction cut in two
    ("c2_olmoe", 1024, 2048, 0, 2600, 1, 3, None),      # one active expert: output rows stored by the down GEMM itself
    ("c2_olmoe", 1024, 1024, 0, 1300, 2, 1, None),      # same sizes, reduction too short to cut: one plane
    ("c3_qwen15", 1024, 384, 2048, 700, 3, 1, 2),       # shared expert's dense down GEMM cut in two
    ("c4_mixtral", 1024, 4096, 0, 3700, 2, 2, None),    # few experts, many rows each
])
def test_down_gemm_schedules(name, d, F, F_shared, T, k, want_routed, want_shared):
    """The down GEMM's launch variants at sizes where the tile schedule runs: split reduction (two partial planes added
    by the combine), direct output rows for k = 1, and the shared expert's split; outputs of sampled tokens against the
    oracle, routing of every token, and the bf16 output as the rounding of the fp32 output."""
    import paper_2509_02753_amd as P
    cfg = S.mini(S.CONFIGS[name], L=1, d=d, F=F, F_shared=F_shared)
    dl, _ = device_and_host_layer(cfg, 0)
    assert P.lexi_moe_down_plan(dl, T, k) == want_routed
    if want_shared is not None:
        assert P.lexi_moe_down_plan(dl, T, k, shared=True) == want_shared
    del dl
    rng = np.random.default_rng(T + k)
    tokens = np.unique(np.concatenate([[0, T - 1, T // 2], rng.integers(0, T, 93)])).astype(np.int32)
    run_and_check_layer(cfg, 0, T, k, tokens=tokens)


@pytest.mark.parametrize("name,T,k,want", [
    ("c4_mixtral", 1, 1, 4),     # one expert with rows: its reduction is dealt out over all sixteen waves
    ("c4_mixtral", 1, 2, 4),     # two experts
    ("c2_olmoe", 1, 3, 4), ("c2_olmoe", 2, 4, 4), ("c2_olmoe", 3, 5, 4),   # 3, up to 8, nine or more experts per pass
    ("c5_dsv2lite", 8, 6, 4),    # more experts than one pass holds, ungated shared expert added in the same launch
    ("c2_olmoe", 8, 8, 4),       # the most tokens and rows the fused launch takes (slots beyond the prefetched eight: none)
    ("c2_olmoe", 4, 16, 4),      # sixteen slots per token: the second half of the slots is fetched in the combine loop
    ("c2_olmoe", 8, 9, 0),       # one row too many: separate down and combine launches
    ("c5_dsv2lite", 9, 2, 0),    # one token too many
    ("c3_qwen15", 4, 4, 0),      # sigmoid-gated shared expert: its coefficient is evaluated by the combine kernel
])
def test_down_projection_with_the_combine_fused_for_a_handful_of_tokens(name, T, k, want):
    """Decode-sized calls: the routed down projection forms y itself (plan value 4) -- every way of dealing the waves
    out over the experts, several passes, the shared expert's rows -- and the sizes just outside that path."""
    import paper_2509_02753_amd as P
    cfg = S.mini(S.CONFIGS[name], L=1, d=256, F=448)     # 14 K-blocks of 32: not divisible by 4, 8 or 16 waves
    dl, _ = device_and_host_layer(cfg, 0)
    assert P.lexi_moe_down_plan(dl, T, k) == want
    del dl
    run_and_check_layer(cfg, 0, T, k)


@pytest.mark.parametrize("name,T", [("c5_dsv2lite", 3), ("c5_dsv2lite", 150), ("c2_olmoe", 2), ("c3_qwen15", 5)])
def test_profiled_stack_records_its_stage_events_and_changes_nothing(name, T):
    """lexi_moe_stack_forward_profiled: the same bits as the plain stack call, and five stage durations per layer
    that are non-negative and add up to the layer's span -- also where the shared expert's join is recorded before
    the launch that holds both the down projection and the combine (T = 2, 3: ungated / no shared expert)."""
    import torch
    import paper_2509_02753_amd as P
    cfg = S.mini(S.CONFIGS[name], L=3, d=256, F=384)
    kv = cfg.k_lexi()
    dls = [device_and_host_layer(cfg, l)[0] for l in range(cfg.L)]
    x = torch.stack([S.device_x(cfg, l, T) for l in range(cfg.L)])
    y0 = torch.empty((cfg.L, T, cfg.d), dtype=torch.float32, device="cuda:0")
    y1 = torch.empty_like(y0)
    ws = P.alloc_workspace(dls, T, int(kv.max()))
    P.lexi_moe_stack_forward(dls, kv, x, y0, ws)
    ev = P.StageEvents(cfg.L)
    P.lexi_moe_stack_forward(dls, kv, x, y1, ws, stage_events=ev)
    torch.cuda.synchronize()
    assert torch.equal(y0, y1)
    for row, st in zip(ev.events, ev.stage_ms()):
        assert len(st) == 5 and all(v >= 0.0 for v in st)
        assert abs(sum(st) - row[0].elapsed_time(row[5])) < 1e-3
        assert st[0] > 0.0 and st[1] > 0.0 and st[2] > 0.0    # routing, gate/up and down always launch something


@pytest.mark.parametrize("name,inter,d,T,k", [
    ("c4_mixtral", 0.0, 256, 1300, 2),     # 8 experts, prefill-sized: packed partials, eight tokens per wave in the top-k
    ("c4_mixtral", 0.0, 640, 2500, 2),     # five router segments (the second workgroup's last three waves idle), 16-token blocks
    ("c2_olmoe", 0.75, 256, 2100, 3),      # 16 experts (the shape inter-pruning three quarters of OLMoE's leaves)
    ("c5_dsv2lite", 0.875, 384, 1100, 4),  # 8 experts with a router bias and a shared expert
    ("c4_mixtral", 0.0, 256, 1024, 2),     # one token fewer than the narrow kernel's range: the 64-lane partials
])
def test_router_partials_for_eight_and_sixteen_experts(name, inter, d, T, k):
    """Prefill-sized batches on layers with exactly 8 or 16 experts take the narrow partial kernel (lane = token,
    weights by scalar loads, packed rows of partials): routing bit-exact on every token, outputs on a sample."""
    cfg = S.mini(S.CONFIGS[name], L=1, d=d, F=256)
    if inter:
        cfg = S.pruned(cfg, inter=inter)
    assert cfg.E in (8, 16)
    rng = np.random.default_rng(T)
    tokens = np.unique(np.concatenate([[0, T - 1], rng.integers(0, T, 62)])).astype(np.int32)
    run_and_check_layer(cfg, 0, T, k, tokens=tokens)
