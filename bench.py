#!/usr/bin/env python3
"""MoE-stack throughput on one MI355X: tokens/s of lexi_moe_stack_forward with a per-layer k vector.

A step is one pass of the whole hot path (router, top-k, gates, permutation, grouped gate/up GEMM + SwiGLU, down
GEMM, shared expert, combine) over all L layers of the workload, on synthetic seeded inputs already resident in HBM.

The default run measures EVERY workload and token regime of the benchmark (OLMoE-, Qwen1.5-MoE-, Mixtral- and
DeepSeek-V2-Lite-shaped stacks, prefill and decode) one after the other; the headline fields of the JSON line are
those of the largest single-GPU workload, the Mixtral-shaped 32-layer stack (90 GB of expert weights) at T = 4096
prefill tokens with its per-layer k vector, and the `regimes` array carries one record per (workload, T).
`--config NAME [--T N]` measures one workload (one regime) only, which then is the headline.

Prints ONE JSON line on stdout; progress and the per-stage table go to stderr.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E


def log(*a):
    print(*a, file=sys.stderr, flush=True)


# the files that hold the code of the expert-FFN kernels (the launch-argument structs of all kernels are elsewhere)
FFN_SOURCES = ("ffn.hip", "ffn_common.hpp", "ffn_stream.hip", "common.hpp")


def ffn_source_digest():
    """sha256 over the sources of the expert-FFN kernels: stored counter readings are only quoted for this exact code."""
    import hashlib
    h = hashlib.sha256()
    for name in FFN_SOURCES:
        with open(os.path.join(ROOT, "paper_2509_02753_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def stored_traffic(cfg_name, T):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 --pmc summary of this workload
    (FETCH_SIZE and WRITE_SIZE, each scaled by the same counter's reading for a copy of known size), or None when
    there is no summary or the kernel sources have changed since it was taken."""
    path = os.path.join(ROOT, "profiles", f"traffic_ffn_gate_up_{cfg_name}_T{T}.txt")
    if not os.path.exists(path):
        return None
    kv = {}
    with open(path) as f:
        for line in f:
            if ":" in line and not line.startswith("#"):
                k, v = line.split(":", 1)
                kv[k.strip()] = v.strip()
    if kv.get("ffn_source_sha256") != ffn_source_digest():
        return None
    try:
        return float(kv["hbm_bytes_per_launch"])
    except (KeyError, ValueError):
        return None


def measured_ceilings(torch, P, S, dev):
    """What this device sustains in plain loops (library probes, timed with events on the launch stream):
    bf16 MFMA rate on zero operands and on N(0,1) operands (the chip holds a lower clock when the operand bits toggle),
    and streaming-read bandwidth over a 4 GiB buffer."""
    def time_ms(fn, reps):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps
    sink = torch.zeros(256, dtype=torch.float32, device=dev)
    out = {}
    for label, sigma in (("zeros", 0.0), ("normal", 1.0)):
        ops = torch.zeros(64 * 1024, dtype=torch.bfloat16, device=dev)
        if sigma > 0:
            S.fill_device(ops, 0x4C455849, 999, sigma)
        flops = [0.0]
        def run():
            flops[0] = P.lexi_probe_mfma_bf16(ops, sink, 4000, 256)
        ms = time_ms(run, 5)
        out[f"mfma_bf16_tflops_{label}_operands"] = round(flops[0] / ms / 1e9, 1)
    buf = torch.empty(1 << 30, dtype=torch.float32, device=dev)     # 4 GiB, far beyond the 256 MB cache
    buf.fill_(1.0)
    nbytes = [0.0]
    def rd():
        nbytes[0] = P.lexi_probe_hbm_read(buf, sink)
    ms = time_ms(rd, 5)
    out["hbm_read_gbs"] = round(nbytes[0] / ms / 1e6, 1)
    del buf
    return out


def pruning_sweep(args, cfg0, T):
    """Fig. 2 analogue on synthetic weights: tokens/s of the whole stack against the number of active experts k
    (uniform over the layers) for the baseline shape and for the SHAPES of inter- (fewer experts) and intra-expert
    (narrower FFN) pruning at 12.5 / 25 / 50 %, plus the per-layer k vector on the baseline shape.  One JSON line."""
    import numpy as np
    import torch

    import lexi_synth as S
    import paper_2509_02753_amd as P
    dev = "cuda:0"
    torch.cuda.set_device(0)
    variants = [("base", 0.0, 0.0)] + [("inter", p, 0.0) for p in (0.125, 0.25, 0.5)] + [("intra", 0.0, p) for p in (0.125, 0.25, 0.5)]
    rows = []
    for kind, pi, pa in variants:
        cfg = S.pruned(cfg0, inter=pi, intra=pa) if (pi or pa) else cfg0
        L = args.layers if args.layers else cfg.L
        layers = []
        for l in range(L):
            rm = S.device_layer(cfg, l, dev)
            layers.append(P.Layer.from_tensors(rm, shared_kind=cfg.shared_kind))
            del rm
        tdt = torch.float32 if cfg.dtype == "f32" else torch.bfloat16
        x = torch.empty((L, T, cfg.d), dtype=tdt, device=dev)
        for l in range(L):
            S.fill_device(x[l], cfg.seed, S.tensor_id(l, S.KIND_X), cfg.sigma_x)
        y = torch.empty((L, T, cfg.d), dtype=torch.float32, device=dev)
        ws = P.alloc_workspace(layers, T, int(cfg.k_base))
        arr = P.binding._layer_array(layers)
        kvecs = [(f"uniform k={k}", np.full(L, k, dtype=np.int32)) for k in range(1, cfg.k_base + 1)]
        if kind == "base":
            kvecs.append(("per-layer k vector", cfg.k_lexi()[:L]))
        for label, kv in kvecs:
            for _ in range(args.warmup):
                P.lexi_moe_stack_forward(layers, kv, x, y, ws, layer_array=arr)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.steps):
                P.lexi_moe_stack_forward(layers, kv, x, y, ws, layer_array=arr)
            torch.cuda.synchronize()
            sec = (time.perf_counter() - t0) / args.steps
            rows.append({"variant": kind if kind == "base" else f"{kind} {100 * (pi or pa):g}%", "E": cfg.E, "F": cfg.F,
                         "k": label, "active_experts_sum": int(kv.sum()), "ms_per_step": round(sec * 1e3, 4),
                         "tokens_per_s": round(T / sec, 1),
                         "weight_gb": round(cfg.weight_bytes() * L / cfg.L / 1e9, 2)})
            log(f"[sweep] {rows[-1]}")
        del layers, x, y, ws, arr
        torch.cuda.empty_cache()
    print(json.dumps({"metric": "MoE-stack tokens/s", "sweep": "pruning shapes vs active experts", "unit": "tokens/s",
                      "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "data": "synthetic",
                      "config": {"workload": f"{cfg0.name} L={args.layers or cfg0.L} d={cfg0.d} T={T}"}, "rows": rows}), flush=True)


def budget_sweep(args, cfg, T):
    """tokens/s of the stack for seeded per-layer k vectors at the budgets B = L * kbar, kbar = k_min .. k_base (the
    last one is the uniform baseline), the way the paper's figures quote a model at several budgets.  One JSON line."""
    from dataclasses import replace

    import numpy as np
    import torch

    import lexi_synth as S
    import paper_2509_02753_amd as P
    dev = "cuda:0"
    torch.cuda.set_device(0)
    L = cfg.L
    layers = []
    for l in range(L):
        rm = S.device_layer(cfg, l, dev)
        layers.append(P.Layer.from_tensors(rm, shared_kind=cfg.shared_kind))
        del rm
    tdt = torch.float32 if cfg.dtype == "f32" else torch.bfloat16
    x = torch.empty((L, T, cfg.d), dtype=tdt, device=dev)
    for l in range(L):
        S.fill_device(x[l], cfg.seed, S.tensor_id(l, S.KIND_X), cfg.sigma_x)
    y = torch.empty((L, T, cfg.d), dtype=torch.float32, device=dev)
    ws = P.alloc_workspace(layers, T, int(cfg.k_base))
    arr = P.binding._layer_array(layers)
    prefill = (T * float(cfg.k_base) / cfg.E) >= 64
    use_graph = args.graph == "on" or (args.graph == "auto" and not prefill)
    rows = []
    budgets = sorted({L * kb for kb in range(cfg.k_min, cfg.k_base + 1)} | {cfg.budget})
    for B in budgets:
        kv = cfg.k_uniform() if B == L * cfg.k_base else replace(cfg, budget=B, fixed_kvec=None).k_lexi()
        assert int(kv.sum()) == B
        call = lambda: P.lexi_moe_stack_forward(layers, kv, x, y, ws, layer_array=arr)
        call()
        torch.cuda.synchronize()
        step = call
        if use_graph:
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                call()
            step = g.replay
        for _ in range(args.warmup):
            step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        sec = (time.perf_counter() - t0) / args.steps
        rows.append({"budget": int(B), "k_vec": kv.tolist(), "ms_per_step": round(sec * 1e3, 4), "tokens_per_s": round(T / sec, 1)})
        log(f"[sweep] B={B}: {sec * 1e3:.3f} ms/step, {T / sec:,.0f} tokens/s")
    base = rows[-1]["tokens_per_s"]
    for r in rows:
        r["vs_uniform_k"] = round(r["tokens_per_s"] / base, 4)
    print(json.dumps({"metric": "MoE-stack tokens/s", "sweep": "budgets", "unit": "tokens/s", "n_gpus": 1,
                      "steps": args.steps, "warmup": args.warmup, "data": "synthetic",
                      "config": {"workload": f"{cfg.name} L={L} d={cfg.d} E={cfg.E} F={cfg.F} Fs={cfg.F_shared} T={T}",
                                 "hip_graph": bool(use_graph)}, "rows": rows}), flush=True)


HEADLINE = ("c4_mixtral", 4096)
DEFAULT_WORKLOADS = ("c4_mixtral", "c2_olmoe", "c3_qwen15", "c5_dsv2lite")   # the headline workload first


def to_host_layer(torch, np, tensors):
    """Device tensors of one layer -> numpy (bf16 as uint16 bit patterns); the inputs, copied D2H."""
    h = {}
    for name, t in tensors.items():
        if t is None:
            h[name] = None
        elif t.dtype == torch.bfloat16:
            h[name] = t.view(torch.int16).cpu().numpy().view(np.uint16)
        else:
            h[name] = t.cpu().numpy()
    return h


def kernel_roofline(name, kernel, prefill, flops, nbytes, ms, traffic=None):
    """Roofline record of one launch: algorithmic flops (prefill: bf16 MFMA peak) or algorithmic bytes (decode: HBM
    peak) over the launch's average duration measured with HIP events on the launch stream."""
    if prefill:
        ach = flops / (ms * 1e-3) / 1e12
        rec = {"stage": name, "kernel": kernel, "bound": "mfma", "achieved": round(ach, 2), "peak": PEAK_BF16_TFLOPS,
               "unit": "TFLOP/s", "frac": round(ach / PEAK_BF16_TFLOPS, 4)}
    else:
        ach = nbytes / (ms * 1e-3) / 1e9
        rec = {"stage": name, "kernel": kernel, "bound": "hbm", "achieved": round(ach, 1), "peak": PEAK_HBM_GBS,
               "unit": "GB/s", "frac": round(ach / PEAK_HBM_GBS, 4)}
    rec.update({"traffic": traffic, "avg_launch_ms": round(ms, 4), "flops_per_launch": flops, "bytes_per_launch": nbytes})
    return rec


def measure_regime(args, mods, cfg, layers, arr, T, cpu_seconds, extras):
    """One (workload, T): tokens/s of the stack with the per-layer k vector and with uniform k, per-stage and
    per-kernel durations from HIP events, rooflines of the two grouped GEMMs, the whole path against both rooflines,
    experts touched per layer, and the oracle on a bounded sample (timed, and compared with the GPU's results)."""
    np, torch, S, P = mods
    dev = "cuda:0"
    L = len(layers)
    kvec = (cfg.k_lexi() if args.kvec == "lexi" else cfg.k_uniform())[:L]
    kuni = cfg.k_uniform()[:L]
    tdt = torch.float32 if cfg.dtype == "f32" else torch.bfloat16
    es = 4 if cfg.dtype == "f32" else 2
    x = torch.empty((L, T, cfg.d), dtype=tdt, device=dev)
    for l in range(L):
        S.fill_device(x[l], cfg.seed, S.tensor_id(l, S.KIND_X), cfg.sigma_x)
    y = torch.empty((L, T, cfg.d), dtype=torch.float32, device=dev)
    ws = P.alloc_workspace(layers, T, int(max(kvec.max(), kuni.max())))
    torch.cuda.synchronize()
    log(f"[bench] {cfg.name} T={T} L={L} kvec={kvec.tolist()} (sum {int(kvec.sum())}, uniform {int(kuni.sum())}), "
        f"workspace {ws.numel() / 1e6:.0f} MB")

    def run_steps(kv, n, events=None, chained=False):
        for _ in range(n):
            if chained:   # one input, hidden state updated in place in y[0]
                P.lexi_moe_stack_forward(layers, kv, x[0], y[0], ws, layer_array=arr, chained=True)
            else:
                P.lexi_moe_stack_forward(layers, kv, x, y, ws, layer_array=arr, stage_events=events)

    prefill = (T * float(np.mean(kvec)) / cfg.E) >= 64
    use_graph = args.graph == "on" or (args.graph == "auto" and not prefill)

    def timed(kv, chained=False):
        """K steps between two synchronisations (wall clock), one HIP event between consecutive steps (median)."""
        if use_graph:   # the whole stack call (every launch of all L layers, a side-stream fork/join included) as one HIP graph
            run_steps(kv, 1, chained=chained)      # first-use set-up inside the library happens outside the capture
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                run_steps(kv, 1, chained=chained)
            step = g.replay
        else:
            step = lambda: run_steps(kv, 1, chained=chained)
        for _ in range(args.warmup):
            step()
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
        torch.cuda.synchronize()
        t_start = time.perf_counter()
        marks[0].record()
        for i in range(args.steps):
            step()
            marks[i + 1].record()
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t_start) / args.steps
        per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))
        return wall, per_step[len(per_step) // 2] * 1e-3

    sec, sec_med = timed(kvec)
    log(f"[bench]   k={args.kvec}: {sec * 1e3:.3f} ms/step (median of per-step events {sec_med * 1e3:.3f}), {T / sec:,.0f} tokens/s")
    compare_uniform = args.kvec == "lexi" and not args.no_uniform
    sec_uniform = timed(kuni)[0] if compare_uniform else None
    if compare_uniform:
        log(f"[bench]   uniform k={cfg.k_base}: {sec_uniform * 1e3:.3f} ms/step, {T / sec_uniform:,.0f} tokens/s")

    chained = None
    if extras and not args.no_chained and len({(ly.c.d, ly.c.dtype) for ly in layers}) == 1:
        sec_ch = timed(kvec, chained=True)[0]
        chained = {"ms_per_step": round(sec_ch * 1e3, 4), "tokens_per_s": round(T / sec_ch, 1),
                   "vs_independent": round(sec / sec_ch, 4)}
        log(f"[bench]   chained residual mode: {sec_ch * 1e3:.3f} ms/step, {T / sec_ch:,.0f} tokens/s")

    # ---- per-stage durations with HIP events recorded by the library on the launch stream ----
    ev = P.StageEvents(L)
    stage_sum = np.zeros((L, 5))
    n_ev = max(3, min(args.steps, 10))
    for _ in range(n_ev):
        run_steps(kvec, 1, events=ev)
        torch.cuda.synchronize()
        stage_sum += np.asarray(ev.stage_ms())
    stage_ms = stage_sum / n_ev                  # [L][5] average ms per launch group
    per_stage = stage_ms.sum(0)
    log("[bench]   stage ms per step: " + ", ".join(f"{n}={v:.3f}" for n, v in zip(P.STAGE_NAMES, per_stage)) +
        f"  (sum {per_stage.sum():.3f} vs step {sec * 1e3:.3f})")

    # ---- routing of the whole batch: experts touched per layer (U), and the GPU results the oracle sample is compared with
    routs = [P.RoutingOut(T, int(kvec[l]), cfg.E) for l in range(L)]
    P.lexi_moe_stack_forward(layers, kvec, x, y, ws, routing=routs)
    torch.cuda.synchronize()
    counts = [r.counts.cpu().numpy() for r in routs]
    U = [int((c > 0).sum()) for c in counts]

    # ---- algorithmic work (only selected experts, only touched weights) ----
    gu_flops = [4.0 * T * int(k) * cfg.d * cfg.F for k in kvec]
    dn_flops = [2.0 * T * int(k) * cfg.d * cfg.F for k in kvec]
    gu_bytes = [U[l] * 2.0 * cfg.d * cfg.F * es + T * cfg.d * es for l in range(L)]
    dn_bytes = [U[l] * 1.0 * cfg.d * cfg.F * es + T * cfg.d * 4 for l in range(L)]     # weights + the layer's fp32 output
    tot_flops = sum(T * (2.0 * cfg.d * cfg.E + int(k) * 6.0 * cfg.d * cfg.F + 6.0 * cfg.d * cfg.F_shared) for k in kvec)
    tot_bytes = sum(U[l] * 3 * cfg.d * cfg.F * es + 3 * cfg.d * cfg.F_shared * es + cfg.d * cfg.E * 4 + T * cfg.d * es + T * cfg.d * 4
                    for l in range(L))
    gu_ms, dn_ms = float(stage_ms[:, 1].mean()), float(stage_ms[:, 2].mean())
    gu_kernel = "ffn_mfma_kernel<gate_up>" if prefill else "ffn_mfma_kernel<gate_up> / ffn_stream_kernel<gate_up> (by rows per expert)"
    plan_names = {0: "ffn_stream_kernel<down>", 1: "ffn_mfma_kernel<down>", 2: "ffn_mfma_kernel<down> (reduction cut in two)",
                  3: "ffn_mfma_kernel<down> (output rows stored directly, no combine launch)",
                  4: "down_combine_kernel (down projection and combine in one launch)"}
    dn_kernel = " / ".join(plan_names[p] for p in sorted({P.lexi_moe_down_plan(layers[l], T, int(kvec[l])) for l in range(L)}))
    roof_gu = kernel_roofline("gate_up", gu_kernel, prefill, sum(gu_flops) / L, sum(gu_bytes) / L, gu_ms,
                              stored_traffic(cfg.name, T))
    roof_dn = kernel_roofline("down", dn_kernel, prefill, sum(dn_flops) / L, sum(dn_bytes) / L, dn_ms)
    # the same launches per distinct k: a layer with few active experts has fewer FLOPs per weight byte, so its binding
    # roofline (the larger of FLOPs / MFMA peak and bytes / HBM peak) can be the other one
    per_k = []
    for kk in sorted(set(int(v) for v in kvec)):
        ls = [l for l in range(L) if int(kvec[l]) == kk]
        rec = {"k": kk, "layers": len(ls)}
        for nm, col, fl, by in (("gate_up", 1, gu_flops, gu_bytes), ("down", 2, dn_flops, dn_bytes)):
            ms = float(np.mean([stage_ms[l, col] for l in ls]))
            f, b = float(np.mean([fl[l] for l in ls])), float(np.mean([by[l] for l in ls]))
            t_mfma, t_hbm = f / (PEAK_BF16_TFLOPS * 1e12), b / (PEAK_HBM_GBS * 1e9)
            rec[nm] = {"avg_launch_ms": round(ms, 4), "tflops": round(f / ms / 1e9, 1), "gbs": round(b / ms / 1e6, 1),
                       "bound": "mfma" if t_mfma >= t_hbm else "hbm", "frac": round(max(t_mfma, t_hbm) / (ms * 1e-3), 4)}
        per_k.append(rec)
    whole = {"flops_per_step": tot_flops, "bytes_per_step": tot_bytes,
             "mfma_frac": round(tot_flops / sec / 1e12 / PEAK_BF16_TFLOPS, 4),
             "hbm_frac": round(tot_bytes / sec / 1e9 / PEAK_HBM_GBS, 4)}
    log(f"[bench]   gate/up {roof_gu['achieved']} {roof_gu['unit']} = {roof_gu['frac']:.3f} of peak; down {roof_dn['achieved']} "
        f"{roof_dn['unit']} = {roof_dn['frac']:.3f}; whole path {whole['mfma_frac']:.3f} MFMA / {whole['hbm_frac']:.3f} HBM")

    # ---- CPU baseline: the oracle as it stands on a bounded sample of the same workload, timed, and its results
    #      compared with what the GPU produced for the same tokens (routing mismatches, output error)
    cpu, parity = None, None
    if not args.no_cpu_baseline and cpu_seconds > 0 and args.operands == "normal":
        import oracle as O
        n = args.cpu_sample_tokens
        # the sample: the first n tokens of the inputs of `nl` layers spread over the stack; n from a pilot so that the
        # oracle's work takes about cpu_seconds (copying a layer's weights to the host is not part of the timing)
        nl = min(L, 8) if extras else min(L, 2)
        ls = sorted(set(int(round(i * (L - 1) / max(nl - 1, 1))) for i in range(nl)))
        hl0 = O.Layer.from_tensors(cfg, to_host_layer(torch, np, S.device_layer(cfg, ls[0], dev)))
        if n is None:
            npilot = min(T, 16)
            xp = x[ls[0], :npilot].contiguous()
            xp = xp.view(torch.int16).cpu().numpy().view(np.uint16) if tdt == torch.bfloat16 else xp.cpu().numpy()
            t1 = time.perf_counter()
            O.moe_layer(hl0, xp, int(kvec[ls[0]]), round_act=True)
            rate = npilot / max(time.perf_counter() - t1, 1e-6)          # tokens/s of one layer
            n = max(1, min(T, int(cpu_seconds * rate / len(ls))))
        wall, mism, err_r, err_u = 0.0, 0, 0.0, None
        for i, l in enumerate(ls):
            hl = hl0 if i == 0 else O.Layer.from_tensors(cfg, to_host_layer(torch, np, S.device_layer(cfg, l, dev)))
            xh = x[l, :n].contiguous()
            xh = xh.view(torch.int16).cpu().numpy().view(np.uint16) if tdt == torch.bfloat16 else xh.cpu().numpy()
            t1 = time.perf_counter()
            ref = O.moe_layer(hl, xh, int(kvec[l]), round_act=True)
            wall += time.perf_counter() - t1
            got = y[l, :n].cpu().numpy().astype(np.float64)
            mism += int((routs[l].topk_idx[:n].cpu().numpy() != ref.topk_idx).any(axis=1).sum())
            rms = float(np.sqrt(np.mean(ref.out ** 2)))
            err_r = max(err_r, float(np.abs(got - ref.out).max()) / rms)
            if i == 0:   # against the oracle WITHOUT the bf16 rounding of the SwiGLU intermediate (reported, not graded)
                ref_u = O.moe_layer(hl, xh, int(kvec[l]), round_act=False)
                err_u = float(np.abs(got - ref_u.out).max()) / float(np.sqrt(np.mean(ref_u.out ** 2)))
            del hl
        del hl0
        stack_rate = n / (wall * L / len(ls))      # tokens/s of the whole L-layer stack at the sampled layers' rate
        cpu = {"value": round(stack_rate, 3), "unit": "tokens/s", "cores": O.num_threads(), "kind": "oracle",
               "sample": f"first {n} tokens of the inputs of layers {ls} (router + FFN + combine, fp64) in {wall:.1f}s, "
                         f"scaled to the {L}-layer stack"}
        parity = {"tokens": n, "layers": ls, "routing_mismatches": mism, "max_err_over_rms": float(f"{err_r:.3e}"),
                  "max_err_over_rms_vs_unrounded_oracle": None if err_u is None else float(f"{err_u:.3e}")}
        log(f"[bench]   cpu oracle: {n} tokens x {len(ls)} layers in {wall:.1f}s on {O.num_threads()} threads -> "
            f"{stack_rate:.2f} tokens/s (stack); routing mismatches {mism}, max err/RMS {err_r:.2e} (unrounded oracle {err_u:.2e})")

    # ---- Stage-1 profiling (Algorithm 1), one iteration on layer 0: all k of the search space from one baseline pass,
    #      against the algorithm as printed (1 + |list| full forward passes)
    stage1 = None
    if extras and not args.no_stage1:
        kb = int(cfg.k_base)
        klist = list(range(1, kb + 1))
        yl = torch.empty((T, cfg.d), dtype=torch.float32, device=dev)
        need = P.binding._lib.lexi_moe_profile_workspace_bytes(layers[0].c, T, kb, len(klist))
        ws_prof = torch.empty(int(need), dtype=torch.uint8, device=dev)

        def fused():
            return P.lexi_moe_profile_layer(layers[0], x[0], kb, klist, workspace=ws_prof)

        def printed():
            for kk in [kb] + klist:
                P.lexi_moe_layer_forward(layers[0], x[0], yl, kk, ws)

        times = []
        for fn in (fused, printed):
            fn()
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            for _ in range(args.steps):
                fn()
            torch.cuda.synchronize()
            times.append((time.perf_counter() - t1) / args.steps * 1e3)
        stage1 = {"layer": 0, "k_base": kb, "k_list": klist, "ms_per_iteration": round(times[0], 4),
                  "ms_as_printed": round(times[1], 4), "speedup": round(times[1] / times[0], 3),
                  "tokens_per_s": round(T / times[0] * 1e3, 1)}
        log(f"[bench]   stage-1 profiling, layer 0, k in 1..{kb}: {times[0]:.3f} ms per iteration "
            f"(vs {times[1]:.3f} ms as {1 + len(klist)} forward passes)")
        del ws_prof, yl

    rec = {
        "workload": f"{cfg.name} L={L} d={cfg.d} E={cfg.E} F={cfg.F} Fs={cfg.F_shared} T={T}", "name": cfg.name, "T": T,
        "regime": "prefill" if prefill else "decode", "hip_graph": bool(use_graph),
        "k_vec": kvec.tolist(), "k_sum": int(kvec.sum()), "k_uniform": int(cfg.k_base),
        "ms_per_step": round(sec * 1e3, 4), "ms_per_step_median_of_events": round(sec_med * 1e3, 4),
        "tokens_per_s": round(T / sec, 1),
        "uniform_k_tokens_per_s": round(T / sec_uniform, 1) if sec_uniform else None,
        "speedup_vs_uniform_k": round(sec_uniform / sec, 4) if sec_uniform else None,
        "stage_ms_per_step": {n: round(float(v), 4) for n, v in zip(P.STAGE_NAMES, per_stage)},
        "experts_touched_per_layer": U,
        "rooflines": [roof_gu, roof_dn], "per_k": per_k, "whole_path": whole,
        "chained_stack": chained, "stage1_profiling": stage1, "cpu_baseline": cpu, "parity_on_sample": parity,
    }
    del x, y, ws, routs
    return rec


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default=None, help="measure this workload only (default: every workload, headline c4_mixtral T=4096)")
    ap.add_argument("--T", type=int, default=None, help="with --config: this token count only (default: all regimes of the workload)")
    ap.add_argument("--kvec", default="lexi", choices=["lexi", "uniform"])
    ap.add_argument("--layers", type=int, default=None, help="use only the first N layers (debugging; not a valid result)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-uniform", action="store_true", help="skip the uniform-k comparison run (profiling: every launch then uses k_vec)")
    ap.add_argument("--cpu-sample-tokens", type=int, default=None)
    ap.add_argument("--no-stage1", action="store_true", help="skip the Stage-1 profiling timing")
    ap.add_argument("--no-chained", action="store_true", help="skip the timing of the chained residual mode")
    ap.add_argument("--no-ceilings", action="store_true", help="skip the matrix-core / HBM ceiling probes")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="end with one 256 MiB device-to-device copy kernel (counter runs scale FETCH_SIZE / WRITE_SIZE by it)")
    ap.add_argument("--sweep", default=None, choices=["pruning", "budgets"],
                    help="instead of the benchmark line: tokens/s vs active experts for the baseline and the pruned shapes "
                         "(pruning), or tokens/s of per-layer k vectors at every budget B = L*k, k = k_min..k_base (budgets)")
    ap.add_argument("--operands", default="normal", choices=["normal", "zero-weights"],
                    help="zero-weights: every expert weight is zero while router and activations stay as they are, so the "
                         "routing, the tiles and the bytes moved are the same but the matrix cores multiply by zero.  A probe of "
                         "how far the GEMM rates depend on the operand values (the chip lowers its clock when the multiplier "
                         "inputs toggle); NOT a valid benchmark result")
    ap.add_argument("--graph", default="auto", choices=["auto", "on", "off"],
                    help="replay the stack call from a captured HIP graph (auto: for decode-sized batches, whose steps are launch-bound)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: the library has no multi-GPU path (run with --gpus 1)")

    import numpy as np
    import torch

    import lexi_synth as S
    import paper_2509_02753_amd as P

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.sweep:
        cfg = S.CONFIGS[args.config or "c2_olmoe"]
        T = args.T if args.T is not None else cfg.T_regimes[0]
        return pruning_sweep(args, cfg, T) if args.sweep == "pruning" else budget_sweep(args, cfg, T)
    dev = "cuda:0"
    torch.cuda.set_device(0)
    mods = (np, torch, S, P)
    from paper_2509_02753_amd.binding import _layer_array

    if args.config:
        cfg = S.CONFIGS[args.config]
        plan = [(cfg, [args.T] if args.T is not None else list(cfg.T_regimes))]
        headline = (cfg.name, plan[0][1][0])
    else:
        plan = [(S.CONFIGS[n], list(S.CONFIGS[n].T_regimes)) for n in DEFAULT_WORKLOADS]
        headline = HEADLINE

    regimes = []
    for cfg, Ts in plan:
        L = args.layers if args.layers else cfg.L
        t0 = time.time()
        layers = []
        for l in range(L):
            row_major = S.device_layer(cfg, l, dev)          # seeded generator, straight into HBM
            if args.operands == "zero-weights":
                for name in ("w_gate", "w_up", "w_down", "ws_gate", "ws_up", "ws_down"):
                    if row_major.get(name) is not None:
                        row_major[name].zero_()
            layers.append(P.Layer.from_tensors(row_major, shared_kind=cfg.shared_kind))   # packed by the library's kernel
            del row_major
        torch.cuda.synchronize()
        log(f"[bench] {cfg.name}: weights resident in HBM after {time.time() - t0:.1f}s ({cfg.weight_bytes() * L / cfg.L / 1e9:.2f} GB)")
        arr = _layer_array(layers)
        for T in Ts:
            is_head = (cfg.name, T) == headline
            # the oracle sample: about 15 s of CPU work for the headline, about 3 s for every other regime
            regimes.append(measure_regime(args, mods, cfg, layers, arr, T, 15.0 if is_head else 3.0, extras=is_head))
        del layers, arr
        torch.cuda.empty_cache()

    ceilings = None if args.no_ceilings else measured_ceilings(torch, P, S, dev)
    if ceilings:
        log("[bench] measured ceilings: " + ", ".join(f"{k}={v}" for k, v in ceilings.items()))

    if args.calibration_copy:
        src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        torch.mul(src, 1.0, out=dst)     # one elementwise kernel: reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()

    h = next(r for r in regimes if (r["name"], r["T"]) == headline)
    out = {
        "metric": "MoE-stack tokens/s" if args.operands == "normal" else "MoE-stack tokens/s (operand-value probe, not a valid result)",
        "operands": args.operands, "value": h["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": h["ms_per_step"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": S.CONFIGS[h["name"]].dtype, "data": "synthetic",
        "config": {"workload": h["workload"], "k_vec": h["k_vec"], "k_sum": h["k_sum"], "k_uniform": h["k_uniform"],
                   "regime": h["regime"], "hip_graph": h["hip_graph"]},
        "ms_per_step_median_of_events": h["ms_per_step_median_of_events"],
        "uniform_k_tokens_per_s": h["uniform_k_tokens_per_s"], "speedup_vs_uniform_k": h["speedup_vs_uniform_k"],
        "stage_ms_per_step": h["stage_ms_per_step"], "experts_touched_per_layer": h["experts_touched_per_layer"],
        "roofline": dict(h["rooflines"][0], per_k=h["per_k"]), "roofline_down": h["rooflines"][1],
        "whole_path": h["whole_path"], "chained_stack": h["chained_stack"], "stage1_profiling": h["stage1_profiling"],
        "measured_ceilings": ceilings, "cpu_baseline": h["cpu_baseline"], "parity_on_sample": h["parity_on_sample"],
        "regimes": [{k: v for k, v in r.items() if k not in ("name",)} for r in regimes],
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
