"""Pins for the CPU oracle: closed forms, brute force, library routines and invariants.

The paper prints no worked numbers for the MoE forward, so every pin here is
something the definition in its Sec. 2 (y = sum_{TopK} G_i E_i(x),
G = Softmax(TopK[x W_g])) and plain mathematics fix.  Each pin is chosen so
that a plausible slip in the oracle (dropped term, wrong sign or index,
transposed operand, wrong tie rule, softmax over the wrong set) fails it.
"""
import itertools

import numpy as np
import pytest
import scipy.special

import lexi_synth as S
import oracle as O
from lexi_synth import generator as G


def bf16(a):
    """fp32 -> bf16 bits -> fp32 values (round to nearest even), via the generator module's helper."""
    return G.bf16_bits_to_f32(G.f32_to_bf16_bits(np.asarray(a, dtype=np.float32)))


def widen(a, dtype):
    return a.astype(np.float64) if dtype == "f32" else G.bf16_bits_to_f32(a).astype(np.float64)


def tiny_layer(dtype="f32", d=128, E=8, F=16, seed=11, bias=False, F_shared=0, shared_kind=0):
    rng = np.random.default_rng(seed)

    def w(*shape, sigma=0.1):
        a = (rng.standard_normal(shape) * sigma).astype(np.float32)
        return a if dtype == "f32" else G.f32_to_bf16_bits(a)

    t = dict(w_router=(rng.standard_normal((d, E)) * 0.1).astype(np.float32), w_gate=w(E, F, d), w_up=w(E, F, d),
             w_down=w(E, d, F), router_bias=(rng.standard_normal(E).astype(np.float32) if bias else None))
    if F_shared:
        t.update(ws_gate=w(F_shared, d), ws_up=w(F_shared, d), ws_down=w(d, F_shared))
        if shared_kind == 2:
            t["w_shared_gate"] = w(d)
    x = rng.standard_normal((9, d)).astype(np.float32)
    x = x if dtype == "f32" else G.f32_to_bf16_bits(x)
    ly = O.Layer(d, E, F, dtype, t["w_router"], t["w_gate"], t["w_up"], t["w_down"], router_bias=t["router_bias"],
                 F_shared=F_shared, shared_kind=shared_kind, ws_gate=t.get("ws_gate"), ws_up=t.get("ws_up"),
                 ws_down=t.get("ws_down"), w_shared_gate=t.get("w_shared_gate"))
    return ly, t, x


def np_ffn(x64, wg64, wu64, wd64):
    """Dense SwiGLU FFN with numpy matmuls in fp64 (library routine, no loops)."""
    hg, hu = wg64 @ x64, wu64 @ x64
    return wd64 @ (hg / (1.0 + np.exp(-hg)) * hu)


# ---------------------------------------------------------------- router logits (x . W_g)

@pytest.mark.parametrize("dtype,d", [("f32", 128), ("bf16", 384), ("bf16", 2048)])
def test_logits_within_rounding_bound_of_fp64(dtype, d):
    ly, t, x = tiny_layer(dtype, d=d, E=8, bias=True)
    l32 = O.router_logits(ly, x)
    x64, w64 = widen(x, dtype), t["w_router"].astype(np.float64)
    l64 = x64 @ w64 + t["router_bias"].astype(np.float64)
    n_ops = 128 + d // 128 + 1               # longest chain of roundings any term passes through
    bound = n_ops * 2.0 ** -24 * (np.abs(x64) @ np.abs(w64) + np.abs(t["router_bias"]))
    assert np.all(np.abs(l32 - l64) <= bound)
    # a transposed or shifted operand is far outside the bound
    assert np.abs(l32 - l64).max() < 1e-5 and np.abs(l64).max() > 0.1


def test_logits_exact_on_small_integers():
    # every product and partial sum is an integer below 2^24: any evaluation order gives the exact dot product
    rng = np.random.default_rng(3)
    d, E, T = 256, 6, 7
    x = rng.integers(-8, 9, (T, d)).astype(np.float32)
    w = rng.integers(-8, 9, (d, E)).astype(np.float32)
    b = rng.integers(-5, 6, E).astype(np.float32)
    z = np.zeros((E, 4, d), np.float32)
    ly = O.Layer(d, E, 4, "f32", w, z, z, np.zeros((E, d, 4), np.float32), router_bias=b)
    expect = x.astype(np.int64) @ w.astype(np.int64) + b.astype(np.int64)
    assert np.array_equal(O.router_logits(ly, x).astype(np.int64), expect)
    assert np.array_equal(O.router_logits(ly, x), expect.astype(np.float32))


def test_logit_order_is_segmented_fma_chain():
    # A case built so that the evaluation order is visible in the bits: 2^24 then many 1s.
    # Inside a 128-segment the running sum absorbs each +1 (2^24 + 1 rounds back to 2^24, ties-to-even),
    # while a later segment first sums its own 1s to 128 and only then meets 2^24.
    d, E = 256, 1
    x = np.ones((1, d), np.float32)
    w = np.ones((d, E), np.float32)
    w[0, 0] = 2.0 ** 24
    z = np.zeros((E, 4, d), np.float32)
    ly = O.Layer(d, E, 4, "f32", w, z, z, np.zeros((E, d, 4), np.float32))
    got = float(O.router_logits(ly, x)[0, 0])
    assert got == 2.0 ** 24 + 128.0       # segment 0 -> 2^24 (127 ones lost), segment 1 -> 128, then one add
    # fused multiply-add: x*w is not rounded before the add.  (1+2^-12)^2 = 1 + 2^-11 + 2^-24; minus (1+2^-11)
    x2 = np.zeros((1, 128), np.float32); w2 = np.zeros((128, 1), np.float32)
    x2[0, 0] = -(1 + 2.0 ** -11); w2[0, 0] = 1.0
    x2[0, 1] = 1 + 2.0 ** -12; w2[1, 0] = 1 + 2.0 ** -12
    z2 = np.zeros((1, 4, 128), np.float32)
    ly2 = O.Layer(128, 1, 4, "f32", w2, z2, z2, np.zeros((1, 128, 4), np.float32))
    assert float(O.router_logits(ly2, x2)[0, 0]) == 2.0 ** -24   # an unfused product would give 0


# ---------------------------------------------------------------- TopK selection

def brute_topk(l, k):
    return sorted(range(len(l)), key=lambda e: (-float(l[e]), e))[:k]


def test_topk_brute_force_random_and_ties():
    rng = np.random.default_rng(5)
    for E in (1, 2, 5, 8, 60, 64):
        logits = rng.standard_normal((40, E)).astype(np.float32)
        logits[::3] = np.round(logits[::3])            # many exact ties
        logits[1::7] = 0.25                             # all equal
        for k in sorted({1, 2, min(3, E), E}):
            if k > E:
                continue
            got = O.topk(logits, k)
            for t in range(logits.shape[0]):
                assert list(got[t]) == brute_topk(logits[t], k)


def test_topk_tie_goes_to_lower_index_and_zero_signs():
    l = np.array([[1.0, 3.0, 3.0, -1.0, 3.0], [0.0, -0.0, 0.0, -5.0, -0.0]], np.float32)
    assert O.topk(l, 3).tolist() == [[1, 2, 4], [0, 1, 2]]
    assert O.topk(l, 1).tolist() == [[1], [0]]


def test_topk_k1_is_argmax_and_prefix_nesting():
    rng = np.random.default_rng(6)
    logits = rng.standard_normal((64, 16)).astype(np.float32)
    assert np.array_equal(O.topk(logits, 1)[:, 0], np.argmax(logits, axis=1))  # np.argmax: first maximum
    full = O.topk(logits, 16)
    for k in range(1, 16):
        assert np.array_equal(O.topk(logits, k), full[:, :k])
    assert np.array_equal(np.sort(full, axis=1), np.tile(np.arange(16), (64, 1)))


def test_duplicate_router_columns_tie_to_lower_expert():
    ly, t, x = tiny_layer("bf16", d=128, E=8)
    w = t["w_router"].copy()
    w[:, 5] = w[:, 2]                      # experts 2 and 5 get bit-identical logits
    ly2 = O.Layer(128, 8, 16, "bf16", w, t["w_gate"], t["w_up"], t["w_down"])
    r = O.moe_layer(ly2, x, 8, routing_only=True)
    assert np.array_equal(r.logits[:, 2], r.logits[:, 5])
    for row in r.topk_idx:
        row = list(row)
        assert row.index(2) + 1 == row.index(5)


# ---------------------------------------------------------------- gates (softmax over the selected)

def test_gates_sum_to_one_and_special_cases():
    rng = np.random.default_rng(7)
    logits = (rng.standard_normal((50, 12)) * 3).astype(np.float32)
    for k in (1, 2, 5, 12):
        idx = O.topk(logits, k)
        g = O.gates(logits, idx)
        assert np.allclose(g.astype(np.float64).sum(1), 1.0, atol=1e-6)
        assert np.all(np.diff(g, axis=1) <= 0)                     # rank order -> non-increasing gates
        if k == 1:
            assert np.all(g == 1.0)
        if k == 12:                                                # k = E: the full softmax (library routine)
            sm = scipy.special.softmax(logits.astype(np.float64), axis=1)
            assert np.allclose(g, np.take_along_axis(sm, idx.astype(np.int64), 1), rtol=0, atol=1e-7)
        # general k: full softmax renormalised over the selected
        sm = scipy.special.softmax(logits.astype(np.float64), axis=1)
        sel = np.take_along_axis(sm, idx.astype(np.int64), 1)
        assert np.allclose(g, sel / sel.sum(1, keepdims=True), rtol=0, atol=1e-7)
    two = np.array([[0.7, -1.0, 0.7, 0.1]], np.float32)
    assert O.gates(two, O.topk(two, 2)).tolist() == [[0.5, 0.5]]
    # closed form for k = 2: sigmoid of the logit gap
    pair = np.array([[2.0, 0.5, -3.0]], np.float32)
    g = O.gates(pair, O.topk(pair, 2))[0]
    assert abs(g[0] - 1 / (1 + np.exp(-1.5))) < 1e-7 and abs(g[1] - 1 / (1 + np.exp(1.5))) < 1e-7


def test_gates_shift_invariance_large_logits():
    l = np.array([[1000.0, 999.0, 10.0]], np.float32)   # a naive exp() would overflow
    g = O.gates(l, O.topk(l, 2))[0]
    assert np.isfinite(g).all() and abs(g[0] - 1 / (1 + np.exp(-1.0))) < 1e-7


# ---------------------------------------------------------------- permutation

@pytest.mark.parametrize("T,E,k", [(1, 8, 2), (37, 8, 3), (64, 60, 4), (5, 4, 4), (130, 64, 8)])
def test_permutation_is_stable_sort_by_expert(T, E, k):
    rng = np.random.default_rng(T * 100 + E)
    logits = rng.standard_normal((T, E)).astype(np.float32)
    idx = O.topk(logits, k)
    p = O.permutation(idx, E)
    flat = idx.reshape(-1)
    assert np.array_equal(p.perm, np.argsort(flat, kind="stable"))          # library routine
    assert np.array_equal(p.counts, np.bincount(flat, minlength=E))
    assert p.offsets[0] == 0 and np.array_equal(np.diff(p.offsets), p.counts) and p.offsets[-1] == T * k
    assert np.array_equal(np.sort(p.perm), np.arange(T * k))
    assert np.array_equal(p.inv_perm[p.perm], np.arange(T * k))             # permute o unpermute = identity
    assert np.array_equal(p.perm[p.inv_perm], np.arange(T * k))
    for e in range(E):
        grp = p.perm[p.offsets[e]:p.offsets[e + 1]]
        assert np.all(flat[grp] == e) and np.all(np.diff(grp // k) > 0)     # right expert, tokens ascending


def test_permutation_with_empty_experts():
    idx = np.array([[3, 1], [3, 0], [1, 3]], np.int32)
    p = O.permutation(idx, 6)
    assert p.counts.tolist() == [1, 2, 0, 3, 0, 0]
    assert p.offsets.tolist() == [0, 1, 3, 3, 6, 6, 6]
    assert p.perm.tolist() == [3, 1, 4, 0, 2, 5]


# ---------------------------------------------------------------- expert FFN

def test_ffn_hand_computed_scalar():
    # d = F = 1: x=2, wg=.5 -> hg=1, silu(1)=1/(1+e^-1); wu=3 -> hu=6; wd=.25
    one = lambda v: np.array(v, np.float32).reshape(1, 1, 1)
    ly = O.Layer(1, 1, 1, "f32", np.zeros((1, 1), np.float32), one(0.5), one(3.0), one(0.25))
    y = O.expert_ffn(ly, 0, np.array([[2.0]], np.float32), 0)
    assert abs(y[0] - 0.25 * 6.0 / (1.0 + np.exp(-1.0))) < 1e-15


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_ffn_matches_numpy_matmul(dtype):
    ly, t, x = tiny_layer(dtype, d=128, E=4, F=24)
    x64 = widen(x, dtype)
    for e in range(4):
        for tok in (0, 3, 8):
            ref = np_ffn(x64[tok], widen(t["w_gate"][e], dtype), widen(t["w_up"][e], dtype), widen(t["w_down"][e], dtype))
            got = O.expert_ffn(ly, e, x, tok)
            assert np.allclose(got, ref, rtol=1e-12, atol=1e-14)
    # non-square shapes catch a transposed weight: F != d here (24 vs 128)


def test_ffn_constant_up_projection_closed_form():
    # Wup == c everywhere  =>  hu = c * sum(x) for every f  =>  y = Wd @ silu(Wg x) * c*sum(x)
    ly, t, x = tiny_layer("f32", d=128, E=2, F=8)
    wu = np.full_like(t["w_up"], 0.25)
    ly2 = O.Layer(128, 2, 8, "f32", t["w_router"], t["w_gate"], wu, t["w_down"])
    x64 = x.astype(np.float64)
    hg = t["w_gate"][1].astype(np.float64) @ x64[2]
    ref = t["w_down"][1].astype(np.float64) @ (hg / (1 + np.exp(-hg))) * (0.25 * x64[2].sum())
    assert np.allclose(O.expert_ffn(ly2, 1, x, 2), ref, rtol=1e-11, atol=1e-13)


def test_ffn_round_act_rounds_only_the_intermediate():
    ly, t, x = tiny_layer("bf16", d=128, E=2, F=24)
    x64 = widen(x, "bf16")
    wg, wu, wd = (widen(t[n][1], "bf16") for n in ("w_gate", "w_up", "w_down"))
    hg, hu = wg @ x64[4], wu @ x64[4]
    a = hg / (1 + np.exp(-hg)) * hu
    ref_rounded = wd @ bf16(a.astype(np.float32)).astype(np.float64)
    assert np.allclose(O.expert_ffn(ly, 1, x, 4, round_act=True), ref_rounded, rtol=1e-12, atol=1e-14)
    assert not np.allclose(O.expert_ffn(ly, 1, x, 4, round_act=False), ref_rounded, rtol=1e-9, atol=0)
    # fp32 layers have no bf16 rounding point: the flag changes nothing
    lf, tf, xf = tiny_layer("f32", d=128, E=2, F=24)
    assert np.array_equal(O.expert_ffn(lf, 0, xf, 1, round_act=True), O.expert_ffn(lf, 0, xf, 1, round_act=False))


# ---------------------------------------------------------------- combine: y = sum_i G_i E_i(x)

def dense_mixture(t, x, dtype, E):
    """sum_e softmax(l)_e * E_e(x): dense loops, no sorting, no permutation."""
    x64, w64 = widen(x, dtype), t["w_router"].astype(np.float64)
    out = np.zeros_like(x64)
    for tok in range(x.shape[0]):
        sm = scipy.special.softmax(x64[tok] @ w64)
        for e in range(E):
            out[tok] += sm[e] * np_ffn(x64[tok], widen(t["w_gate"][e], dtype), widen(t["w_up"][e], dtype), widen(t["w_down"][e], dtype))
    return out


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_k_equals_E_is_dense_softmax_mixture(dtype):
    ly, t, x = tiny_layer(dtype, d=128, E=6, F=16)
    r = O.moe_layer(ly, x, 6)
    assert np.allclose(r.out, dense_mixture(t, x, dtype, 6), rtol=1e-5, atol=1e-7)   # gates are stored fp32


def test_k1_is_the_argmax_expert():
    ly, t, x = tiny_layer("f32", d=128, E=6, F=16)
    r = O.moe_layer(ly, x, 1)
    x64 = x.astype(np.float64)
    for tok in range(x.shape[0]):
        e = int(np.argmax(r.logits[tok]))
        ref = np_ffn(x64[tok], *(t[n][e].astype(np.float64) for n in ("w_gate", "w_up", "w_down")))
        assert np.allclose(r.out[tok], ref, rtol=1e-12, atol=1e-14)


def test_identical_experts_give_one_expert_for_every_k():
    ly, t, x = tiny_layer("f32", d=128, E=5, F=16)
    same = {n: np.repeat(t[n][:1], 5, axis=0) for n in ("w_gate", "w_up", "w_down")}
    ly2 = O.Layer(128, 5, 16, "f32", t["w_router"], same["w_gate"], same["w_up"], same["w_down"])
    ref = O.moe_layer(ly2, x, 1).out
    for k in (2, 3, 5):
        assert np.allclose(O.moe_layer(ly2, x, k).out, ref, rtol=1e-6, atol=1e-9)  # gates sum to 1 (fp32-stored)


def test_general_k_against_independent_composition_and_linearity():
    ly, t, x = tiny_layer("bf16", d=128, E=8, F=16, bias=True)
    x64 = widen(x, "bf16")
    for k in (2, 3):
        r = O.moe_layer(ly, x, k)
        for tok in range(x.shape[0]):
            order = brute_topk(r.logits[tok], k)
            assert list(r.topk_idx[tok]) == order
            z = np.array([float(r.logits[tok][e]) for e in order])
            gte = np.exp(z - z.max()); gte /= gte.sum()
            ref = sum(gte[s] * np_ffn(x64[tok], *(widen(t[n][order[s]], "bf16") for n in ("w_gate", "w_up", "w_down")))
                      for s in range(k))
            assert np.allclose(r.out[tok], ref, rtol=1e-5, atol=1e-8)
    # linear in Wdown: doubling it (exact in bf16) doubles the output exactly
    wd2 = G.f32_to_bf16_bits(2.0 * G.bf16_bits_to_f32(t["w_down"]))
    ly2 = O.Layer(128, 8, 16, "bf16", t["w_router"], t["w_gate"], t["w_up"], wd2, router_bias=t["router_bias"])
    assert np.array_equal(O.moe_layer(ly2, x, 3).out, 2.0 * O.moe_layer(ly, x, 3).out)


def test_token_subset_equals_rows_of_full_result():
    ly, t, x = tiny_layer("bf16", d=128, E=8, F=16)
    full = O.moe_layer(ly, x, 2, round_act=True)
    sub = O.moe_layer(ly, x, 2, tokens=[7, 0, 3], round_act=True)
    assert np.array_equal(sub.out, full.out[[7, 0, 3]])
    assert np.array_equal(sub.topk_idx, full.topk_idx) and np.array_equal(sub.perm, full.perm)


# ---------------------------------------------------------------- shared expert

def test_shared_sigmoid_gate_zero_weight_is_half():
    ly, t, x = tiny_layer("f32", d=128, E=4, F=8, F_shared=16, shared_kind=2)
    ly0 = O.Layer(128, 4, 8, "f32", t["w_router"], t["w_gate"], t["w_up"], t["w_down"], F_shared=16, shared_kind=2,
                  ws_gate=t["ws_gate"], ws_up=t["ws_up"], ws_down=t["ws_down"], w_shared_gate=np.zeros(128, np.float32))
    assert O.shared_coeff(ly0, x, 3) == 0.5
    routed = O.Layer(128, 4, 8, "f32", t["w_router"], t["w_gate"], t["w_up"], t["w_down"])
    r0, rr = O.moe_layer(ly0, x, 2), O.moe_layer(routed, x, 2)
    x64 = x.astype(np.float64)
    for tok in range(x.shape[0]):
        sh = np_ffn(x64[tok], *(t[n].astype(np.float64) for n in ("ws_gate", "ws_up", "ws_down")))
        assert np.allclose(r0.out[tok], rr.out[tok] + 0.5 * sh, rtol=1e-12, atol=1e-14)
    # general gate value: logistic function of the dot product
    z = x64[5] @ t["w_shared_gate"].astype(np.float64)
    assert abs(O.shared_coeff(ly, x, 5) - scipy.special.expit(z)) < 1e-15


def test_two_ungated_shared_experts_equal_one_concatenated():
    ly, t, x = tiny_layer("bf16", d=128, E=4, F=8, F_shared=32, shared_kind=1)
    routed = O.Layer(128, 4, 8, "bf16", t["w_router"], t["w_gate"], t["w_up"], t["w_down"])
    r, rr = O.moe_layer(ly, x, 2), O.moe_layer(routed, x, 2)
    x64 = widen(x, "bf16")
    wg, wu, wd = (widen(t[n], "bf16") for n in ("ws_gate", "ws_up", "ws_down"))
    for tok in range(x.shape[0]):
        two = np_ffn(x64[tok], wg[:16], wu[:16], wd[:, :16]) + np_ffn(x64[tok], wg[16:], wu[16:], wd[:, 16:])
        assert np.allclose(r.out[tok], rr.out[tok] + two, rtol=1e-11, atol=1e-13)
        assert O.shared_coeff(ly, x, tok) == 1.0


# ---------------------------------------------------------------- stack with a per-layer k vector

def test_stack_is_per_layer_calls_with_k_vec():
    cfg = S.mini(S.C5, L=3, d=128, F=32, F_shared=64)
    layers = [O.Layer.from_tensors(cfg, S.host_layer(cfg, l)) for l in range(cfg.L)]
    xs = [S.host_x(cfg, l, 6) for l in range(cfg.L)]
    kv = [2, 5, 3]
    res = O.moe_stack(layers, xs, kv, round_act=True)
    for l in range(cfg.L):
        one = O.moe_layer(layers[l], xs[l], kv[l], round_act=True)
        assert np.array_equal(res[l].out, one.out) and np.array_equal(res[l].topk_idx, one.topk_idx)
    # UpdateTopk changes k only: calling k=5 after k=2 on the same layer object gives the k=5 result again
    a = O.moe_layer(layers[0], xs[0], 5).out
    O.moe_layer(layers[0], xs[0], 2)
    assert np.array_equal(O.moe_layer(layers[0], xs[0], 5).out, a)
    # the Zipf bias skews the load: experts are far from uniformly used
    r = O.moe_layer(layers[0], S.host_x(cfg, 0, 512), 6, routing_only=True)
    assert r.counts.max() > 4 * max(1, np.median(r.counts))


def test_bad_k_is_rejected():
    ly, t, x = tiny_layer("f32", d=128, E=4, F=8)
    for k in (0, 5, -1):
        with pytest.raises(RuntimeError):
            O.moe_layer(ly, x, k)


# ---------------------------------------------------------------- Stage-1 perturbation profiling (Algorithm 1)
def _tiny_layer(rng, d=128, E=6, F=64, identical=False):
    wg = rng.normal(0, 0.3, (E, F, d)).astype(np.float32)
    wu = rng.normal(0, 0.3, (E, F, d)).astype(np.float32)
    wd = rng.normal(0, 0.3, (E, d, F)).astype(np.float32)
    if identical:
        wg[:], wu[:], wd[:] = wg[0], wu[0], wd[0]
    return O.Layer(d, E, F, "f32", rng.normal(0, 0.5, (d, E)).astype(np.float32), wg, wu, wd)


def test_profile_delta_is_zero_at_k_base_and_for_identical_experts():
    """Delta_{k_base} = 0 exactly; with identical experts every k gives E_0(x) (gates sum to 1), so every Delta is 0 up
    to the fp32 storage of the gates (2^-24 relative per gate)."""
    rng = np.random.default_rng(21)
    x = rng.normal(0, 1, (9, 128)).astype(np.float32)
    ly = _tiny_layer(rng)
    d = O.profile_layer(ly, x, 4, [1, 2, 3, 4])
    assert d[3] == 0.0 and np.all(d[:3] > 0)
    same = _tiny_layer(rng, identical=True)
    ref = np.sqrt(np.sum(O.moe_layer(same, x, 4).out ** 2))
    assert np.all(O.profile_layer(same, x, 4, [1, 2, 3]) <= 1e-6 * ref)


def test_profile_delta_matches_the_closed_form_in_the_dropped_experts():
    """Y_k - Y_base = sum_s (g_k[s]*[s<k] - g_base[s]) * E_{sel_s}(x): recomputed here from the gates' closed form
    (softmax over prefixes of the selected logits) and per-expert outputs, without calling the profiling function."""
    rng = np.random.default_rng(22)
    T, kb = 7, 5
    x = rng.normal(0, 1, (T, 128)).astype(np.float32)
    ly = _tiny_layer(rng, E=6)
    base = O.moe_layer(ly, x, kb)
    got = O.profile_layer(ly, x, kb, [1, 3])
    for i, k in enumerate((1, 3)):
        total = 0.0
        for t in range(T):
            sel = base.topk_idx[t]
            l = base.logits[t][sel].astype(np.float64)
            gb = np.exp(l - l[0]) / np.exp(l - l[0]).sum()
            gk = np.zeros(kb)
            gk[:k] = np.exp(l[:k] - l[0]) / np.exp(l[:k] - l[0]).sum()
            diff = sum((gk[s] - gb[s]) * O.expert_ffn(ly, int(sel[s]), x, t) for s in range(kb))
            total += float(np.sum(diff ** 2))
        assert abs(got[i] - np.sqrt(total)) <= 1e-6 * np.sqrt(total)   # the oracle stores its gates in fp32


# ---------------------------------------------------------------- chained residual stack
def test_bf16_rounding_helper_matches_exhaustive_definition():
    """bf16_rne against the definition (nearest representable, ties to even mantissa) on values around boundaries."""
    vals = np.array([1.0, 1.00390625, 1.0078125, 1.01171875, 1.005859375, -2.5, 3.1415927, 1e-20, 65504.0], dtype=np.float32)
    got = O.bf16_to_f64(O.bf16_rne(vals))
    for v, g in zip(vals.astype(np.float64), got):
        lo = np.float32(v).view(np.uint32) & np.uint32(0xFFFF0000)
        c0 = float(np.uint32(lo).view(np.float32))
        c1 = float(np.uint32(lo + np.uint32(0x10000)).view(np.float32))
        best = min((abs(v - c0), (lo >> 16) & 1, c0), (abs(v - c1), ((lo >> 16) + 1) & 1, c1))[2]
        assert g == best


def test_chained_stack_special_cases():
    """Zero down-projections leave the hidden state untouched; one layer equals x + f(norm(x)); the normalised input
    has unit mean square."""
    rng = np.random.default_rng(31)
    x = rng.normal(0, 3.0, (6, 128)).astype(np.float32)
    ly = _tiny_layer(rng)
    u = O.rms_norm(x)
    assert np.allclose(np.mean(u * u, axis=1), 1.0, atol=1e-6)
    assert np.allclose(O.rms_norm(1000.0 * x), u, rtol=0, atol=1e-6)          # scale-invariant up to the epsilon
    hand = O.rms_norm(np.array([[3.0, -4.0, 0.0, 0.0]]))                       # mean square 25/4
    assert np.allclose(hand, np.array([[3.0, -4.0, 0.0, 0.0]]) / np.sqrt(6.25 + 1e-6), rtol=1e-15)
    assert abs(hand[0, 0] - 1.2) < 1e-6 and abs(hand[0, 1] + 1.6) < 1e-6
    hs = O.chained_stack([ly], x, [3])
    direct = x.astype(np.float64) + O.moe_layer(ly, u.astype(np.float32), 3).out
    assert np.array_equal(hs[0], direct)
    zero = O.Layer(128, 6, 64, "f32", ly.w_router, ly.w_gate, ly.w_up, np.zeros_like(ly.w_down))
    hs = O.chained_stack([zero, zero, zero], x, [1, 2, 3])
    assert np.array_equal(hs[-1], x.astype(np.float64))


def test_chained_layer_teacher_forcing_uses_the_given_input():
    rng = np.random.default_rng(32)
    x = rng.normal(0, 1.0, (5, 128)).astype(np.float32)
    ly = _tiny_layer(rng)
    forced = rng.normal(0, 1.0, (5, 128)).astype(np.float32)
    h1, u, res = O.chained_layer(ly, x, 2, u_forced=forced)
    assert u is forced and np.array_equal(h1, x.astype(np.float64) + O.moe_layer(ly, forced, 2).out)
