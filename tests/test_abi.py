"""The C-ABI library: loads, exports every declared symbol, and rejects bad arguments before touching the GPU."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    """Every function any header under include/ declares."""
    names = set()
    inc = os.path.join(ROOT, "include")
    for fn in sorted(os.listdir(inc)):
        if fn.endswith(".h"):
            text = re.sub(r"/\*.*?\*/", "", open(os.path.join(inc, fn)).read(), flags=re.S)
            names |= set(re.findall(r"\b(lexi_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    import paper_2509_02753_amd as P
    names = declared_functions()
    assert set(names) == set(P.EXPORTS)
    lib = ctypes.CDLL(P.LIB_PATH)
    for n in names:
        assert getattr(lib, n) is not None
    assert P.version().startswith("lexi-moe")
    assert P.strerror(0) == "ok" and "k" in P.strerror(-3)


def fake_layer(P, **over):
    """A lexi_layer_t with plausible shapes and fake (never dereferenced) aligned device addresses."""
    f = dict(d=256, E=8, F=128, F_shared=0, dtype=P.LEXI_BF16, shared_kind=0, w_router=0x10000, router_bias=None,
             w_gate=0x20000, w_up=0x30000, w_down=0x40000, ws_gate=None, ws_up=None, ws_down=None, w_shared_gate=None)
    f.update(over)
    from paper_2509_02753_amd.binding import lexi_layer_t
    return lexi_layer_t(*[f[n] for n, _ in lexi_layer_t._fields_])


def call_layer(P, ly, x=0x50000, y=0x60000, y_dtype=0, T=16, k=2, ws=0x70000, ws_bytes=1 << 40):
    from paper_2509_02753_amd.binding import _lib
    return _lib.lexi_moe_layer_forward(ctypes.byref(ly), x, y, y_dtype, T, k, ws, ws_bytes, None, None)


def test_argument_validation_returns_codes_without_launching():
    """Every case fails validation (or is T == 0), so no kernel is launched and no GPU is needed."""
    import paper_2509_02753_amd as P
    ok = fake_layer(P)
    assert call_layer(P, ok, T=0) == 0                                   # T = 0: nothing to do
    assert call_layer(P, ok, k=0) == -3 and call_layer(P, ok, k=9) == -3 and call_layer(P, ok, k=-1) == -3
    assert call_layer(P, ok, T=-1) == -2
    assert call_layer(P, ok, x=None) == -1 and call_layer(P, ok, y=None) == -1 and call_layer(P, ok, ws=None) == -1
    assert call_layer(P, ok, x=0x50004) == -6 and call_layer(P, ok, ws=0x70008) == -6
    assert call_layer(P, ok, y_dtype=7) == -4
    assert call_layer(P, ok, ws_bytes=1024) == -5
    assert call_layer(P, fake_layer(P, E=65)) == -2 and call_layer(P, fake_layer(P, E=0)) == -2
    assert call_layer(P, fake_layer(P, d=192)) == -2 and call_layer(P, fake_layer(P, F=100)) == -2
    assert call_layer(P, fake_layer(P, dtype=3)) == -4
    assert call_layer(P, fake_layer(P, w_gate=None)) == -1
    assert call_layer(P, fake_layer(P, w_up=0x30002)) == -6
    assert call_layer(P, fake_layer(P, F_shared=128, shared_kind=1)) == -1          # shared weights missing
    assert call_layer(P, fake_layer(P, F_shared=128, shared_kind=0)) == -2          # width without a kind
    assert call_layer(P, fake_layer(P, F_shared=128, shared_kind=2, ws_gate=0x80000, ws_up=0x90000,
                                    ws_down=0xA0000)) == -1                         # sigmoid gate vector missing
    assert call_layer(P, ok, T=1 << 23, k=2) == -2                                  # T*k >= 2^24
    assert call_layer(P, fake_layer(P, F=65536), T=16384, k=2) == -2                # intermediate of 4 GiB or more
    assert call_layer(P, fake_layer(P, d=65536), T=32768, k=1) == -2                # x of 4 GiB or more


def test_profile_entry_point_validates_before_launching():
    """lexi_moe_profile_layer applies the limits of the forward entry points up front (fake pointers: any launch
    would fail, so a validation code coming back shows nothing was enqueued)."""
    import paper_2509_02753_amd as P
    from paper_2509_02753_amd.binding import _lib

    def prof(ly, T=16, k_base=2, k_list=(1, 2), x=0x50000, delta=0x60000, ws=0x70000, ws_bytes=1 << 40):
        kl = (ctypes.c_int32 * len(k_list))(*k_list)
        return _lib.lexi_moe_profile_layer(ctypes.byref(ly), x, T, k_base, kl, len(k_list), delta, ws, ws_bytes, None)

    ok = fake_layer(P)
    assert prof(ok, T=0) == -2 and prof(ok, k_base=0) == -3 and prof(ok, k_base=9) == -3
    assert prof(ok, k_list=(3,)) == -3                                     # a listed k above k_base
    assert prof(ok, x=None) == -1 and prof(ok, delta=None) == -1 and prof(ok, ws=None) == -1
    assert prof(ok, ws_bytes=1024) == -5
    assert prof(ok, T=1 << 23) == -2                                       # T*k >= 2^24
    assert prof(fake_layer(P, F=65536), T=16384) == -2                     # intermediate of 4 GiB or more
    assert prof(fake_layer(P, d=65536), T=32768, k_base=1, k_list=(1,)) == -2   # x of 4 GiB or more


def test_static_scratch_entry_point_validates_before_launching():
    """lexi_moe_layer_forward_static: the same argument checks, and a call that needs more than the library's 64 MiB
    static scratch is refused with LEXI_ERR_WORKSPACE (fake pointers: nothing may be launched)."""
    import paper_2509_02753_amd as P
    from paper_2509_02753_amd.binding import _lib
    call = lambda ly, x=0x50000, y=0x60000, y_dtype=0, T=16, k=2: _lib.lexi_moe_layer_forward_static(
        ctypes.byref(ly), x, y, y_dtype, T, k, None, None)
    ok = fake_layer(P)
    assert call(ok, T=0) == 0
    assert call(ok, k=0) == -3 and call(ok, T=-1) == -2 and call(ok, x=None) == -1 and call(ok, y=0x60004) == -6
    assert call(ok, y_dtype=5) == -4
    assert call(fake_layer(P, d=2048, F=1024, E=64), T=4096, k=8) == -5       # 353 MB of workspace


def test_down_gemm_plan_is_host_logic():
    """lexi_moe_down_plan only reads the layer's sizes: the schedule of every case the GPU schedule test runs, and of
    the full-size workloads, checked here without a GPU (0 streaming, 1 tiles, 2 split reduction, 3 direct rows)."""
    import paper_2509_02753_amd as P
    from paper_2509_02753_amd.binding import _lib
    shared = dict(ws_gate=0x80000, ws_up=0x90000, ws_down=0xA0000, w_shared_gate=0xB0000)

    def plan(T, k, which=0, **kw):
        ly = fake_layer(P, dtype=1, **kw)
        return _lib.lexi_moe_down_plan(ctypes.byref(ly), T, k, which)

    assert plan(1300, 2, d=1024, E=64, F=2048) == 2
    assert plan(2600, 1, d=1024, E=64, F=2048) == 3
    assert plan(1300, 2, d=1024, E=64, F=1024) == 1
    assert plan(700, 3, d=1024, E=60, F=384, F_shared=2048, shared_kind=2, **shared) == 1
    assert plan(700, 3, 1, d=1024, E=60, F=384, F_shared=2048, shared_kind=2, **shared) == 2
    assert plan(3700, 2, d=1024, E=8, F=4096) == 2
    # full sizes: prefill runs plain tiles (several rounds of work items), decode streams the weights
    assert plan(4096, 2, d=4096, E=8, F=14336) == 1 and plan(32, 2, d=4096, E=8, F=14336) == 0
    # a handful of tokens (T <= 8, T*k <= 64, no sigmoid-gated shared expert): the combine rides in the down launch
    assert plan(1, 6, d=2048, E=64, F=1408, F_shared=2816, shared_kind=1, ws_gate=0x80000, ws_up=0x90000,
                ws_down=0xA0000) == 4
    assert plan(8, 2, d=4096, E=8, F=14336) == 4 and plan(9, 2, d=4096, E=8, F=14336) == 0
    assert plan(8, 8, d=2048, E=64, F=1024) == 4 and plan(8, 9, d=2048, E=64, F=1024) == 0
    assert plan(16, 16, d=2048, E=64, F=1024) == 1     # enough work items for the tile schedule: not fused
    assert plan(4, 4, d=2048, E=60, F=1408, F_shared=5632, shared_kind=2, **shared) == 0
    assert plan(4096, 8, d=2048, E=64, F=1024) == 1 and plan(4096, 1, d=2048, E=64, F=1024) == 3
    assert plan(8192, 4, 1, d=2048, E=60, F=1408, F_shared=5632, shared_kind=2, **shared) == 1
    assert plan(64, 4, 1, d=2048, E=60, F=1408, F_shared=5632, shared_kind=2, **shared) == 0
    # a k = 1 layer with a shared expert still needs the combine
    assert plan(2600, 1, d=1024, E=60, F=2048, F_shared=2048, shared_kind=2, **shared) != 3
    assert plan(16, 1, 1, d=1024, E=8, F=2048) == -1 and plan(0, 1, d=1024, E=8, F=2048) == -1
    assert plan(16, 9, d=1024, E=8, F=2048) == -1


def test_workspace_query_is_monotone_and_checked():
    import paper_2509_02753_amd as P
    from paper_2509_02753_amd.binding import _lib, lexi_layer_t
    arr = (lexi_layer_t * 2)(fake_layer(P), fake_layer(P, F=256, F_shared=128, shared_kind=1, ws_gate=0x80000,
                                                       ws_up=0x90000, ws_down=0xA0000))
    q = lambda T, k: int(_lib.lexi_moe_workspace_bytes(arr, 2, T, k))
    assert q(64, 2) > 0 and q(128, 2) > q(64, 2) and q(64, 4) > q(64, 2)
    assert q(64, 9) == q(64, 8) and q(-1, 2) == 0 and q(64, 0) == 0     # k is capped by the layer's E (8 here)
    assert int(_lib.lexi_moe_workspace_bytes(None, 1, 64, 2)) == 0
    # a stack call validates every layer before launching: bad k in the second layer is reported, nothing runs
    kv = (ctypes.c_int32 * 2)(2, 0)
    st = _lib.lexi_moe_stack_forward(arr, 2, kv, 0x50000, 0, 0x60000, 64 * 256, 0, 64, 0, 0x70000, 1 << 40, None, None)
    assert st == -3
    kv = (ctypes.c_int32 * 2)(2, 2)
    call = lambda y_dtype, x_stride, mode: _lib.lexi_moe_stack_forward(
        arr, 2, kv, 0x50000, x_stride, 0x60000, 64 * 256, y_dtype, 64, mode, 0x70000, 1 << 40, None, None)
    assert call(0, 0, 2) == -4                       # unknown mode
    assert call(1, 0, 1) == -4                       # chained mode keeps the hidden state in fp32
    assert call(0, 64 * 256, 1) == -4                # chained mode has one input
    assert _lib.lexi_moe_stack_forward(arr, 2, kv, 0x50000, 0, 0x60000, 10, 0, 64, 0, 0x70000, 1 << 40, None, None) == -2
    assert _lib.lexi_moe_stack_forward(arr, 2, None, 0x50000, 0, 0x60000, 64 * 256, 0, 64, 0, 0x70000, 1 << 40, None, None) == -1


def test_product_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2509_02753_amd")
    for dirpath, _, files in os.walk(pkg):
        for fn in files:
            if fn.endswith((".py", ".hip", ".hpp", ".h", ".cpp")):
                src = open(os.path.join(dirpath, fn)).read()
                assert "oracle" not in src.lower(), f"{fn} mentions the oracle"
    src = open(os.path.join(ROOT, "oracle", "__init__.py")).read() + open(os.path.join(ROOT, "oracle", "lexi_oracle.c")).read()
    assert "paper_2509_02753_amd" not in src and "lexi_moe.h" not in src
