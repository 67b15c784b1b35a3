"""LExI Stage 2 (Algorithm 2): pins of the oracle, and the library's host implementation against the oracle."""
import ctypes
import itertools

import numpy as np
import pytest

from oracle import stage2 as O2


def random_table(rng, L, k_max, convex):
    """Losses that fall with k (D[j][k_max] = 0, as the profiling of Algorithm 1 gives at k = k_base)."""
    D = np.zeros((L, k_max + 1))
    for j in range(L):
        steps = np.sort(rng.uniform(0.1, 3.0, k_max)) if convex else rng.uniform(0.1, 3.0, k_max)   # convex: gains shrink as k grows
        for k in range(k_max - 1, -1, -1):
            D[j][k] = D[j][k + 1] + steps[k_max - 1 - k] * (1 + j % 3)
    return D


def brute_force(D, B, k_min, k_max):
    best = None
    for k in itertools.product(range(k_min, k_max + 1), repeat=D.shape[0]):
        if sum(k) == B:
            phi = sum(D[j][k[j]] for j in range(len(k)))
            if best is None or phi < best - 1e-12:
                best = phi
    return best


def test_oracle_result_is_feasible_and_never_worse_than_the_flat_vector():
    rng = np.random.default_rng(5)
    for L, k_min, k_max, B in ((16, 2, 8, 96), (24, 1, 4, 72), (32, 1, 2, 48), (26, 2, 6, 104)):
        D = random_table(rng, L, k_max, convex=False)
        k, phi = O2.allocate_topk(D, B, k_min, k_max, 32, 300, 0.1, seed=7)
        assert k.sum() == B and k.min() >= k_min and k.max() <= k_max
        flat = [B // L + (1 if j < B % L else 0) for j in range(L)]
        assert abs(phi - O2.fitness(D, k)) < 1e-12 and phi <= O2.fitness(D, flat) + 1e-12


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_oracle_reaches_the_exhaustive_optimum_on_tiny_instances(seed):
    """L = 5 layers, k in 1..4: 4^5 allocations enumerated; the search must end at the minimum of phi."""
    rng = np.random.default_rng(seed)
    D = random_table(rng, 5, 4, convex=False)
    for B in (8, 12, 15):
        _, phi = O2.allocate_topk(D, B, 1, 4, 32, 800, 0.2, seed=seed)
        assert abs(phi - brute_force(D, B, 1, 4)) < 1e-9


def test_oracle_equals_the_greedy_optimum_for_convex_losses():
    """With convex per-layer losses the optimum is the greedy one (take the B - L*k_min largest marginal gains)."""
    rng = np.random.default_rng(11)
    L, k_min, k_max, B = 12, 1, 6, 40
    D = random_table(rng, L, k_max, convex=True)
    gains = sorted((D[j][k] - D[j][k + 1] for j in range(L) for k in range(k_min, k_max)), reverse=True)
    opt = sum(D[j][k_min] for j in range(L)) - sum(gains[:B - L * k_min])
    _, phi = O2.allocate_topk(D, B, k_min, k_max, 32, 600, 0.15, seed=3)
    assert abs(phi - opt) < 1e-9


def test_projection_repairs_any_vector():
    rng = np.random.default_rng(2)
    D = random_table(rng, 8, 5, convex=False)
    for _ in range(50):
        k = rng.integers(-3, 9, 8).tolist()
        p = O2.project(D, k, 24, 1, 5)
        assert sum(p) == 24 and min(p) >= 1 and max(p) <= 5


def test_stream_is_the_published_splitmix64():
    """First outputs of SplitMix64 seeded with 1234567 (reference values of the published generator): the stream
    draw(i) = mix(seed + i*golden) is that generator's output i + 1... with its state pre-incremented, so draw(i) for
    seed s equals the published generator seeded with s - golden."""
    s = O2._Stream((1234567 + O2.GOLDEN) & O2.MASK)
    assert [s.draw() for _ in range(3)] == [6457827717110365317, 3203168211198807973, 9817491932198370423]


# ---------------------------------------------------------------- the library's host implementation
def _lib_allocate(D, B, k_min, k_max, n_pop, g_max, eta, seed):
    import paper_2509_02753_amd as P
    lib = ctypes.CDLL(P.LIB_PATH)
    if not hasattr(lib, "lexi_allocate_topk"):
        pytest.skip("library built without lexi_allocate_topk")
    lib.lexi_allocate_topk.restype = ctypes.c_int32
    lib.lexi_allocate_topk.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                       ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_double, ctypes.c_uint64,
                                       ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_double)]
    D = np.ascontiguousarray(D, dtype=np.float64)
    L = D.shape[0]
    out = (ctypes.c_int32 * L)()
    phi = ctypes.c_double()
    st = lib.lexi_allocate_topk(D.ctypes.data_as(ctypes.POINTER(ctypes.c_double)), L, B, k_min, k_max, n_pop, g_max, eta,
                                seed, out, ctypes.byref(phi))
    return st, np.array(list(out), dtype=np.int32), phi.value


@pytest.mark.parametrize("L,k_min,k_max,B,seed", [(16, 2, 8, 96, 1), (24, 1, 4, 72, 2), (32, 1, 2, 48, 3),
                                                   (26, 2, 6, 104, 4), (5, 1, 4, 12, 5), (40, 1, 2, 60, 6)])
def test_library_matches_the_oracle_exactly(L, k_min, k_max, B, seed):
    """Same table, same parameters, same seed: the same k vector, element by element (integer work: bit-exact)."""
    rng = np.random.default_rng(100 + seed)
    D = random_table(rng, L, k_max, convex=bool(seed % 2))
    k_ref, phi_ref = O2.allocate_topk(D, B, k_min, k_max, 24, 250, 0.1, seed=seed)
    st, k, phi = _lib_allocate(D, B, k_min, k_max, 24, 250, 0.1, seed)
    assert st == 0
    assert np.array_equal(k, k_ref)
    assert abs(phi - phi_ref) <= 1e-12 * max(1.0, abs(phi_ref))


def test_library_rejects_infeasible_arguments():
    D = np.zeros((4, 5))
    assert _lib_allocate(D, 100, 1, 4, 8, 10, 0.1, 1)[0] < 0      # budget above L * k_max
    assert _lib_allocate(D, 2, 1, 4, 8, 10, 0.1, 1)[0] < 0        # below L * k_min
    assert _lib_allocate(D, 8, 1, 4, 1, 10, 0.1, 1)[0] < 0        # population of one
    assert _lib_allocate(D, 8, 3, 2, 8, 10, 0.1, 1)[0] < 0        # k_min > k_max
