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


# ---------------------------------------------------------------- the steps of Algorithm 2, one by one
class _Scripted:
    """A stand-in random stream with the draws written out by hand, so that a step's outcome can be worked on paper."""
    def __init__(self, ints=(), coins=()):
        self.ints, self.coins = list(ints), list(coins)

    def below(self, n):
        v = self.ints.pop(0)
        assert 0 <= v < n
        return v

    def bernoulli(self, p):
        return self.coins.pop(0) < p      # coins are uniform numbers in [0, 1)


def test_tournament_returns_the_fitter_of_its_two_draws():
    """Algorithm 2, "Select parents via tournament": of the two individuals drawn the one with the lower phi wins,
    whichever was drawn first; equal phi goes to the lower index."""
    phi = [5.0, 1.0, 3.0, 1.0, 9.0]
    assert O2.tournament(_Scripted(ints=[0, 2]), phi) == 2
    assert O2.tournament(_Scripted(ints=[2, 0]), phi) == 2
    assert O2.tournament(_Scripted(ints=[4, 1]), phi) == 1
    assert O2.tournament(_Scripted(ints=[1, 3]), phi) == 1     # tie: lower index
    assert O2.tournament(_Scripted(ints=[3, 1]), phi) == 1
    assert O2.tournament(_Scripted(ints=[4, 4]), phi) == 4     # the same individual twice
    # against the real stream: the winner is one of the two drawn indices and no drawn index beats it
    for seed in range(40):
        probe = O2._Stream(seed)
        a, b = probe.below(len(phi)), probe.below(len(phi))
        w = O2.tournament(O2._Stream(seed), phi)
        assert w in (a, b) and phi[w] == min(phi[a], phi[b])


def test_crossover_takes_every_gene_from_one_of_the_parents():
    """Algorithm 2, "Apply Crossover": k'_j = alpha_j p1_j + (1 - alpha_j) p2_j, alpha_j in {0, 1}."""
    p1, p2 = [1, 1, 1, 1, 1, 1], [4, 4, 4, 4, 4, 4]
    c = O2.crossover(_Scripted(coins=[0.1, 0.9, 0.49, 0.5, 0.0, 0.99]), p1, p2)
    assert c == [1, 4, 1, 4, 1, 4]                              # alpha_j = 1 (coin < 0.5) takes p1
    for seed in range(20):
        q1, q2 = list(range(10)), list(range(100, 110))
        c = O2.crossover(O2._Stream(seed), q1, q2)
        assert all(c[j] in (q1[j], q2[j]) for j in range(10))
    mixed = [O2.crossover(O2._Stream(s), [0] * 64, [1] * 64) for s in range(8)]
    assert all(8 < sum(c) < 56 for c in mixed)                  # both parents contribute


def test_mutation_is_balanced_and_moves_a_layer_at_most_once():
    """Algorithm 2, "Apply Mutation": Delta_j in {-1, 0, +1} and sum_j Delta_j = 0, before any projection."""
    base = [5] * 12
    for seed in range(60):
        for eta in (0.05, 0.3, 1.0):
            m = O2.mutate(O2._Stream(seed), base, eta)
            delta = [m[j] - base[j] for j in range(12)]
            assert set(delta) <= {-1, 0, 1} and sum(delta) == 0
    assert O2.mutate(O2._Stream(1), base, 0.0) == base           # eta = 0: nothing moves
    assert any(O2.mutate(O2._Stream(s), base, 0.3) != base for s in range(5))
    # with eta = 1 every layer tries to move; layer 0 moves first, so it always ends at +1 and its partner at -1
    for seed in range(10):
        m = O2.mutate(O2._Stream(seed), base, 1.0)
        assert m[0] == 6 and sorted(set(m)) == [4, 5, 6][-len(set(m)):] and m.count(6) == m.count(4) >= 1
    # a hand-worked case: layers 0..3; layer 1 fires with partner draw 2 -> i = 3 (skips j); layer 3 fires with partner
    # draw 0 -> i = 0, but layer 3 has already moved, so nothing happens
    m = O2.mutate(_Scripted(ints=[2, 0], coins=[0.9, 0.0, 0.9, 0.0]), [3, 3, 3, 3], 0.5)
    assert m == [3, 4, 3, 2]
    # partner draw below j maps to itself: layer 2 fires, draw 1 -> partner 1
    m = O2.mutate(_Scripted(ints=[1], coins=[0.9, 0.9, 0.0, 0.9]), [3, 3, 3, 3], 0.5)
    assert m == [3, 2, 4, 3]


def test_single_layer_has_nothing_to_mutate():
    """L = 1: the only feasible vector is (B); the search returns it and the mutation step draws nothing."""
    D = np.array([[0.0, 3.0, 2.0, 1.0, 0.0]])
    s = O2._Stream(9)
    assert O2.mutate(s, [3], 0.9) == [3] and s.i == 0
    k, phi = O2.allocate_topk(D, 3, 1, 4, 4, 50, 0.9, seed=1)
    assert k.tolist() == [3] and phi == 1.0


def test_projection_hand_worked_cases():
    """Clamp, then one unit at a time: down where the loss rises least, up where it falls most, ties to the lower index."""
    D = np.array([[9.0, 6.0, 4.0, 3.0, 2.5],     # layer 0: gains 3, 2, 1, 0.5
                  [9.0, 8.0, 3.0, 2.0, 0.0],     # layer 1: gains 1, 5, 1, 2
                  [9.0, 5.0, 4.0, 1.0, 0.5]])    # layer 2: gains 4, 1, 3, 0.5
    # sum too high by 2, from (4, 4, 4): cheapest decrements are layer 0 (0.5) and layer 2 (0.5); tie -> layer 0 first
    assert O2.project(D, [4, 4, 4], 11, 1, 4) == [3, 4, 4]
    assert O2.project(D, [4, 4, 4], 10, 1, 4) == [3, 4, 3]
    # sum too low by 1 from (1, 1, 1): best gains are 2 (layer 0), 5 (layer 1), 1 (layer 2) -> layer 1
    assert O2.project(D, [1, 1, 1], 4, 1, 4) == [1, 2, 1]
    assert O2.project(D, [1, 1, 1], 5, 1, 4) == [2, 2, 1]       # next: gains 2, 1, 1 -> layer 0
    # clamping comes first: (9, -2, 2) -> (4, 1, 2), sum 7; budget 7 leaves it alone
    assert O2.project(D, [9, -2, 2], 7, 1, 4) == [4, 1, 2]
    # a feasible vector is a fixed point
    assert O2.project(D, [2, 3, 1], 6, 1, 4) == [2, 3, 1]


def test_one_generation_is_select_crossover_mutate_project_update_in_that_order():
    """Algorithm 2's generation, composed by hand from the steps pinned above on one shared stream, against the
    search run for one generation.  The seed is one where the mutation changes the child and the projected child is the
    new best, so a search that skipped or reordered a step would return something else."""
    L, k_min, k_max, B, n_pop, seed = 6, 1, 4, 14, 3, 3
    D = random_table(np.random.default_rng(77), L, k_max, convex=False)
    s = O2._Stream(seed)
    pop = O2.initial_population(s, L, B, k_min, k_max, n_pop)
    phi = [O2.fitness(D, k) for k in pop]
    p1 = pop[O2.tournament(s, phi)]
    p2 = pop[O2.tournament(s, phi)]
    crossed = O2.crossover(s, p1, p2)
    mutated = O2.mutate(s, crossed, 0.5)
    child = O2.project(D, mutated, B, k_min, k_max)
    assert mutated != crossed and child != O2.project(D, crossed, B, k_min, k_max)    # the mutation matters here
    assert O2.fitness(D, child) < min(phi) - 1e-9                                     # and the child is the new best
    k, f = O2.allocate_topk(D, B, k_min, k_max, n_pop, 1, 0.5, seed=seed)
    assert k.tolist() == child and abs(f - O2.fitness(D, child)) < 1e-12
    # zero generations: the best of the initial population
    k0, f0 = O2.allocate_topk(D, B, k_min, k_max, n_pop, 0, 0.5, seed=seed)
    assert k0.tolist() == pop[int(np.argmin(phi))] and abs(f0 - min(phi)) < 1e-12


def test_search_improves_on_its_initial_population():
    """Selection pressure: the result beats the best of the initial population on a table where that is possible."""
    rng = np.random.default_rng(21)
    D = random_table(rng, 16, 8, convex=True)
    pop = O2.initial_population(O2._Stream(4), 16, 96, 2, 8, 16)
    assert all(sum(k) == 96 and min(k) >= 2 and max(k) <= 8 for k in pop)
    start = min(O2.fitness(D, k) for k in pop)
    _, phi = O2.allocate_topk(D, 96, 2, 8, 16, 400, 0.1, seed=4)
    assert phi < start - 1e-9


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


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_library_reaches_the_exhaustive_optimum_on_tiny_instances(seed):
    """The library by itself (no oracle in the loop): 4^5 allocations enumerated, the search must end at the minimum."""
    rng = np.random.default_rng(seed)
    D = random_table(rng, 5, 4, convex=False)
    for B in (8, 12, 15):
        st, k, phi = _lib_allocate(D, B, 1, 4, 32, 800, 0.2, seed)
        assert st == 0 and k.sum() == B and k.min() >= 1 and k.max() <= 4
        assert abs(phi - brute_force(D, B, 1, 4)) < 1e-9
        assert abs(phi - sum(D[j][k[j]] for j in range(5))) < 1e-12


def test_library_result_is_feasible_never_worse_than_flat_and_greedy_optimal_for_convex_losses():
    rng = np.random.default_rng(5)
    for L, k_min, k_max, B in ((16, 2, 8, 96), (24, 1, 4, 72), (32, 1, 2, 48), (26, 2, 6, 104)):
        D = random_table(rng, L, k_max, convex=False)
        st, k, phi = _lib_allocate(D, B, k_min, k_max, 32, 300, 0.1, 7)
        assert st == 0 and k.sum() == B and k.min() >= k_min and k.max() <= k_max
        flat = [B // L + (1 if j < B % L else 0) for j in range(L)]
        assert phi <= sum(D[j][flat[j]] for j in range(L)) + 1e-12
    L, k_min, k_max, B = 12, 1, 6, 40
    D = random_table(np.random.default_rng(11), L, k_max, convex=True)
    gains = sorted((D[j][k] - D[j][k + 1] for j in range(L) for k in range(k_min, k_max)), reverse=True)
    opt = sum(D[j][k_min] for j in range(L)) - sum(gains[:B - L * k_min])
    st, k, phi = _lib_allocate(D, B, k_min, k_max, 32, 600, 0.15, 3)
    assert st == 0 and abs(phi - opt) < 1e-9


def test_library_single_layer():
    """L = 1 (one feasible vector): the mutation has no partner to draw and must not touch memory past the vector."""
    D = np.array([[0.0, 3.0, 2.0, 1.0, 0.0]])
    for B in (1, 3, 4):
        st, k, phi = _lib_allocate(D, B, 1, 4, 4, 50, 0.9, 1)
        assert st == 0 and k.tolist() == [B] and phi == D[0][B]
