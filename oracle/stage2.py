"""Oracle for LExI Stage 2 (paper Algorithm 2): evolutionary allocation of the per-layer top-k under a budget.

Test infrastructure only (see the package header).  Plain Python, the algorithm's steps in the paper's order and
notation.  The paper leaves several steps open; the reading taken here is:

  population   N_pop feasible vectors: the flattest vector with sum B, then 4*L random balanced +-1 moves each
  fitness      phi(k) = sum_j D[j][k_j]                                   (lower is better)
  parents      two tournaments of size 2 (two random individuals, the fitter wins, ties to the lower index)
  crossover    uniform: k'_j = p1_j if alpha_j else p2_j, alpha_j ~ Bernoulli(0.5)
  mutation     for every layer j, with probability eta_mut: a random partner i != j; k_j += 1, k_i -= 1
               (Delta in {-1, 0, +1}, sum 0: a layer already touched in this mutation is left alone; a single layer
               has no partner, so with L = 1 the step does nothing and draws nothing)
  projection   clamp to [k_min, k_max]; then, while the sum is above B, decrement the layer whose loss rises least,
               while it is below B, increment the layer whose loss falls most (ties to the lower index)
  update       the offspring joins the population; above N_pop the worst individual leaves (ties: highest index)
  result       argmin phi over the final population (ties to the lower index)

Random numbers: one counter-based stream, draw(i) = splitmix64 output function of (seed + i * 0x9E3779B97F4A7C15),
i = 0, 1, 2, ... in the order the steps above consume them; integers in [0, n) as ((draw >> 32) * n) >> 32,
Bernoulli(p) as (draw >> 11) * 2^-53 < p.
"""
import numpy as np

MASK = (1 << 64) - 1
GOLDEN = 0x9E3779B97F4A7C15


def _mix64(z):
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9 & MASK
    z = (z ^ (z >> 27)) * 0x94D049BB133111EB & MASK
    return z ^ (z >> 31)


class _Stream:
    def __init__(self, seed):
        self.seed, self.i = seed & MASK, 0

    def draw(self):
        v = _mix64((self.seed + self.i * GOLDEN) & MASK)
        self.i += 1
        return v

    def below(self, n):
        return ((self.draw() >> 32) * n) >> 32

    def bernoulli(self, p):
        return (self.draw() >> 11) * 2.0 ** -53 < p


def fitness(D, k):
    return float(sum(D[j][k[j]] for j in range(len(k))))


def project(D, k, B, k_min, k_max):
    k = [min(max(v, k_min), k_max) for v in k]
    L = len(k)
    while sum(k) > B:
        best, best_cost = -1, None
        for j in range(L):
            if k[j] > k_min:
                cost = D[j][k[j] - 1] - D[j][k[j]]
                if best_cost is None or cost < best_cost:
                    best, best_cost = j, cost
        k[best] -= 1
    while sum(k) < B:
        best, best_gain = -1, None
        for j in range(L):
            if k[j] < k_max:
                gain = D[j][k[j]] - D[j][k[j] + 1]
                if best_gain is None or gain > best_gain:
                    best, best_gain = j, gain
        k[best] += 1
    return k


def initial_population(rng, L, B, k_min, k_max, n_pop):
    """N_pop feasible vectors: the flattest vector with sum B, then 4*L random balanced +-1 moves each."""
    pop = []
    for _ in range(n_pop):
        k = [B // L + (1 if j < B % L else 0) for j in range(L)]
        for _ in range(4 * L):
            i, j = rng.below(L), rng.below(L)
            if i != j and k[i] < k_max and k[j] > k_min:
                k[i] += 1
                k[j] -= 1
        pop.append(k)
    return pop


def tournament(rng, phi):
    """Index of one parent: two random individuals are drawn, the one with the lower phi wins (ties: lower index)."""
    a, b = rng.below(len(phi)), rng.below(len(phi))
    lo, hi = min(a, b), max(a, b)
    return hi if phi[hi] < phi[lo] else lo


def crossover(rng, p1, p2):
    """Uniform crossover: k'_j = alpha_j p1_j + (1 - alpha_j) p2_j with alpha_j ~ Bernoulli(0.5)."""
    return [p1[j] if rng.bernoulli(0.5) else p2[j] for j in range(len(p1))]


def mutate(rng, child, eta_mut):
    """Balanced mutation: every layer j, with probability eta_mut, takes +1 and a random partner i != j takes -1; a
    layer moves at most once, so every Delta_j is in {-1, 0, +1} and the Deltas sum to 0.  With a single layer there
    is no partner and nothing moves (and nothing is drawn)."""
    L = len(child)
    child = list(child)
    if L < 2:
        return child
    touched = [False] * L
    for j in range(L):
        if rng.bernoulli(eta_mut):
            i = rng.below(L - 1)
            i += i >= j
            if not touched[i] and not touched[j]:
                child[j] += 1
                child[i] -= 1
                touched[i] = touched[j] = True
    return child


def allocate_topk(D, B, k_min, k_max, n_pop, g_max, eta_mut, seed):
    """D: [L][k_max + 1] losses (entry [j][k] for k_min <= k <= k_max).  Returns (k*, phi(k*))."""
    D = np.asarray(D, dtype=np.float64)
    L = D.shape[0]
    if not (L * k_min <= B <= L * k_max) or n_pop < 2:
        raise ValueError("infeasible budget or population")
    rng = _Stream(seed)
    pop = initial_population(rng, L, B, k_min, k_max, n_pop)
    for _ in range(g_max):
        phi = [fitness(D, k) for k in pop]
        p1 = pop[tournament(rng, phi)]
        p2 = pop[tournament(rng, phi)]
        child = crossover(rng, p1, p2)
        child = mutate(rng, child, eta_mut)
        child = project(D, child, B, k_min, k_max)
        pop.append(child)
        if len(pop) > n_pop:
            phi = [fitness(D, k) for k in pop]
            worst = max(range(len(pop)), key=lambda q: (phi[q], q))
            pop.pop(worst)
    phi = [fitness(D, k) for k in pop]
    best = min(range(len(pop)), key=lambda q: (phi[q], q))
    return np.asarray(pop[best], dtype=np.int32), phi[best]
