// LExI Stage 2 (paper Algorithm 2): evolutionary allocation of the per-layer top-k under a total budget, guided by
// the Stage-1 losses.  Host code only (the search runs on the loss table alone and needs no model weights, Sec. 4): nothing here touches the GPU.
//
// The paper leaves several steps open; the reading implemented here:
//   population   n_pop feasible vectors: the flattest vector with sum B, then 4*L random balanced +-1 moves each
//   fitness      phi(k) = sum_j D[j][k_j], lower is better
//   parents      two tournaments of size 2 (the fitter of two random individuals, ties to the lower index)
//   crossover    uniform, alpha_j ~ Bernoulli(0.5)
//   mutation     for every layer j with probability eta_mut: a random partner i != j, k_j += 1, k_i -= 1; a layer moves
//                at most once per mutation, so every Delta_j is in {-1, 0, +1} and the Deltas sum to 0; a single
//                layer has no partner: with L = 1 the step moves nothing and draws nothing
//   projection   clamp to [k_min, k_max]; while the sum exceeds B decrement the layer whose loss rises least, while it
//                is below B increment the layer whose loss falls most (ties to the lower index)
//   update       the offspring joins; beyond n_pop the worst individual leaves (ties: the highest index)
//   result       the individual with the lowest phi (ties to the lower index)
// Random numbers: draw(i) = SplitMix64 output function of (seed + i * 0x9E3779B97F4A7C15), i = 0, 1, 2, ... in
// consumption order; an integer below n is ((draw >> 32) * n) >> 32; Bernoulli(p) is (draw >> 11) * 2^-53 < p.
#include "../../include/lexi_moe.h"

#include <cstdint>
#include <utility>
#include <vector>

namespace {

struct Stream {
    uint64_t seed, i = 0;
    explicit Stream(uint64_t s) : seed(s) {}
    uint64_t draw() {
        uint64_t z = seed + (i++) * 0x9E3779B97F4A7C15ull;
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
        return z ^ (z >> 31);
    }
    int below(int n) { return (int)(((draw() >> 32) * (uint64_t)n) >> 32); }
    bool bernoulli(double p) { return (double)(draw() >> 11) * 0x1.0p-53 < p; }
};

// The search keeps every individual's phi next to it: phi is evaluated once per individual (when it is created),
// a generation costs O(L + n_pop) instead of O(n_pop * L).
struct Individual {
    std::vector<int> k;
    double phi;
};

struct Search {
    const double* D;
    int L, B, k_min, k_max;
    Stream rng;
    std::vector<Individual> pop;

    double loss(int j, int k) const { return D[(size_t)j * (k_max + 1) + k]; }
    double phi(const std::vector<int>& k) const {
        double s = 0.0;
        for (int j = 0; j < L; ++j) s += loss(j, k[j]);
        return s;
    }

    // Flattest vector with sum B, shuffled by 4*L balanced moves that stay inside the box.
    std::vector<int> random_feasible() {
        std::vector<int> k(L);
        for (int j = 0; j < L; ++j) k[j] = B / L + (j < B % L ? 1 : 0);
        for (int m = 0; m < 4 * L; ++m) {
            const int up = rng.below(L), down = rng.below(L);
            if (up != down && k[up] < k_max && k[down] > k_min) { ++k[up]; --k[down]; }
        }
        return k;
    }

    // Tournament of two: the fitter of two random individuals; equal fitness goes to the lower index.
    const std::vector<int>& select_parent() {
        const int a = rng.below((int)pop.size()), b = rng.below((int)pop.size());
        const int first = a < b ? a : b, second = a < b ? b : a;
        return pop[pop[second].phi < pop[first].phi ? second : first].k;
    }

    // Uniform crossover followed by the balanced mutation (Algorithm 2: sum_j Delta_j = 0).
    std::vector<int> offspring(const std::vector<int>& p1, const std::vector<int>& p2, double eta_mut) {
        std::vector<int> c(L);
        for (int j = 0; j < L; ++j) c[j] = rng.bernoulli(0.5) ? p1[j] : p2[j];
        if (L < 2) return c;   // a balanced move needs two distinct layers
        std::vector<char> moved(L, 0);
        for (int j = 0; j < L; ++j) {
            if (!rng.bernoulli(eta_mut)) continue;
            int partner = rng.below(L - 1);
            if (partner >= j) ++partner;   // uniform over the other L - 1 layers
            if (moved[partner] || moved[j]) continue;
            ++c[j];
            --c[partner];
            moved[partner] = moved[j] = 1;
        }
        return c;
    }

    // Back into the feasible set: clamp, then repair the sum one unit at a time where it costs least / gains most.
    void project(std::vector<int>& k) const {
        int sum = 0;
        for (int j = 0; j < L; ++j) {
            k[j] = k[j] < k_min ? k_min : (k[j] > k_max ? k_max : k[j]);
            sum += k[j];
        }
        for (; sum > B; --sum) {
            int best = -1;
            double best_cost = 0.0;
            for (int j = 0; j < L; ++j) {
                if (k[j] <= k_min) continue;
                const double cost = loss(j, k[j] - 1) - loss(j, k[j]);
                if (best < 0 || cost < best_cost) { best = j; best_cost = cost; }
            }
            --k[best];
        }
        for (; sum < B; ++sum) {
            int best = -1;
            double best_gain = 0.0;
            for (int j = 0; j < L; ++j) {
                if (k[j] >= k_max) continue;
                const double gain = loss(j, k[j]) - loss(j, k[j] + 1);
                if (best < 0 || gain > best_gain) { best = j; best_gain = gain; }
            }
            ++k[best];
        }
    }

    // The offspring joins; the population stays at n_pop by dropping the worst (of equals: the newest).
    void insert_and_truncate(std::vector<int>&& k, int n_pop) {
        const double f = phi(k);
        pop.push_back(Individual{std::move(k), f});
        if ((int)pop.size() <= n_pop) return;
        size_t worst = 0;
        for (size_t q = 1; q < pop.size(); ++q)
            if (pop[q].phi >= pop[worst].phi) worst = q;
        pop.erase(pop.begin() + (long)worst);
    }
};

}  // namespace

extern "C" lexi_status lexi_allocate_topk(const double* D, int32_t L, int32_t B, int32_t k_min, int32_t k_max,
                                          int32_t n_pop, int32_t g_max, double eta_mut, uint64_t seed, int32_t* k_out,
                                          double* phi_out) {
    if (!D || !k_out) return LEXI_ERR_NULL;
    if (L < 1 || k_min < 1 || k_max < k_min || n_pop < 2 || g_max < 0) return LEXI_ERR_SHAPE;
    if ((int64_t)B < (int64_t)L * k_min || (int64_t)B > (int64_t)L * k_max) return LEXI_ERR_BAD_K;
    Search s{D, L, B, k_min, k_max, Stream(seed), {}};
    s.pop.reserve((size_t)n_pop + 1);
    for (int n = 0; n < n_pop; ++n) {
        std::vector<int> k = s.random_feasible();
        const double f = s.phi(k);
        s.pop.push_back(Individual{std::move(k), f});
    }
    for (int g = 0; g < g_max; ++g) {
        const std::vector<int>& p1 = s.select_parent();
        const std::vector<int>& p2 = s.select_parent();
        std::vector<int> child = s.offspring(p1, p2, eta_mut);
        s.project(child);
        s.insert_and_truncate(std::move(child), n_pop);
    }
    size_t best = 0;
    for (size_t q = 1; q < s.pop.size(); ++q)
        if (s.pop[q].phi < s.pop[best].phi) best = q;
    for (int j = 0; j < L; ++j) k_out[j] = s.pop[best].k[j];
    if (phi_out) *phi_out = s.pop[best].phi;
    return LEXI_OK;
}
