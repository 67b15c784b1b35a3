// LExI Stage 2 (paper Algorithm 2): evolutionary allocation of the per-layer top-k under a total budget, guided by
// the Stage-1 losses.  Host code only (the search runs on the loss table alone and needs no model weights, Sec. 4): nothing here touches the GPU.
//
// The paper leaves several steps open; the reading implemented here:
//   population   n_pop feasible vectors: the flattest vector with sum B, then 4*L random balanced +-1 moves each
//   fitness      phi(k) = sum_j D[j][k_j], lower is better
//   parents      two tournaments of size 2 (the fitter of two random individuals, ties to the lower index)
//   crossover    uniform, alpha_j ~ Bernoulli(0.5)
//   mutation     for every layer j with probability eta_mut: a random partner i != j, k_j += 1, k_i -= 1; a layer moves
//                at most once per mutation, so every Delta_j is in {-1, 0, +1} and the Deltas sum to 0
//   projection   clamp to [k_min, k_max]; while the sum exceeds B decrement the layer whose loss rises least, while it
//                is below B increment the layer whose loss falls most (ties to the lower index)
//   update       the offspring joins; beyond n_pop the worst individual leaves (ties: the highest index)
//   result       the individual with the lowest phi (ties to the lower index)
// Random numbers: draw(i) = SplitMix64 output function of (seed + i * 0x9E3779B97F4A7C15), i = 0, 1, 2, ... in
// consumption order; an integer below n is ((draw >> 32) * n) >> 32; Bernoulli(p) is (draw >> 11) * 2^-53 < p.
#include "../../include/lexi_moe.h"

#include <cstdint>
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

struct Problem {
    const double* D;
    int L, B, k_min, k_max;
    double loss(int j, int k) const { return D[(size_t)j * (k_max + 1) + k]; }
    double phi(const std::vector<int>& k) const {
        double s = 0.0;
        for (int j = 0; j < L; ++j) s += loss(j, k[j]);
        return s;
    }
    void project(std::vector<int>& k) const {
        int sum = 0;
        for (int j = 0; j < L; ++j) {
            k[j] = k[j] < k_min ? k_min : (k[j] > k_max ? k_max : k[j]);
            sum += k[j];
        }
        while (sum > B) {
            int best = -1;
            double best_cost = 0.0;
            for (int j = 0; j < L; ++j)
                if (k[j] > k_min) {
                    const double cost = loss(j, k[j] - 1) - loss(j, k[j]);
                    if (best < 0 || cost < best_cost) { best = j; best_cost = cost; }
                }
            --k[best];
            --sum;
        }
        while (sum < B) {
            int best = -1;
            double best_gain = 0.0;
            for (int j = 0; j < L; ++j)
                if (k[j] < k_max) {
                    const double gain = loss(j, k[j]) - loss(j, k[j] + 1);
                    if (best < 0 || gain > best_gain) { best = j; best_gain = gain; }
                }
            ++k[best];
            ++sum;
        }
    }
};

}  // namespace

extern "C" lexi_status lexi_allocate_topk(const double* D, int32_t L, int32_t B, int32_t k_min, int32_t k_max,
                                          int32_t n_pop, int32_t g_max, double eta_mut, uint64_t seed, int32_t* k_out,
                                          double* phi_out) {
    if (!D || !k_out) return LEXI_ERR_NULL;
    if (L < 1 || k_min < 1 || k_max < k_min || n_pop < 2 || g_max < 0) return LEXI_ERR_SHAPE;
    if ((int64_t)B < (int64_t)L * k_min || (int64_t)B > (int64_t)L * k_max) return LEXI_ERR_BAD_K;
    const Problem pb{D, L, B, k_min, k_max};
    Stream rng(seed);
    std::vector<std::vector<int>> pop;
    for (int n = 0; n < n_pop; ++n) {
        std::vector<int> k(L);
        for (int j = 0; j < L; ++j) k[j] = B / L + (j < B % L ? 1 : 0);
        for (int m = 0; m < 4 * L; ++m) {
            const int i = rng.below(L), j = rng.below(L);
            if (i != j && k[i] < k_max && k[j] > k_min) { ++k[i]; --k[j]; }
        }
        pop.push_back(k);
    }
    std::vector<double> phi;
    auto evaluate = [&]() {
        phi.resize(pop.size());
        for (size_t q = 0; q < pop.size(); ++q) phi[q] = pb.phi(pop[q]);
    };
    for (int g = 0; g < g_max; ++g) {
        evaluate();
        const std::vector<int>* parent[2];
        for (int t = 0; t < 2; ++t) {
            const int a = rng.below((int)pop.size()), b = rng.below((int)pop.size());
            const int lo = a < b ? a : b, hi = a < b ? b : a;
            parent[t] = phi[hi] < phi[lo] ? &pop[hi] : &pop[lo];
        }
        std::vector<int> child(L);
        for (int j = 0; j < L; ++j) child[j] = rng.bernoulli(0.5) ? (*parent[0])[j] : (*parent[1])[j];
        std::vector<char> touched(L, 0);
        for (int j = 0; j < L; ++j)
            if (rng.bernoulli(eta_mut)) {
                int i = rng.below(L - 1);
                i += i >= j;
                if (!touched[i] && !touched[j]) {
                    ++child[j];
                    --child[i];
                    touched[i] = touched[j] = 1;
                }
            }
        pb.project(child);
        pop.push_back(child);
        if ((int)pop.size() > n_pop) {
            evaluate();
            size_t worst = 0;
            for (size_t q = 1; q < pop.size(); ++q)
                if (phi[q] >= phi[worst]) worst = q;   // ties: the highest index leaves
            pop.erase(pop.begin() + (long)worst);
        }
    }
    evaluate();
    size_t best = 0;
    for (size_t q = 1; q < pop.size(); ++q)
        if (phi[q] < phi[best]) best = q;
    for (int j = 0; j < L; ++j) k_out[j] = pop[best][j];
    if (phi_out) *phi_out = phi[best];
    return LEXI_OK;
}
