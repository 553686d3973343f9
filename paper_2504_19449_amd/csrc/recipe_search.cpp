// Host search for the sparsification recipe (R-Sparse, Sec. 3.5, "Search Algorithm for Sparsification
// Recipe"): differential-evolution style mutation and crossover over the per-layer shares rho_i of the
// sparse part, lowest-loss selection, optimised one group of layers at a time.  Plain host code; the
// loss (the paper uses the perplexity of the sparsified model on 16 calibration samples) is the caller's.
#include "../../include/rsparse.h"

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <new>
#include <vector>

namespace {

// u_k = (splitmix64(seed, k) >> 11) * 2^-53, k = 0, 1, 2, ... in the order the draws are made below.
struct Uniform {
    uint64_t seed, k = 0;
    explicit Uniform(uint64_t s) : seed(s) {}
    double operator()()
    {
        uint64_t z = seed + (k + 1) * 0x9E3779B97F4A7C15ull;
        ++k;
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
        z ^= z >> 31;
        return (double)(z >> 11) * (1.0 / 9007199254740992.0);
    }
};

struct Member {
    double loss;
    int age, index;          // age 0: current generation G, 1: offspring G_hat
    std::vector<double> rho;
};

}  // namespace

extern "C" rsparse_status rsparse_search_recipe(rsparse_loss_fn loss, void *user, int32_t n_layers, int32_t population,
                                                int32_t generations, double p_m, double p_c, int32_t group_size,
                                                uint64_t seed, double lo, double hi, const double *rho_start,
                                                double *rho_out, double *loss_out, double *history_out)
{
    if (!loss || !rho_out || !loss_out) return RSPARSE_EINVAL;
    if (n_layers < 1 || population < 1 || generations < 0 || group_size < 1) return RSPARSE_EINVAL;
    if (!(lo <= hi) || !(p_m == p_m) || !(p_c == p_c)) return RSPARSE_EINVAL;
    const int L = n_layers, P = population, T = generations;
    try {
        Uniform u(seed);
        std::vector<double> S(L);
        for (int l = 0; l < L; ++l) S[l] = rho_start ? rho_start[l] : lo + (hi - lo) * u();
        double S_loss = loss(S.data(), L, user);
        size_t h = 0;
        if (history_out) history_out[h++] = S_loss;
        for (int g0 = 0; g0 < L; g0 += group_size) {
            const int g1 = std::min(L, g0 + group_size);
            // individual 0 is the best recipe so far; the others are random in this group's coordinates
            std::vector<Member> G(P);
            G[0] = Member{S_loss, 0, 0, S};
            for (int i = 1; i < P; ++i) {
                G[i] = Member{0.0, 0, i, S};
                for (int c = g0; c < g1; ++c) G[i].rho[c] = lo + (hi - lo) * u();
            }
            for (int i = 1; i < P; ++i) G[i].loss = loss(G[i].rho.data(), L, user);
            for (int t = 0; t < T; ++t) {
                std::vector<Member> pool = G;
                for (int i = 0; i < P; ++i) {
                    const int x1 = (int)(u() * P), x2 = (int)(u() * P), x3 = (int)(u() * P);
                    Member child{0.0, 1, i, G[i].rho};
                    for (int c = g0; c < g1; ++c) {
                        const double alpha = u();
                        double m = G[x1].rho[c] + p_m * (G[x2].rho[c] - G[x3].rho[c]);      // mutation
                        m = std::min(std::max(m, lo), hi);
                        child.rho[c] = alpha > p_c ? m : G[i].rho[c];                        // crossover
                    }
                    child.loss = loss(child.rho.data(), L, user);
                    pool.push_back(std::move(child));
                }
                // next generation: the P lowest losses of G u G_hat (ties: older first, then by index)
                std::sort(pool.begin(), pool.end(), [](const Member &a, const Member &b) {
                    if (a.loss != b.loss) return a.loss < b.loss;
                    if (a.age != b.age) return a.age < b.age;
                    return a.index < b.index;
                });
                pool.resize(P);
                for (int i = 0; i < P; ++i) { pool[i].age = 0; pool[i].index = i; }
                G.swap(pool);
                if (history_out) history_out[h++] = G[0].loss;
            }
            S = G[0].rho;
            S_loss = G[0].loss;
        }
        for (int l = 0; l < L; ++l) rho_out[l] = S[l];
        *loss_out = S_loss;
    } catch (const std::bad_alloc &) {
        return RSPARSE_ENOMEM;
    }
    return RSPARSE_OK;
}
