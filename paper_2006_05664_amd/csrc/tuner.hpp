// OpEvo search loop (Alg. 1, Sec. 4.4): selection + recombination (Sec. 4.2, Eq. 2),
// q-random-walk mutation (Sec. 4.3) and the no-duplicate rule, in ask/tell form.
#pragma once

#include <cstdint>
#include <unordered_set>
#include <vector>

#include "space.hpp"

namespace opevo {

struct CfgHash {
    size_t operator()(const std::vector<int32_t> &c) const
    {
        uint64_t h = 0xcbf29ce484222325ull;     // FNV-1a over the ints
        for (int32_t a : c) { h ^= uint32_t(a); h *= 0x100000001b3ull; }
        return size_t(h);
    }
};

// One child by Eq. 2; parents best first, fitness already clamped at 0.
void recombine(const opevo_space &space, const int32_t *parents, const double *fitness,
               int n_parents, Rng &rng, int32_t *child);

}  // namespace opevo

struct opevo_tuner {
    const opevo_space *space;
    int lambda, rho;
    double q;
    opevo::Rng rng;
    int mutation = 0;       // 0: q-random walk on the parameter graphs (Sec. 4.3); 1: uniform resampling (control)
    bool started = false;
    std::vector<std::vector<int32_t>> configs;   // Q in trial order
    std::vector<double> fitness;
    std::unordered_set<std::vector<int32_t>, opevo::CfgHash> sampled;  // told or pending

    opevo_tuner(const opevo_space *s, int lam, int r, double qq, uint64_t seed)
        : space(s), lambda(lam), rho(r), q(qq), rng(seed) {}

    std::vector<int> top(int n) const;   // trial indices, best first, ties: earlier first
    // false if no unsampled configuration could be found (space exhausted)
    bool random_unsampled(std::vector<int32_t> &cfg);
    int ask(int32_t *out, int max_n);
    void tell(const int32_t *cfgs, const double *fit, int n);
    void mutate(int32_t *cfg) { if (mutation == 1) space->mutate_uniform(q, rng, cfg); else space->mutate(q, rng, cfg); }
};
