// OpEvo search loop (Alg. 1): see tuner.hpp.
#include "tuner.hpp"

#include <algorithm>
#include <cmath>
#include <cstring>
#include <new>
#include <numeric>

namespace opevo {

static const int kRemutateCap = 100;           // re-mutations of a duplicate child
static const double kEnumLimit = 1048576.0;    // spaces up to 2^20 list their unsampled members
static const int kRejectTries = 10000;         // larger spaces: rejection sampling

static inline double clamp_fitness(double f) { return f > 0.0 ? f : 0.0; }  // NaN -> 0 too

void recombine(const opevo_space &space, const int32_t *parents, const double *fitness,
               int n_parents, Rng &rng, int32_t *child)
{
    const int w = space.width;
    double total = 0.0;
    for (int j = 0; j < n_parents; ++j) total += fitness[j];
    for (const Param &p : space.params) {
        int pick = -1;
        if (total > 0.0) {
            // P(x_i = x_i^j) = f(x^j) / sum_k f(x^k)   (Eq. 2)
            const double t = rng.next_double() * total;
            double acc = 0.0;
            int last_pos = -1;
            for (int j = 0; j < n_parents; ++j) {
                acc += fitness[j];
                if (fitness[j] > 0.0) last_pos = j;
                if (t < acc) { pick = j; break; }
            }
            if (pick < 0) pick = last_pos;
        } else {
            pick = int(rng.next_below(uint32_t(n_parents)));   // all parents invalid: uniform
        }
        std::memcpy(child + p.offset, parents + size_t(pick) * w + p.offset, sizeof(int32_t) * p.width);
    }
}

}  // namespace opevo

using namespace opevo;

std::vector<int> opevo_tuner::top(int n) const
{
    std::vector<int> order(configs.size());
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return fitness[a] > fitness[b]; });
    if (int(order.size()) > n) order.resize(n);
    return order;
}

bool opevo_tuner::random_unsampled(std::vector<int32_t> &cfg)
{
    const double n = space->size();
    if (double(sampled.size()) >= n) return false;
    if (n <= kEnumLimit) {
        const int64_t total = int64_t(n);
        std::vector<char> taken(size_t(total), 0);
        for (const auto &c : sampled) taken[size_t(space->rank(c.data()))] = 1;
        std::vector<int64_t> free_ranks;
        for (int64_t r = 0; r < total; ++r) if (!taken[size_t(r)]) free_ranks.push_back(r);
        space->unrank(free_ranks[rng.next_below(uint32_t(free_ranks.size()))], cfg.data());
        return true;
    }
    for (int t = 0; t < kRejectTries; ++t) {
        space->random(rng, cfg.data());
        if (!sampled.count(cfg)) return true;
    }
    return false;
}

int opevo_tuner::ask(int32_t *out, int max_n)
{
    int want = started ? rho : lambda;
    if (max_n > 0) want = std::min(want, max_n);
    const int w = space->width;
    std::vector<int32_t> x(w);
    int n = 0;

    if (!started) {
        // Alg. 1 step 1: lambda random configurations (uniform per parameter)
        started = true;
        for (; n < want; ++n) {
            space->random(rng, x.data());
            int tries = 0;
            bool ok = true;
            while (sampled.count(x)) {
                if (tries == kRemutateCap) { ok = random_unsampled(x); break; }
                space->random(rng, x.data());
                ++tries;
            }
            if (!ok) break;
            sampled.insert(x);
            std::memcpy(out + size_t(n) * w, x.data(), sizeof(int32_t) * w);
        }
        return n;
    }

    // Alg. 1 steps 4-5: top-lambda parents -> rho children by recombination + mutation
    const std::vector<int> par = top(lambda);
    std::vector<int32_t> pc(size_t(par.size()) * w);
    std::vector<double> pf(par.size());
    for (size_t j = 0; j < par.size(); ++j) {
        std::memcpy(pc.data() + j * w, configs[par[j]].data(), sizeof(int32_t) * w);
        pf[j] = fitness[par[j]];
    }
    for (; n < want; ++n) {
        recombine(*space, pc.data(), pf.data(), int(par.size()), rng, x.data());
        mutate(x.data());
        int tries = 0;
        bool ok = true;
        while (sampled.count(x)) {                 // already sampled: mutate again (Sec. 4.4)
            if (tries == kRemutateCap) { ok = random_unsampled(x); break; }
            mutate(x.data());
            ++tries;
        }
        if (!ok) break;
        sampled.insert(x);
        std::memcpy(out + size_t(n) * w, x.data(), sizeof(int32_t) * w);
    }
    return n;
}

void opevo_tuner::tell(const int32_t *cfgs, const double *fit, int n)
{
    const int w = space->width;
    for (int i = 0; i < n; ++i) {
        std::vector<int32_t> x(cfgs + size_t(i) * w, cfgs + size_t(i + 1) * w);
        sampled.insert(x);
        configs.push_back(std::move(x));
        fitness.push_back(clamp_fitness(fit[i]));
    }
}

extern "C" {

int opevo_recombine(const opevo_space *space, const int32_t *parents, const double *fitness,
                    int n_parents, opevo_rng *rng, int32_t *child_out)
{
    if (!space || !parents || !fitness || !rng || !child_out || n_parents < 1)
        return fail(OPEVO_E_ARG, "recombine: bad arguments");
    std::vector<double> f(n_parents);
    for (int j = 0; j < n_parents; ++j) {
        if (!space->is_legal(parents + size_t(j) * space->width))
            return fail(OPEVO_E_ILLEGAL, "recombine: parent %d is not in the space", j);
        f[j] = clamp_fitness(fitness[j]);
    }
    recombine(*space, parents, f.data(), n_parents, rng->rng, child_out);
    return OPEVO_OK;
}

int opevo_tuner_create(const opevo_space *space, int lambda, int rho, double q, uint64_t seed,
                       opevo_tuner **out)
{
    if (!space || !out) return fail(OPEVO_E_ARG, "tuner_create: NULL argument");
    if (lambda < 1 || rho < 1) return fail(OPEVO_E_ARG, "tuner_create: lambda and rho must be >= 1");
    if (!(q >= 0.0 && q < 1.0)) return fail(OPEVO_E_ARG, "tuner_create: need 0 <= q < 1");
    if (space->size() <= kEnumLimit && !space->rankable())
        return fail(OPEVO_E_ARG, "tuner_create: inconsistent space");
    *out = new (std::nothrow) opevo_tuner(space, lambda, rho, q, seed);
    return *out ? OPEVO_OK : fail(OPEVO_E_ARG, "out of memory");
}

int opevo_tuner_destroy(opevo_tuner *tuner) { delete tuner; return OPEVO_OK; }

int opevo_tuner_set_mutation(opevo_tuner *tuner, int kind)
{
    if (!tuner) return fail(OPEVO_E_ARG, "tuner_set_mutation: NULL argument");
    if (kind != 0 && kind != 1) return fail(OPEVO_E_ARG, "tuner_set_mutation: kind must be 0 (q-random walk) or 1 (uniform resampling)");
    tuner->mutation = kind;
    return OPEVO_OK;
}

int opevo_tuner_ask(opevo_tuner *tuner, int32_t *cfgs_out, int max_n, int *n_out)
{
    if (!tuner || !cfgs_out || !n_out) return fail(OPEVO_E_ARG, "tuner_ask: NULL argument");
    if (tuner->started && tuner->configs.empty())
        return fail(OPEVO_E_STATE, "tuner_ask: tell() the first generation before asking again");
    *n_out = tuner->ask(cfgs_out, max_n);
    return OPEVO_OK;
}

int opevo_tuner_tell(opevo_tuner *tuner, const int32_t *cfgs, const double *fitness, int n)
{
    if (!tuner || (n > 0 && (!cfgs || !fitness)) || n < 0) return fail(OPEVO_E_ARG, "tuner_tell: bad arguments");
    for (int i = 0; i < n; ++i)
        if (!tuner->space->is_legal(cfgs + size_t(i) * tuner->space->width))
            return fail(OPEVO_E_ILLEGAL, "tuner_tell: configuration %d is not in the space", i);
    tuner->tell(cfgs, fitness, n);
    return OPEVO_OK;
}

int opevo_tuner_num_trials(const opevo_tuner *tuner, int *n)
{
    if (!tuner || !n) return fail(OPEVO_E_ARG, "tuner_num_trials: NULL argument");
    *n = int(tuner->configs.size());
    return OPEVO_OK;
}

int opevo_tuner_best(const opevo_tuner *tuner, int32_t *cfg_out, double *fitness, int *trial)
{
    if (!tuner) return fail(OPEVO_E_ARG, "tuner_best: NULL argument");
    if (tuner->configs.empty()) return fail(OPEVO_E_STATE, "tuner_best: nothing evaluated yet");
    const int t = tuner->top(1)[0];
    if (cfg_out) std::memcpy(cfg_out, tuner->configs[t].data(), sizeof(int32_t) * tuner->space->width);
    if (fitness) *fitness = tuner->fitness[t];
    if (trial) *trial = t;
    return OPEVO_OK;
}

int opevo_tuner_history(const opevo_tuner *tuner, int32_t *cfgs_out, double *fitness_out,
                        int cap_trials, int *n)
{
    if (!tuner || !n) return fail(OPEVO_E_ARG, "tuner_history: NULL argument");
    *n = int(tuner->configs.size());
    if (cap_trials < *n) return fail(OPEVO_E_ARG, "tuner_history: capacity %d < %d trials", cap_trials, *n);
    const int w = tuner->space->width;
    for (int i = 0; i < *n; ++i) {
        if (cfgs_out) std::memcpy(cfgs_out + size_t(i) * w, tuner->configs[i].data(), sizeof(int32_t) * w);
        if (fitness_out) fitness_out[i] = tuner->fitness[i];
    }
    return OPEVO_OK;
}

}  // extern "C"
