// astraea_budget_search and its operators: the evolutionary search of the per-timestep token budgets
// (paper Sec. 3.3 "Algorithm": crossover, mutation, repair; supplementary algorithm "Evolutionary Search for
// Token Scheduling").  Host code only: the search runs once per model offline and spends its time in the
// caller's fitness function (a full generation per candidate in the paper), not here.
//
// A schedule is T integers in tenths, theta_i in 0..10 (0 %, 10 %, ..., 100 % of the tokens at timestep i);
// the budget is their sum.  Random draws come from SplitMix64 (state += 0x9E3779B97F4A7C15, two
// xor-shift-multiply rounds) with below(n) = floor(next * n / 2^64) and unit() = (next >> 11) * 2^-53, consumed
// in the order of the loops below, so that a seed fixes the result.
#include <algorithm>
#include <cstring>
#include <numeric>
#include <vector>

#include "common.h"

namespace astraea {
namespace {

constexpr int kLevels = 11;

struct Rng {
    uint64_t state;
    uint64_t next()
    {
        state += 0x9E3779B97F4A7C15ull;
        uint64_t z = state;
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
        return z ^ (z >> 31);
    }
    uint32_t below(uint32_t n) { return (uint32_t)(((unsigned __int128)next() * n) >> 64); }
    double unit() { return (double)(next() >> 11) * (1.0 / 9007199254740992.0); }
};

using Schedule = std::vector<int32_t>;

void bounds(int64_t budget, int64_t &lo, int64_t &hi)
{
    lo = (9 * budget + 9) / 10;      // ceil(0.9 B)
    hi = (11 * budget) / 10;         // floor(1.1 B)
}

void crossover_uniform(const int32_t *p0, const int32_t *p1, int32_t T, Rng &rng, int32_t *child)
{
    for (int32_t i = 0; i < T; ++i) child[i] = rng.below(2) == 0 ? p0[i] : p1[i];
}

void crossover_block(const int32_t *p0, const int32_t *p1, int32_t T, Rng &rng, int32_t *child)
{
    const uint32_t a = rng.below((uint32_t)T + 1), b = rng.below((uint32_t)T + 1);
    const int32_t lo = (int32_t)std::min(a, b), hi = (int32_t)std::max(a, b);
    for (int32_t i = 0; i < T; ++i) child[i] = (i >= lo && i < hi) ? p0[i] : p1[i];
}

#pragma clang fp contract(off)
double mutation_probability(double p_start, double p_final, int32_t generation, int32_t generations)
{
    const double frac = (double)generation / (double)generations;
    const double drop = frac * (p_start - p_final);
    return p_start - drop;
}

void mutate(int32_t *theta, int32_t T, double p_mut, Rng &rng)
{
    for (int32_t i = 0; i < T; ++i)
        if (rng.unit() < p_mut) theta[i] = (int32_t)rng.below(kLevels);
}

void repair(int32_t *theta, int32_t T, int64_t budget, Rng &rng)
{
    int64_t lo, hi;
    bounds(budget, lo, hi);
    int64_t total = 0;
    for (int32_t i = 0; i < T; ++i) total += theta[i];
    std::vector<int32_t> movable;
    movable.reserve(T);
    while (total > hi) {
        movable.clear();
        for (int32_t i = 0; i < T; ++i)
            if (theta[i] > 0) movable.push_back(i);
        const int32_t i = movable[rng.below((uint32_t)movable.size())];
        --theta[i];
        --total;
    }
    while (total < lo) {
        movable.clear();
        for (int32_t i = 0; i < T; ++i)
            if (theta[i] < kLevels - 1) movable.push_back(i);
        if (movable.empty()) break;          // every timestep at 100 %: the range cannot be reached
        const int32_t i = movable[rng.below((uint32_t)movable.size())];
        ++theta[i];
        ++total;
    }
}

bool contains(const std::vector<Schedule> &set, const Schedule &c)
{
    for (const Schedule &s : set)
        if (s == c) return true;
    return false;
}

bool valid_schedule(const int32_t *theta, int32_t T)
{
    for (int32_t i = 0; i < T; ++i)
        if (theta[i] < 0 || theta[i] >= kLevels) return false;
    return true;
}

// best-first order with ties keeping the earlier candidate first
void keep_best(std::vector<Schedule> &pop, std::vector<double> &fit, size_t keep)
{
    std::vector<size_t> order(pop.size());
    std::iota(order.begin(), order.end(), (size_t)0);
    std::stable_sort(order.begin(), order.end(), [&](size_t a, size_t b) { return fit[a] < fit[b]; });
    if (order.size() > keep) order.resize(keep);
    std::vector<Schedule> p2;
    std::vector<double> f2;
    for (size_t i : order) {
        p2.push_back(std::move(pop[i]));
        f2.push_back(fit[i]);
    }
    pop.swap(p2);
    fit.swap(f2);
}

}  // namespace
}  // namespace astraea

using namespace astraea;

extern "C" {

int astraea_search_crossover(const int32_t *parent0, const int32_t *parent1, int32_t T, int kind, uint64_t *rng_state,
                             int32_t *child)
{
    if (!parent0 || !parent1 || !child || !rng_state || T <= 0)
        return fail(ASTRAEA_ERR_INVALID, "astraea_search_crossover: NULL argument or T <= 0");
    if (kind != ASTRAEA_CROSSOVER_UNIFORM && kind != ASTRAEA_CROSSOVER_BLOCK)
        return fail(ASTRAEA_ERR_INVALID, "astraea_search_crossover: unknown kind %d", kind);
    Rng rng{*rng_state};
    if (kind == ASTRAEA_CROSSOVER_UNIFORM)
        crossover_uniform(parent0, parent1, T, rng, child);
    else
        crossover_block(parent0, parent1, T, rng, child);
    *rng_state = rng.state;
    return ASTRAEA_OK;
}

int astraea_search_mutate(int32_t *theta, int32_t T, double p_mutation, uint64_t *rng_state)
{
    if (!theta || !rng_state || T <= 0) return fail(ASTRAEA_ERR_INVALID, "astraea_search_mutate: NULL argument or T <= 0");
    if (!(p_mutation >= 0.0 && p_mutation <= 1.0))
        return fail(ASTRAEA_ERR_INVALID, "astraea_search_mutate: probability outside [0, 1]");
    Rng rng{*rng_state};
    mutate(theta, T, p_mutation, rng);
    *rng_state = rng.state;
    return ASTRAEA_OK;
}

int astraea_search_repair(int32_t *theta, int32_t T, int64_t budget_tenths, uint64_t *rng_state)
{
    if (!theta || !rng_state || T <= 0) return fail(ASTRAEA_ERR_INVALID, "astraea_search_repair: NULL argument or T <= 0");
    if (budget_tenths < 0) return fail(ASTRAEA_ERR_INVALID, "astraea_search_repair: negative budget");
    if (!valid_schedule(theta, T)) return fail(ASTRAEA_ERR_INVALID, "astraea_search_repair: a level outside 0..10");
    Rng rng{*rng_state};
    repair(theta, T, budget_tenths, rng);
    *rng_state = rng.state;
    return ASTRAEA_OK;
}

int astraea_budget_search(const astraea_search_config *cfg, astraea_fitness_fn fitness, void *user,
                          int32_t *best_theta, double *best_fitness, int32_t *population_out, double *fitness_out,
                          int32_t *population_size_out)
{
    const char *fn = "astraea_budget_search";
    if (!cfg || !fitness || !best_theta) return fail(ASTRAEA_ERR_INVALID, "%s: NULL argument", fn);
    if (cfg->T <= 0 || cfg->T > (1 << 20)) return fail(ASTRAEA_ERR_INVALID, "%s: T=%d out of range", fn, (int)cfg->T);
    if (cfg->budget_tenths < 0 || cfg->budget_tenths > 10 * (int64_t)cfg->T)
        return fail(ASTRAEA_ERR_INVALID, "%s: budget outside [0, 10*T]", fn);
    if (cfg->population <= 0 || cfg->children < 0 || cfg->generations < 0 || cfg->population > (1 << 20) ||
        cfg->children > (1 << 20))
        return fail(ASTRAEA_ERR_INVALID, "%s: population, children or generations out of range", fn);
    if (!(cfg->p_mutation_start >= 0.0 && cfg->p_mutation_start <= 1.0 && cfg->p_mutation_final >= 0.0 &&
          cfg->p_mutation_final <= 1.0))
        return fail(ASTRAEA_ERR_INVALID, "%s: mutation probabilities outside [0, 1]", fn);
    const int32_t T = cfg->T;
    const int64_t attempts_cap = 64;
    Rng rng{cfg->seed};
    std::vector<Schedule> pop;
    std::vector<double> fit;
    // initial generation: uniform random levels, repaired into the budget range, distinct
    for (int64_t attempts = 0; (int64_t)pop.size() < cfg->population && attempts < attempts_cap * cfg->population;
         ++attempts) {
        Schedule c(T);
        for (int32_t i = 0; i < T; ++i) c[i] = (int32_t)rng.below(kLevels);
        repair(c.data(), T, cfg->budget_tenths, rng);
        if (!contains(pop, c)) pop.push_back(std::move(c));
    }
    for (const Schedule &c : pop) fit.push_back(fitness(c.data(), T, user));
    keep_best(pop, fit, (size_t)cfg->population);
    for (int32_t g = 1; g <= cfg->generations; ++g) {
        const double p_mut = mutation_probability(cfg->p_mutation_start, cfg->p_mutation_final, g, cfg->generations);
        const uint32_t k = (uint32_t)pop.size();
        std::vector<Schedule> fresh;
        for (int64_t attempts = 0; (int64_t)fresh.size() < cfg->children && attempts < attempts_cap * cfg->children;
             ++attempts) {
            const uint32_t a = rng.below(k);
            uint32_t b = a;
            if (k > 1) {
                b = rng.below(k - 1);
                if (b >= a) ++b;
            }
            Schedule child(T);
            if (rng.below(2) == 0)
                crossover_uniform(pop[a].data(), pop[b].data(), T, rng, child.data());
            else
                crossover_block(pop[a].data(), pop[b].data(), T, rng, child.data());
            mutate(child.data(), T, p_mut, rng);
            repair(child.data(), T, cfg->budget_tenths, rng);
            if (!contains(pop, child) && !contains(fresh, child)) fresh.push_back(std::move(child));
        }
        for (Schedule &c : fresh) {
            fit.push_back(fitness(c.data(), T, user));
            pop.push_back(std::move(c));
        }
        keep_best(pop, fit, (size_t)cfg->population);
    }
    std::memcpy(best_theta, pop[0].data(), sizeof(int32_t) * (size_t)T);
    if (best_fitness) *best_fitness = fit[0];
    if (population_size_out) *population_size_out = (int32_t)pop.size();
    for (size_t i = 0; i < pop.size(); ++i) {
        if (population_out) std::memcpy(population_out + i * (size_t)T, pop[i].data(), sizeof(int32_t) * (size_t)T);
        if (fitness_out) fitness_out[i] = fit[i];
    }
    return ASTRAEA_OK;
}

}  // extern "C"
