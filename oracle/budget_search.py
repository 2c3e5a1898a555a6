"""Oracle of the token-budget search (test infrastructure only; plain Python loops).

Paper Sec. 3.3 "Algorithm" (crossover, mutation, repair) and the supplementary algorithm "Evolutionary Search
for Token Scheduling": an evolutionary algorithm over schedules theta = (theta_0 .. theta_{T-1}),
theta_i in {0, 10 %, ..., 100 %}, under a total budget.  The steps are taken in the paper's order; where the
paper is silent the reading is stated next to the step.  Percentages are held as integers in tenths (0..10),
the budget as their sum, so everything the search decides is integer work; the only floating point is the
mutation probability and the caller's fitness values, both compared in binary64.

The search draws random numbers.  Oracle and library each implement the same counter-based generator from
its published definition (SplitMix64: state += 0x9E3779B97F4A7C15, then the two xor-shift-multiply rounds),
with  below(n) = floor(next() * n / 2^64)  and  unit() = (next() >> 11) * 2^-53,  and consume draws in the
order written here.
"""
from __future__ import annotations

from typing import Callable, List, Sequence, Tuple

MASK = (1 << 64) - 1
LEVELS = 11          # theta in tenths: 0..10  (Sec. 3.3, search space)


class SplitMix64:
    def __init__(self, seed: int):
        self.state = seed & MASK

    def next(self) -> int:
        self.state = (self.state + 0x9E3779B97F4A7C15) & MASK
        z = self.state
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & MASK
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & MASK
        return z ^ (z >> 31)

    def below(self, n: int) -> int:
        return (self.next() * n) >> 64

    def unit(self) -> float:
        return (self.next() >> 11) * (1.0 / 9007199254740992.0)


def budget_bounds(budget: int) -> Tuple[int, int]:
    """Acceptable totals [0.9 B, 1.1 B] (Sec. 3.3 "Repair"), as integers in tenths: ceil and floor."""
    return (9 * budget + 9) // 10, (11 * budget) // 10


def crossover_uniform(p0: Sequence[int], p1: Sequence[int], rng: SplitMix64) -> List[int]:
    """Each theta_i from either parent with equal probability (Sec. 3.3 "Crossover")."""
    return [p0[i] if rng.below(2) == 0 else p1[i] for i in range(len(p0))]


def crossover_block(p0: Sequence[int], p1: Sequence[int], rng: SplitMix64) -> List[int]:
    """A contiguous range of timesteps from one parent, the rest from the other (Sec. 3.3 "Crossover").
    Reading: the two ends are drawn uniformly from 0..T and ordered; the range [lo, hi) comes from the first
    parent."""
    t = len(p0)
    a, b = rng.below(t + 1), rng.below(t + 1)
    lo, hi = (a, b) if a <= b else (b, a)
    return [p0[i] if lo <= i < hi else p1[i] for i in range(t)]


def mutation_probability(p_start: float, p_final: float, generation: int, generations: int) -> float:
    """P_mutation = P_0 - (beta_i / beta_max) (P_0 - P_final), beta_i the generation counted from 1."""
    frac = generation / generations
    drop = frac * (p_start - p_final)
    return p_start - drop


def mutate(theta: Sequence[int], p_mut: float, rng: SplitMix64) -> List[int]:
    """Each timestep is mutated with probability p_mut; a mutated one takes a value drawn from all 11 levels
    (Sec. 3.3 "Mutation"; the new value may equal the old one)."""
    out = list(theta)
    for i in range(len(out)):
        if rng.unit() < p_mut:
            out[i] = rng.below(LEVELS)
    return out


def repair(theta: Sequence[int], budget: int, rng: SplitMix64) -> List[int]:
    """Brings the total into [0.9 B, 1.1 B] (Sec. 3.3 "Repair"): above the range, random timesteps are lowered;
    below it, random timesteps are raised.  Reading: one level (10 %) at a time, the timestep drawn uniformly
    among those that can still move in that direction."""
    out = list(theta)
    lo, hi = budget_bounds(budget)
    total = sum(out)
    while total > hi:
        movable = [i for i in range(len(out)) if out[i] > 0]
        i = movable[rng.below(len(movable))]
        out[i] -= 1
        total -= 1
    while total < lo:
        movable = [i for i in range(len(out)) if out[i] < LEVELS - 1]
        if not movable:
            break                       # every timestep is at 100 %: the range cannot be reached
        i = movable[rng.below(len(movable))]
        out[i] += 1
        total += 1
    return out


def parent_pair(k: int, rng: SplitMix64) -> Tuple[int, int]:
    """Two parents drawn from the k candidates of the current population (Sec. 3.3 "Algorithm": a random pair).
    Reading: uniform over ordered pairs of distinct candidates; with a single candidate it is its own partner."""
    a = rng.below(k)
    b = a
    if k > 1:
        b = rng.below(k - 1)
        if b >= a:
            b += 1
    return a, b


def search(T: int, budget: int, population: int, children: int, generations: int, p_start: float, p_final: float,
           seed: int, fitness: Callable[[Sequence[int]], float], max_attempts_factor: int = 64):
    """The search loop (supplementary algorithm; Sec. 3.3 "Algorithm").

    population K candidates; each generation: the K best by fitness (lower is better) are the parents; `children`
    new candidates are made, each from a random parent pair by crossover (one of the two kinds, chosen with equal
    probability), mutation, repair, and added unless already present; all are evaluated and the best K survive.
    Readings: initial candidates are uniform random levels put through repair; the two parents of a pair are
    distinct when K > 1; a duplicate child is dropped and drawn again, at most max_attempts_factor * children draws
    per generation (after that the generation goes on with fewer children); ties in fitness keep the earlier
    candidate first.  Returns (best schedule, its fitness, final population best-first, their fitness).
    """
    rng = SplitMix64(seed)
    pop: List[List[int]] = []
    attempts = 0
    while len(pop) < population and attempts < max_attempts_factor * population:
        attempts += 1
        cand = repair([rng.below(LEVELS) for _ in range(T)], budget, rng)
        if cand not in pop:
            pop.append(cand)
    fit = [fitness(c) for c in pop]
    order = sorted(range(len(pop)), key=lambda i: (fit[i], i))
    pop, fit = [pop[i] for i in order], [fit[i] for i in order]
    for g in range(1, generations + 1):
        p_mut = mutation_probability(p_start, p_final, g, generations)
        k = len(pop)
        new: List[List[int]] = []
        attempts = 0
        while len(new) < children and attempts < max_attempts_factor * children:
            attempts += 1
            a, b = parent_pair(k, rng)
            if rng.below(2) == 0:
                child = crossover_uniform(pop[a], pop[b], rng)
            else:
                child = crossover_block(pop[a], pop[b], rng)
            child = mutate(child, p_mut, rng)
            child = repair(child, budget, rng)
            if child not in pop and child not in new:
                new.append(child)
        pop = pop + new
        fit = fit + [fitness(c) for c in new]
        order = sorted(range(len(pop)), key=lambda i: (fit[i], i))[:population]
        pop, fit = [pop[i] for i in order], [fit[i] for i in order]
    return pop[0], fit[0], pop, fit
