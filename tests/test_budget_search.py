"""Token-budget search (paper Sec. 3.3; supplementary algorithm "Evolutionary Search for Token Scheduling").

First the oracle (oracle/budget_search.py) against what the paper and the mathematics fix: the generator's
published test vectors, the operators' defining properties, the repair range, and brute force on a search space
small enough to enumerate.  Then the library's host implementation against the oracle, bit for bit."""
import itertools

import numpy as np
import pytest

from oracle import budget_search as ob


# ---------------------------------------------------------------- generator --

def test_splitmix64_published_vectors():
    r = ob.SplitMix64(0)
    assert [r.next() for _ in range(3)] == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]
    r = ob.SplitMix64(1234567)
    assert [r.next() for _ in range(5)] == [6457827717110365317, 3203168211198807973, 9817491932198370423,
                                            4593380528125082431, 16408922859458223821]


def test_generator_ranges():
    r = ob.SplitMix64(7)
    draws = [r.below(11) for _ in range(20000)]
    assert min(draws) == 0 and max(draws) == 10
    assert np.all(np.abs(np.bincount(draws, minlength=11) / 20000 - 1 / 11) < 0.01)
    u = [r.unit() for _ in range(20000)]
    assert 0.0 <= min(u) and max(u) < 1.0 and abs(np.mean(u) - 0.5) < 0.01
    assert ob.SplitMix64(3).below(1) == 0


# ---------------------------------------------------------------- operators --

def test_budget_bounds():
    assert ob.budget_bounds(50) == (45, 55)
    assert ob.budget_bounds(55) == (50, 60)       # 49.5 -> 50, 60.5 -> 60
    assert ob.budget_bounds(0) == (0, 0)
    assert ob.budget_bounds(1) == (1, 1)


def test_crossover_takes_every_gene_from_a_parent_at_the_same_position():
    T = 40
    p0, p1 = [0] * T, [1] * T                     # the child then shows which parent each gene came from
    seen_from_both = False
    for seed in range(50):
        c = ob.crossover_uniform(p0, p1, ob.SplitMix64(seed))
        assert len(c) == T and set(c) <= {0, 1}
        seen_from_both |= 0 < sum(c) < T
    assert seen_from_both
    frac = np.mean([np.mean(ob.crossover_uniform(p0, p1, ob.SplitMix64(s))) for s in range(300)])
    assert abs(frac - 0.5) < 0.02                 # equal probability
    lengths = []
    for seed in range(200):
        c = ob.crossover_block(p0, p1, ob.SplitMix64(seed))
        from_p0 = [i for i, v in enumerate(c) if v == 0]
        if from_p0:                               # one contiguous block of timesteps comes from the first parent
            assert from_p0 == list(range(from_p0[0], from_p0[-1] + 1))
        lengths.append(len(from_p0))
    assert min(lengths) == 0 or min(lengths) < 5
    assert max(lengths) > T // 2                  # blocks of all sizes occur
    # genes are copied by position, not by value
    a, b = list(range(10)), list(range(100, 110))
    for seed in range(20):
        for op in (ob.crossover_block, ob.crossover_uniform):
            c = op(a, b, ob.SplitMix64(seed))
            assert all(c[i] in (a[i], b[i]) for i in range(10))


def test_block_crossover_range_has_uniform_ends():
    """Both ends uniform on 0..T, the range [lo, hi) from the first parent: timestep i then comes from it with
    probability 1 - ((i + 1) / (T + 1))^2 - ((T - i) / (T + 1))^2, the whole child with 2 / (T + 1)^2."""
    T, draws = 6, 40000
    p0, p1 = [0] * T, [1] * T
    r = ob.SplitMix64(11)
    from_p0 = np.zeros(T)
    whole = 0
    for _ in range(draws):
        c = ob.crossover_block(p0, p1, r)
        from_p0 += 1 - np.array(c)
        whole += sum(c) == 0
    want = np.array([1 - ((i + 1) / (T + 1)) ** 2 - ((T - i) / (T + 1)) ** 2 for i in range(T)])
    assert np.all(np.abs(from_p0 / draws - want) < 4 * np.sqrt(want * (1 - want) / draws))
    pw = 2 / (T + 1) ** 2
    assert abs(whole / draws - pw) < 4 * np.sqrt(pw * (1 - pw) / draws)


def test_parent_pairs_are_distinct_and_uniform():
    k, draws = 4, 24000
    r = ob.SplitMix64(21)
    counts = np.zeros((k, k))
    for _ in range(draws):
        a, b = ob.parent_pair(k, r)
        counts[a, b] += 1
    assert np.all(np.diag(counts) == 0)
    off = counts[~np.eye(k, dtype=bool)] / draws
    p = 1 / (k * (k - 1))
    assert np.all(np.abs(off - p) < 4 * np.sqrt(p * (1 - p) / draws))
    assert ob.parent_pair(1, ob.SplitMix64(0)) == (0, 0)


def test_mutation_probability_schedule():
    g_max = 30
    p = [ob.mutation_probability(0.4, 0.1, g, g_max) for g in range(1, g_max + 1)]
    assert abs(p[-1] - 0.1) < 1e-15 and abs(p[0] - (0.4 - 0.3 / 30)) < 1e-15
    assert all(x > y for x, y in zip(p, p[1:]))   # decreases every generation
    assert ob.mutation_probability(0.2, 0.2, 5, 30) == 0.2


def test_mutation():
    theta = [3] * 1000
    r = ob.SplitMix64(5)
    assert ob.mutate(theta, 0.0, r) == theta
    s_after = r.state
    r2 = ob.SplitMix64(5)
    for _ in range(1000):
        r2.next()
    assert s_after == r2.state                    # one draw per timestep when nothing mutates
    m = ob.mutate(theta, 1.0, ob.SplitMix64(5))
    assert min(m) == 0 and max(m) == 10           # a mutated timestep takes any of the 11 levels
    changed = np.mean([np.mean(np.array(ob.mutate(theta, 0.3, ob.SplitMix64(s))) != 3) for s in range(20)])
    assert abs(changed - 0.3 * 10 / 11) < 0.01    # mutated with probability 0.3; 1 in 11 redraws the old value


def test_repair():
    B = 50
    lo, hi = ob.budget_bounds(B)
    rng = np.random.default_rng(0)
    for trial in range(200):
        theta = list(rng.integers(0, 11, size=10))
        before = sum(theta)
        r = ob.SplitMix64(trial)
        s0 = r.state
        out = ob.repair(theta, B, r)
        assert lo <= sum(out) <= hi and all(0 <= v <= 10 for v in out)
        if before > hi:
            assert all(o <= t for o, t in zip(out, theta)) and sum(out) == hi     # only lowered, just into range
        elif before < lo:
            assert all(o >= t for o, t in zip(out, theta)) and sum(out) == lo     # only raised
        else:
            assert out == theta and r.state == s0                                 # in range: untouched, no draws
    # the range cannot be reached: everything ends at 100 %
    assert ob.repair([10, 10], 40, ob.SplitMix64(0)) == [10, 10]
    assert ob.repair([10, 10, 10], 0, ob.SplitMix64(0)) == [0, 0, 0]


# -------------------------------------------------------------------- search --

def _fitness(weights):
    # separable, convex: the loss of computing fewer tokens at timestep i, weighted by how much that step matters
    return lambda th: float(sum(w * (10 - t) ** 2 for w, t in zip(weights, th)))


def test_search_finds_the_enumerated_optimum_on_a_small_space():
    T, B = 4, 20
    f = _fitness([5.0, 1.0, 3.0, 0.5])
    lo, hi = ob.budget_bounds(B)
    best = min((c for c in itertools.product(range(11), repeat=T) if lo <= sum(c) <= hi), key=f)
    for seed in (1, 2, 3):
        sched, val, pop, fit = ob.search(T, B, 30, 20, 60, 0.4, 0.05, seed, f)
        assert list(sched) == list(best) and val == f(best)
        assert fit == sorted(fit) and fit == [f(c) for c in pop]
        assert len({tuple(c) for c in pop}) == len(pop)                       # no duplicates
        assert all(lo <= sum(c) <= hi for c in pop)                           # every survivor within budget


def test_search_never_gets_worse_with_more_generations():
    T, B = 12, 60
    f = _fitness(list(np.linspace(3.0, 0.2, T)))
    vals = [ob.search(T, B, 16, 10, g, 0.3, 0.05, 9, f)[1] for g in (0, 1, 5, 20)]
    # the draws of the first generations do not depend on how many follow only through p_mutation, so compare loosely
    assert vals[-1] <= vals[0] and vals[-1] < vals[0]
    # zero generations: the best of the initial population
    s0 = ob.search(T, B, 16, 10, 0, 0.3, 0.05, 9, f)
    assert s0[1] == min(s0[3]) and len(s0[2]) == 16


# ------------------------------------------- the library against the oracle --

from paper_2506_05096_amd import binding as ab   # noqa: E402  (host-only entry points; no GPU is touched)


@pytest.mark.parametrize("seed", [0, 1, 99, 2 ** 63 + 5])
def test_library_operators_match_the_oracle_bit_for_bit(seed):
    rng = np.random.default_rng(seed % 1000)
    T = 37
    p0, p1 = rng.integers(0, 11, T), rng.integers(0, 11, T)
    for kind, fn in ((ab.CROSSOVER_UNIFORM, ob.crossover_uniform), (ab.CROSSOVER_BLOCK, ob.crossover_block)):
        r = ob.SplitMix64(seed)
        want = fn(list(p0), list(p1), r)
        got, st = ab.astraea_search_crossover(p0, p1, kind, seed)
        assert list(got) == want and st == r.state
    for p in (0.0, 0.05, 0.3, 1.0):
        r = ob.SplitMix64(seed)
        want = ob.mutate(list(p0), p, r)
        got, st = ab.astraea_search_mutate(p0, p, seed)
        assert list(got) == want and st == r.state
    for budget in (0, 40, 185, 300, 370):
        r = ob.SplitMix64(seed)
        want = ob.repair(list(p0), budget, r)
        got, st = ab.astraea_search_repair(p0, budget, seed)
        assert list(got) == want and st == r.state


@pytest.mark.parametrize("T,budget,pop,children,gens,seed", [(4, 20, 30, 20, 60, 3), (50, 250, 50, 30, 30, 0),
                                                             (12, 60, 16, 10, 0, 9), (3, 30, 8, 5, 10, 4),
                                                             (20, 0, 6, 6, 4, 1)])
def test_library_search_matches_the_oracle_bit_for_bit(T, budget, pop, children, gens, seed):
    f = _fitness(list(np.linspace(3.0, 0.2, T)))
    want = ob.search(T, budget, pop, children, gens, 0.3, 0.05, seed, f)
    got = ab.astraea_budget_search(T, budget, pop, children, gens, 0.3, 0.05, seed, f)
    assert list(got[0]) == list(want[0]) and got[1] == want[1]
    assert got[2].tolist() == [list(c) for c in want[2]]
    assert got[3].tolist() == want[3]


def test_library_search_rejects_bad_arguments():
    f = lambda th: 0.0
    for kw in (dict(T=0), dict(budget_tenths=-1), dict(budget_tenths=1000), dict(population=0), dict(children=-1),
               dict(p_mutation_start=1.5), dict(p_mutation_final=float("nan"))):
        args = dict(T=10, budget_tenths=50, population=5, children=3, generations=2, p_mutation_start=0.3,
                    p_mutation_final=0.1, seed=1)
        args.update(kw)
        with pytest.raises(ab.AstraeaError) as e:
            ab.astraea_budget_search(fitness=f, **args)
        assert e.value.status == ab.ERR_INVALID
    with pytest.raises(ab.AstraeaError):
        ab.astraea_search_repair([3, 11, 2], 10, 0)          # a level outside 0..10
    with pytest.raises(ab.AstraeaError):
        ab.astraea_search_mutate([1, 2], 2.0, 0)
