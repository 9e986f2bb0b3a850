"""Pins for the search-space / OpEvo oracle (CPU only).

The oracle is tied to: counts and closed forms typed into tests/golden/, the paper's
adjacency definitions re-checked by brute force over all vertex pairs, Theorem 1 and
Lemma 2 of App. A, a Monte-Carlo run of the walk process, the qualitative statements
of Sec. 4.3 about its example graph, and the invariants of Alg. 1.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import search as S

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    with open(os.path.join(GOLDEN, name)) as fh:
        return [ln.strip() for ln in fh if ln.strip() and not ln.startswith("#")]


# ----------------------------------------------------------------------------- RNG
def test_splitmix64_published_vector():
    # first outputs for seed 1234567, as circulated with the generator's reference code
    r = S.SplitMix64(1234567)
    assert [r.next_u64() for _ in range(5)] == [6457827717110365317, 3203168211198807973,
                                                9817491932198370423, 4593380528125082431,
                                                16408922859458223821]


def test_rng_ranges():
    r = S.SplitMix64(7)
    xs = [r.next_double() for _ in range(20000)]
    assert 0.0 <= min(xs) and max(xs) < 1.0 and abs(np.mean(xs) - 0.5) < 0.01
    ks = [r.next_below(7) for _ in range(70000)]
    counts = np.bincount(ks, minlength=7)
    assert counts.min() > 9500 and counts.max() < 10500 and max(ks) == 6


# --------------------------------------------------------------- factorization (Sec. 3)
def test_factorization_counts_golden_and_products():
    for row in _rows("space_sizes.txt"):
        C, nu, want = map(int, row.split())
        V = S.Factor(C, nu).vertices()
        assert len(V) == want == len(set(V)), (C, nu)
        assert all(len(v) == nu and math.prod(v) == C and min(v) >= 1 for v in V)
        assert V == sorted(V)


def _paper_adjacent(u, v):
    """g(u,v) of Sec. 3 by brute force: distinct positions n, m and a prime z with
    u_m = v_m * z and u_n = v_n / z, every other position unchanged."""
    nu = len(u)
    for n in range(nu):
        for m in range(nu):
            if n == m:
                continue
            if any(u[t] != v[t] for t in range(nu) if t not in (n, m)):
                continue
            if v[m] == 0 or u[m] % v[m] or v[n] % max(u[n], 1):
                continue
            z = u[m] // v[m]
            if z > 1 and all(z % d for d in range(2, int(z ** 0.5) + 1)) and u[n] * z == v[n]:
                return True
    return False


@pytest.mark.parametrize("C,nu", [(8, 3), (12, 2), (12, 3), (36, 3), (30, 2), (64, 2), (56, 4)])
def test_factor_neighbors_match_paper_adjacency_bruteforce(C, nu):
    P = S.Factor(C, nu)
    V = P.vertices()
    for u in V:
        nb = P.neighbors(u)
        assert len(nb) == len(set(nb)), "each (n, m, z) must give a different neighbour"
        want = {v for v in V if v != u and _paper_adjacent(u, v)}
        assert set(nb) == want
        assert len(nb) == (nu - 1) * sum(len(S.distinct_primes(a)) for a in u)
        assert all(u in P.neighbors(v) for v in nb)  # undirected


def test_factor_example_graph_degrees_and_connectivity():
    P = S.Factor(8, 3)
    deg = {v: len(P.neighbors(v)) for v in P.vertices()}
    assert [deg[v] for v in [(8, 1, 1), (1, 8, 1), (1, 1, 8)]] == [2, 2, 2]
    assert all(deg[v] == 4 for v in deg if sorted(v) == [1, 2, 4])
    assert deg[(2, 2, 2)] == 6
    assert set(S.Factor(12, 2).neighbors((12, 1))) == {(6, 2), (4, 3)}
    for C, nu in [(8, 3), (960, 2), (56, 4)]:
        P = S.Factor(C, nu)
        V = P.vertices()
        seen, todo = {V[0]}, [V[0]]
        while todo:
            for v in P.neighbors(todo.pop()):
                if v not in seen:
                    seen.add(v); todo.append(v)
        assert len(seen) == len(V)


def test_factor_isolated_cases():
    assert S.Factor(1, 3).vertices() == [(1, 1, 1)] and S.Factor(1, 3).neighbors((1, 1, 1)) == []
    assert S.Factor(7, 1).vertices() == [(7,)] and S.Factor(7, 1).neighbors((7,)) == []


# ------------------------------------------------- permutation / discrete / categorical
def test_permutation_graph():
    P = S.Permutation(3)
    V = P.vertices()
    assert len(V) == 6
    for u in V:
        nb = set(P.neighbors(u))
        want = {v for v in V if sum(a != b for a, b in zip(u, v)) == 2}
        assert nb == want and len(nb) == 3
    P4 = S.Permutation(4)
    assert len(P4.vertices()) == 24 and all(len(set(P4.neighbors(u))) == 6 for u in P4.vertices())


def test_discrete_graph_is_path_on_sorted_values():
    P = S.Discrete([1, 2, 3, 4])
    assert [sorted(P.neighbors((i,))) for i in range(4)] == [[(1,)], [(0,), (2,)], [(1,), (3,)], [(2,)]]
    P = S.Discrete([0.5, 2.0, 10.0])
    assert sorted(P.neighbors((1,))) == [(0,), (2,)] and P.neighbors((0,)) == [(1,)]
    assert S.Discrete([3.0]).neighbors((0,)) == []
    with pytest.raises(AssertionError):
        S.Discrete([1, 1, 2])


def test_categorical_graph_is_complete():
    P = S.Categorical(6)
    for i in range(6):
        assert sorted(P.neighbors((i,))) == [(j,) for j in range(6) if j != i]
    assert S.Categorical(1).neighbors((0,)) == []


# --------------------------------------------------- q-random walk (Sec. 4.3, App. A)
def _param_from_spec(spec):
    kind, *args = spec.split()
    if kind == "factor":
        return S.Factor(int(args[0]), int(args[1]))
    if kind == "discrete":
        return S.Discrete([float(a) for a in args])
    if kind == "categorical":
        return S.Categorical(int(args[0]))
    if kind == "permutation":
        return S.Permutation(int(args[0]))
    raise ValueError(spec)


def test_qwalk_law_golden_rationals():
    rows = _rows("qwalk_laws.txt")
    assert len(rows) >= 30
    cache = {}
    for row in rows:
        spec, start, q, v, p = [t.strip() for t in row.split("|")]
        key = (spec, start, q)
        if key not in cache:
            cache[key] = S.qwalk_law(_param_from_spec(spec), tuple(map(int, start.split(","))), Fraction(q))
        assert cache[key][tuple(map(int, v.split(",")))] == Fraction(p), row


@pytest.mark.parametrize("J", [2, 3, 6, 9])
@pytest.mark.parametrize("q", [Fraction(1, 10), Fraction(1, 2), Fraction(9, 10)])
def test_qwalk_complete_graph_closed_form(J, q):
    law = S.qwalk_law(S.Categorical(J), (0,), q)
    assert law[(0,)] == (J - 1 - (J - 2) * q) / (J - 1 + q)
    assert all(law[(j,)] == q / (J - 1 + q) for j in range(1, J))


@pytest.mark.parametrize("param", [S.Factor(8, 3), S.Factor(12, 3), S.Permutation(3),
                                   S.Discrete([1, 2, 3, 4]), S.Categorical(5), S.Factor(1, 2)])
def test_theorem1_lemma2_and_column_sums(param):
    q = Fraction(3, 5)
    V, Q = S.transition_matrix(param, q)
    for c, u in enumerate(V):  # every column of Q sums to q (App. A), 0 for an isolated vertex
        assert sum(Q[r][c] for r in range(len(V))) == (q if param.neighbors(u) else 0)
    for u in V:
        law = S.qwalk_law(param, u, q)
        assert all(p >= 0 for p in law.values())
        assert sum(law.values()) == 1          # Thm 1; equals Lemma 2: column sum of (I-Q)^-1 is 1/(1-q)
    # q = 0: no mutation (Sec. 4.3)
    law0 = S.qwalk_law(param, V[0], Fraction(0))
    assert law0[V[0]] == 1 and sum(law0.values()) == 1


def test_qwalk_series_definition_matches_closed_form():
    P = S.Factor(8, 3)
    for q in (0.3, 0.5, 0.7):
        exact = S.qwalk_law(P, (8, 1, 1), Fraction(q).limit_denominator(100))
        series = S.qwalk_law_series(P, (8, 1, 1), q)
        assert all(abs(float(exact[v]) - series[v]) < 1e-12 for v in exact)


def test_qwalk_statements_about_the_example_graph():
    """Sec. 4.3: nearer vertices are likelier; a larger q spreads wider; among the
    vertices at equal distance (2,1,4), (2,2,2), (2,4,1), the one with the largest
    degree, (2,2,2), is the likeliest."""
    P = S.Factor(8, 3)
    a = S.qwalk_law(P, (8, 1, 1), Fraction(1, 2))
    b = S.qwalk_law(P, (8, 1, 1), Fraction(7, 10))
    assert a[(2, 2, 2)] > a[(2, 1, 4)] == a[(2, 4, 1)]
    assert b[(2, 2, 2)] > b[(2, 1, 4)] == b[(2, 4, 1)]
    dist = {(8, 1, 1): 0}
    frontier = [(8, 1, 1)]
    while frontier:
        nxt = []
        for u in frontier:
            for v in P.neighbors(u):
                if v not in dist:
                    dist[v] = dist[u] + 1; nxt.append(v)
        frontier = nxt
    for law in (a, b):
        for d in range(max(dist.values())):
            assert min(law[v] for v in dist if dist[v] == d) > max(law[v] for v in dist if dist[v] == d + 1)
    assert b[(8, 1, 1)] < a[(8, 1, 1)]
    mean_a = sum(float(a[v]) * dist[v] for v in dist)
    mean_b = sum(float(b[v]) * dist[v] for v in dist)
    assert mean_b > mean_a


@pytest.mark.parametrize("param,start,q", [(S.Factor(8, 3), (8, 1, 1), 0.5), (S.Factor(12, 2), (12, 1), 0.7),
                                           (S.Permutation(3), (0, 1, 2), 0.5), (S.Discrete([1, 2, 3, 4]), (0,), 0.5)])
def test_qwalk_process_montecarlo_matches_law(param, start, q):
    law = S.qwalk_law(param, start, Fraction(q).limit_denominator(100))
    rng = S.SplitMix64(99)
    n = 120000
    counts = {}
    for _ in range(n):
        v = S.qwalk(param, start, q, rng)
        counts[v] = counts.get(v, 0) + 1
    assert set(counts) <= set(law)
    for v, p in law.items():
        p = float(p)
        sigma = math.sqrt(p * (1 - p) / n)
        assert abs(counts.get(v, 0) / n - p) < 5 * sigma + 1e-9, (v, counts.get(v, 0) / n, p)


def test_qwalk_isolated_vertex_draws_nothing():
    rng = S.SplitMix64(5)
    before = rng.state
    assert S.qwalk(S.Factor(1, 3), (1, 1, 1), 0.9, rng) == (1, 1, 1)
    assert rng.state == before


# ------------------------------------------------------------------ recombination (Eq. 2)
def test_recombine_probabilities_eq2():
    assert S.recombine_probs([3.0, 1.0, 0.0]) == [0.75, 0.25, 0.0]
    assert S.recombine_probs([0.0, 0.0]) == [0.5, 0.5]
    space = S.Space([S.Categorical(3), S.Categorical(3)])
    parents = [(((0,), (0,)), 3.0), (((1,), (1,)), 1.0), (((2,), (2,)), 0.0)]
    rng = S.SplitMix64(11)
    n = 60000
    c = np.zeros((2, 3))
    mixed = 0
    for _ in range(n):
        x = S.recombine(space, parents, rng)
        c[0, x[0][0]] += 1; c[1, x[1][0]] += 1
        mixed += x[0] != x[1]
    assert c[0, 2] == 0 and c[1, 2] == 0          # zero-fitness parent never inherited (Sec. 4.2)
    assert np.all(np.abs(c[:, 0] / n - 0.75) < 0.01) and np.all(np.abs(c[:, 1] / n - 0.25) < 0.01)
    assert abs(mixed / n - 2 * 0.75 * 0.25) < 0.01  # parameters choose their parent independently
    zero = [(p, 0.0) for p, _ in parents]
    c = np.zeros(3)
    for _ in range(30000):
        c[S.recombine(space, zero, rng)[0][0]] += 1
    assert np.all(np.abs(c / 30000 - 1 / 3) < 0.01)


def test_select_parents_ranking_and_ties():
    Q = [("a", 1.0), ("b", 3.0), ("c", 3.0), ("d", 0.0), ("e", 2.0)]
    assert S.select_parents(Q, 3) == [1, 2, 4]
    assert S.select_parents(Q, 10) == [1, 2, 4, 0, 3]
    assert S.clamp_fitness(float("nan")) == 0.0 and S.clamp_fitness(-1.0) == 0.0


# ----------------------------------------------------------------------- Alg. 1 invariants
def _cfg1_space():
    return S.Space([S.Factor(64, 2), S.Factor(64, 2), S.Factor(64, 2)])


def _peak_fitness(target):
    def f(x):
        d = 0.0
        for v, t in zip(x, target):
            d += sum((math.log2(a + 1) - math.log2(b + 1)) ** 2 for a, b in zip(v, t))
        return 100.0 / (1.0 + d)
    return f


def test_space_rank_unrank_roundtrip():
    sp = S.Space([S.Factor(12, 2), S.Categorical(2), S.Permutation(3)])
    n = sp.size()
    assert n == 6 * 2 * 6
    allx = [sp.unrank(r) for r in range(n)]
    assert len(set(allx)) == n and all(sp.rank(x) == r for r, x in enumerate(allx))
    assert all(sp.is_legal(x) for x in allx)
    assert sp.unflat(sp.flat(allx[17])) == allx[17]


def test_opevo_never_repeats_all_legal_exact_budget():
    sp = S.Space([S.Factor(512, 4), S.Factor(1024, 4), S.Factor(1024, 2), S.Categorical(2)])
    f = _peak_fitness(((4, 2, 2, 32), (4, 2, 4, 32), (16, 64), (1,)))
    log = S.run_opevo(sp, f, budget=500, seed=3)
    assert len(log) == 500                      # 8 + 61*8 + 4: the last generation is cut short
    xs = [x for x, _ in log]
    assert len(set(xs)) == 500 and all(sp.is_legal(x) for x in xs)
    best = np.maximum.accumulate([fx for _, fx in log])
    assert best[-1] >= best[0] and np.all(np.diff(best) >= 0)


def test_opevo_exhausts_small_space_then_stops():
    sp = _cfg1_space()
    log = S.run_opevo(sp, _peak_fitness(((8, 8), (4, 16), (2, 32))), budget=1000, seed=1)
    assert len(log) == 343 and len({x for x, _ in log}) == 343
    t = S.OpEvo(sp, seed=1)
    while True:
        xs = t.ask()
        if not xs:
            break
        t.tell(xs, [1.0] * len(xs))
    assert len(t.Q) == 343 and t.ask() == []


def test_opevo_seed_reproducible_and_seed_sensitive():
    sp = _cfg1_space()
    f = _peak_fitness(((8, 8), (4, 16), (2, 32)))
    a = S.run_opevo(sp, f, 120, seed=42)
    b = S.run_opevo(sp, f, 120, seed=42)
    c = S.run_opevo(sp, f, 120, seed=43)
    assert a == b and a != c


def test_opevo_handles_all_zero_fitness():
    sp = _cfg1_space()
    log = S.run_opevo(sp, lambda x: 0.0, 64, seed=0)
    assert len(log) == 64 and len({x for x, _ in log}) == 64


def test_opevo_beats_uniform_random_search_on_average():
    sp = S.Space([S.Factor(512, 4), S.Factor(1024, 4), S.Factor(1024, 2)])
    target = ((4, 2, 2, 32), (4, 2, 4, 32), (16, 64))
    f = _peak_fitness(target)
    evo, rnd = [], []
    for seed in range(12):
        evo.append(max(fx for _, fx in S.run_opevo(sp, f, 300, seed=seed)))
        rng = S.SplitMix64(1000 + seed)
        rnd.append(max(f(sp.random(rng)) for _ in range(300)))
    assert np.mean(evo) > 1.5 * np.mean(rnd)


# ------------------------------------------ the plain-EA control (not the paper's; header-defined)
def test_uniform_mutation_law_and_draw_count():
    """Pin of the control: with probability p a parameter is redrawn uniformly, so every other vertex has
    probability p/|X_i| and the current one 1 - p + p/|X_i|; parameters are independent; a kept parameter
    costs one draw, a redrawn one two."""
    sp = S.Space([S.Factor(8, 3), S.Categorical(4)])
    x0 = ((8, 1, 1), (2,))
    p, n = 0.4, 100000
    rng = S.SplitMix64(123)
    counts = [{}, {}]
    joint_kept = 0
    for _ in range(n):
        y = sp.mutate_uniform(x0, p, rng)
        assert sp.is_legal(y)
        for i in range(2):
            counts[i][y[i]] = counts[i].get(y[i], 0) + 1
        joint_kept += (y == x0)
    for i, size in enumerate((10, 4)):
        assert len(counts[i]) == size
        for v, c in counts[i].items():
            want = p / size + ((1 - p) if v == x0[i] else 0.0)
            assert abs(c / n - want) < 5 * math.sqrt(want * (1 - want) / n), (v, c / n, want)
    want = (1 - p + p / 10) * (1 - p + p / 4)                    # independence of the parameters
    assert abs(joint_kept / n - want) < 5 * math.sqrt(want * (1 - want) / n)
    # p = 0 keeps everything and draws once per parameter; p close to 1 redraws everything (two draws each)
    a, b = S.SplitMix64(5), S.SplitMix64(5)
    assert sp.mutate_uniform(x0, 0.0, a) == x0
    for _ in range(2):
        b.next_u64()
    assert a.state == b.state
    a, b = S.SplitMix64(6), S.SplitMix64(6)
    sp.mutate_uniform(x0, 1.0 - 1e-16, a)
    for _ in range(4):
        b.next_u64()
    assert a.state == b.state


def test_uniform_mutation_control_keeps_the_rules_of_alg1():
    sp = _cfg1_space()
    f = _peak_fitness(((8, 8), (4, 16), (2, 32)))
    log = S.run_opevo(sp, f, budget=1000, seed=2, mutation="uniform")
    assert len(log) == 343 and len({x for x, _ in log}) == 343          # no duplicates, exhausts, stops
    a = S.run_opevo(sp, f, 100, seed=2, mutation="uniform")
    b = S.run_opevo(sp, f, 100, seed=2, mutation="walk")
    assert a[:8] == b[:8] and a != b                                    # same first generation, other children
