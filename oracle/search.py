"""TEST INFRASTRUCTURE ONLY: the search-space and OpEvo oracle, in plain Python.

Written from the paper's definitions, step by step and in its notation:

* the four parameter types and their adjacency graphs (Sec. 3),
* the q-random-walk distribution, both as the stochastic process of Sec. 4.3 /
  Eq. 3 and as the closed form S = (1-q)(I-Q)^-1 p0 of App. A (in exact
  rational arithmetic),
* selection + recombination (Sec. 4.2, Eq. 2) and the loop of Alg. 1 (Sec. 4.4)
  with its no-duplicate rule.

The product library implements the same method in C++; the two share no code.
So that whole trajectories can be compared bit for bit, both sides draw their
random numbers from the same published counter-based generator (SplitMix64,
Steele, Lea & Flood 2014) in the same documented order; that order is part of
the interface and is restated where each draw happens.

Where the paper is silent this file takes these readings (all listed again in
the design notes of the repository):
  R-ties     top-lambda ranking: higher fitness first, earlier trial first among equals
  R-zero     Eq. 2 with all-zero parent fitness: parents drawn uniformly; fitness < 0 or NaN counts as 0
  R-isolated a vertex with no neighbour ends the walk at once (Eq. 3 would divide by 0)
  R-init     "randomly generate": each parameter uniform over its feasible set, independently
  R-dup      a child that was sampled before (evaluated or still pending) is mutated again,
             starting from the rejected mutant; after 100 such re-mutations a uniformly
             random unsampled configuration is taken; none left => the space is exhausted
  R-budget   a trial is one evaluated configuration, the initial lambda included

One thing here is NOT the paper's: `Space.mutate_uniform` and `OpEvo(..., mutation="uniform")`,
the control experiment that replaces the topology-aware walk by the mutation of a plain
evolutionary algorithm (per parameter, with probability p, a uniformly random vertex of its
feasible set), so that what Sec. 4.3's walk buys can be measured.  Its definition is the one
stated in the library's header; its law is p/|X_i| for every other vertex and 1 - p + p/|X_i| for
the current one, which is what the tests pin it to.
"""
from __future__ import annotations

from fractions import Fraction
from itertools import permutations as _permutations
from typing import Callable, Dict, List, Optional, Sequence, Tuple

MASK64 = (1 << 64) - 1
REMUTATE_CAP = 100
ENUM_LIMIT = 1 << 20      # spaces up to this size list their unsampled members exactly
REJECT_TRIES = 10000      # larger spaces: rejection sampling of an unsampled member

Vertex = Tuple[int, ...]


# --------------------------------------------------------------------------- RNG
class SplitMix64:
    """Counter-based generator: output i is mix(seed + (i+1)*gamma)."""

    GAMMA = 0x9E3779B97F4A7C15

    def __init__(self, seed: int):
        self.state = seed & MASK64

    def next_u64(self) -> int:
        self.state = (self.state + self.GAMMA) & MASK64
        z = self.state
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & MASK64
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & MASK64
        return z ^ (z >> 31)

    def next_double(self) -> float:
        """Uniform in [0,1): top 53 bits scaled by 2^-53."""
        return (self.next_u64() >> 11) * (1.0 / 9007199254740992.0)

    def next_below(self, n: int) -> int:
        """Integer in [0,n) for 0 < n < 2^32: high half of (top 32 bits) * n."""
        assert 0 < n < (1 << 32)
        return ((self.next_u64() >> 32) * n) >> 32


# ----------------------------------------------------------- parameter types (Sec. 3)
def distinct_primes(n: int) -> List[int]:
    ps, p = [], 2
    while p * p <= n:
        if n % p == 0:
            ps.append(p)
            while n % p == 0:
                n //= p
        p += 1
    if n > 1:
        ps.append(n)
    return ps


class Param:
    """One component feasible set X_i with its adjacency graph."""

    width = 1  # int32 slots in the flat encoding

    def vertices(self) -> List[Vertex]:
        raise NotImplementedError

    def neighbors(self, u: Vertex) -> List[Vertex]:
        raise NotImplementedError

    def is_legal(self, u: Vertex) -> bool:
        return tuple(u) in set(self.vertices())


class Factor(Param):
    """nu-tuples of positive integers with product C.  u ~ v iff v is u with one
    prime z moved from factor n to another factor m (Sec. 3)."""

    def __init__(self, C: int, nu: int):
        assert C >= 1 and nu >= 1
        self.C, self.nu, self.width = C, nu, nu

    def vertices(self) -> List[Vertex]:
        # lexicographic order: first factor ascending, then the second, ...
        def rec(c: int, slots: int) -> List[Vertex]:
            if slots == 1:
                return [(c,)]
            out = []
            for d in range(1, c + 1):
                if c % d == 0:
                    out += [(d,) + t for t in rec(c // d, slots - 1)]
            return out
        return rec(self.C, self.nu)

    def neighbors(self, u: Vertex) -> List[Vertex]:
        # order: source position n ascending, prime z of u_n ascending, target m ascending
        out = []
        for n in range(self.nu):
            for z in distinct_primes(u[n]):
                for m in range(self.nu):
                    if m != n:
                        v = list(u)
                        v[n] //= z
                        v[m] *= z
                        out.append(tuple(v))
        return out

    def is_legal(self, u: Vertex) -> bool:
        if len(u) != self.nu or any(a < 1 for a in u):
            return False
        p = 1
        for a in u:
            p *= a
        return p == self.C


class Permutation(Param):
    """All orders of n items; u ~ v iff they differ by one transposition (Sec. 3)."""

    def __init__(self, n: int):
        assert n >= 1
        self.n, self.width = n, n

    def vertices(self) -> List[Vertex]:
        return [tuple(p) for p in _permutations(range(self.n))]  # lexicographic

    def neighbors(self, u: Vertex) -> List[Vertex]:
        out = []
        for i in range(self.n):
            for j in range(i + 1, self.n):
                v = list(u)
                v[i], v[j] = v[j], v[i]
                out.append(tuple(v))
        return out

    def is_legal(self, u: Vertex) -> bool:
        return sorted(u) == list(range(self.n))


class Discrete(Param):
    """Finitely many reals; u ~ v iff no member lies strictly between them, u != v
    (Sec. 3).  A vertex is the index into the ascending value list."""

    def __init__(self, values: Sequence[float]):
        vals = list(values)
        assert len(vals) >= 1 and all(a < b for a, b in zip(vals, vals[1:])), \
            "values must be strictly ascending"
        self.values = vals

    def vertices(self) -> List[Vertex]:
        return [(i,) for i in range(len(self.values))]

    def neighbors(self, u: Vertex) -> List[Vertex]:
        # straight from the adjacency function, so the path structure is derived, not assumed
        i = u[0]
        out = []
        for j in range(len(self.values)):
            if j == i:
                continue
            between = any((w - self.values[i]) * (w - self.values[j]) < 0 for w in self.values)
            if not between:
                out.append((j,))
        return out

    def is_legal(self, u: Vertex) -> bool:
        return len(u) == 1 and 0 <= u[0] < len(self.values)


class Categorical(Param):
    """J unordered choices; every two distinct choices are adjacent (Sec. 3)."""

    def __init__(self, J: int):
        assert J >= 1
        self.J = J

    def vertices(self) -> List[Vertex]:
        return [(i,) for i in range(self.J)]

    def neighbors(self, u: Vertex) -> List[Vertex]:
        return [(j,) for j in range(self.J) if j != u[0]]

    def is_legal(self, u: Vertex) -> bool:
        return len(u) == 1 and 0 <= u[0] < self.J


# -------------------------------------------------- q-random walk (Sec. 4.3, App. A)
def transition_matrix(param: Param, q) -> Tuple[List[Vertex], List[List]]:
    """Q with Q[v][u] = q/|S(u)| for v in S(u) (Eq. 3); p(t) = Q p(t-1) (App. A)."""
    V = param.vertices()
    index = {v: i for i, v in enumerate(V)}
    zero = q - q
    Q = [[zero for _ in V] for _ in V]
    for u in V:
        S = param.neighbors(u)
        for v in S:
            Q[index[v]][index[u]] += q / len(S)
    return V, Q


def qwalk_law(param: Param, start: Vertex, q) -> Dict[Vertex, Fraction]:
    """Exact stop distribution S = (1-q)(I-Q)^-1 p0 (App. A, proof of Thm 1),
    by Gauss-Jordan elimination over the rationals."""
    q = Fraction(q)
    V, Q = transition_matrix(param, q)
    n = len(V)
    if not param.neighbors(tuple(start)):
        # R-isolated: Eq. 3 has no meaning for |S(u)| = 0; the walk cannot move, so it stops at u
        return {v: Fraction(1 if v == tuple(start) else 0) for v in V}
    A = [[(Fraction(1) if i == j else Fraction(0)) - Q[i][j] for j in range(n)] for i in range(n)]
    b = [(1 - q) if V[i] == tuple(start) else Fraction(0) for i in range(n)]
    for c in range(n):
        piv = next(r for r in range(c, n) if A[r][c] != 0)
        A[c], A[piv] = A[piv], A[c]
        b[c], b[piv] = b[piv], b[c]
        inv = 1 / A[c][c]
        A[c] = [a * inv for a in A[c]]
        b[c] *= inv
        for r in range(n):
            if r != c and A[r][c] != 0:
                f = A[r][c]
                A[r] = [x - f * y for x, y in zip(A[r], A[c])]
                b[r] -= f * b[c]
    return {V[i]: b[i] for i in range(n)}


def qwalk_law_series(param: Param, start: Vertex, q: float, terms: int = 400) -> Dict[Vertex, float]:
    """The same law from its definition as a series, S = (1-q) sum_t Q^t p0
    (App. A, first line of the proof of Thm 1), truncated after `terms` steps."""
    V, Q = transition_matrix(param, float(q))
    n = len(V)
    if not param.neighbors(tuple(start)):
        return {v: (1.0 if v == tuple(start) else 0.0) for v in V}
    p = [1.0 if V[i] == tuple(start) else 0.0 for i in range(n)]
    S = [0.0] * n
    for _ in range(terms):
        S = [s + (1.0 - q) * x for s, x in zip(S, p)]
        p = [sum(Q[i][j] * p[j] for j in range(n)) for i in range(n)]
    return {V[i]: S[i] for i in range(n)}


def qwalk(param: Param, u: Vertex, q: float, rng: SplitMix64) -> Vertex:
    """One draw from the q-random-walk distribution, as the process of Sec. 4.3:
    with probability 1-q stop, otherwise move to a uniformly chosen neighbour.
    Draw order: [next_double() for stop/continue, then next_below(|S(u)|)] per step;
    an isolated vertex returns without drawing."""
    u = tuple(u)
    while True:
        S = param.neighbors(u)
        if not S:
            return u
        if not (rng.next_double() < q):
            return u
        u = S[rng.next_below(len(S))]


# ------------------------------------------------------ configurations (Sec. 3, Eq. 1)
Config = Tuple[Vertex, ...]


class Space:
    """Cartesian product of the component feasible sets."""

    def __init__(self, params: Sequence[Param]):
        self.params = list(params)
        self._verts = [p.vertices() for p in self.params]
        self._index = [{v: i for i, v in enumerate(vs)} for vs in self._verts]

    def size(self) -> int:
        n = 1
        for vs in self._verts:
            n *= len(vs)
        return n

    def flat(self, x: Config) -> List[int]:
        return [a for v in x for a in v]

    def unflat(self, flat: Sequence[int]) -> Config:
        out, k = [], 0
        for p in self.params:
            out.append(tuple(int(a) for a in flat[k:k + p.width]))
            k += p.width
        assert k == len(flat)
        return tuple(out)

    def is_legal(self, x: Config) -> bool:
        return len(x) == len(self.params) and all(p.is_legal(v) for p, v in zip(self.params, x))

    def rank(self, x: Config) -> int:
        """Mixed-radix index, parameter 0 most significant, digits in enumeration order."""
        r = 0
        for vs, idx, v in zip(self._verts, self._index, x):
            r = r * len(vs) + idx[v]
        return r

    def unrank(self, r: int) -> Config:
        out = []
        for vs in reversed(self._verts):
            out.append(vs[r % len(vs)])
            r //= len(vs)
        return tuple(reversed(out))

    def random(self, rng: SplitMix64) -> Config:
        """R-init: parameter by parameter, index = next_below(|X_i|) in enumeration order."""
        return tuple(vs[rng.next_below(len(vs))] for vs in self._verts)

    def mutate(self, x: Config, q: float, rng: SplitMix64) -> Config:
        """Sec. 4.3: an independent q-random walk on every parameter, in order."""
        return tuple(qwalk(p, v, q, rng) for p, v in zip(self.params, x))


    def mutate_uniform(self, x: Config, p: float, rng: SplitMix64) -> Config:
        """The control (not in the paper): the parameter graphs are ignored.  Parameter by parameter,
        in order: u = next_double(); if u < p the parameter becomes vertex number
        next_below(|X_i|) of its feasible set in enumeration order (which may be the vertex it
        already had); otherwise it is kept and no second number is drawn."""
        out = []
        for vs, v in zip(self._verts, x):
            if rng.next_double() < p:
                v = vs[rng.next_below(len(vs))]
            out.append(v)
        return tuple(out)


# ----------------------------------------------- selection + recombination (Sec. 4.2)
def clamp_fitness(f: float) -> float:
    return f if f > 0.0 else 0.0  # also maps NaN to 0


def select_parents(Q: List[Tuple[Config, float]], lam: int) -> List[int]:
    """Indices into Q of the top-lambda individuals (R-ties)."""
    order = sorted(range(len(Q)), key=lambda t: (-Q[t][1], t))
    return order[:lam]


def recombine_probs(fitness: Sequence[float]) -> List[float]:
    """Eq. 2: P(x_i = x_i^j) = f(x^j) / sum_k f(x^k); uniform if the sum is 0 (R-zero)."""
    tot = 0.0
    for f in fitness:
        tot += f
    if tot > 0.0:
        return [f / tot for f in fitness]
    return [1.0 / len(fitness)] * len(fitness)


def recombine(space: Space, parents: List[Tuple[Config, float]], rng: SplitMix64) -> Config:
    """One child: each parameter copied whole from a parent drawn by Eq. 2.
    Draw order per parameter: if total > 0, t = next_double()*total and the parent is the
    first j with t < f_1+...+f_j (running sum in rank order, last positive parent if rounding
    runs past the end); else j = next_below(number of parents)."""
    total = 0.0
    for _, f in parents:
        total += f
    child = []
    for i in range(len(space.params)):
        if total > 0.0:
            t = rng.next_double() * total
            acc, j, last_pos = 0.0, None, None
            for idx, (_, f) in enumerate(parents):
                acc += f
                if f > 0.0:
                    last_pos = idx
                if t < acc:
                    j = idx
                    break
            if j is None:
                j = last_pos
        else:
            j = rng.next_below(len(parents))
        child.append(parents[j][0][i])
    return tuple(child)


# ------------------------------------------------------------------ Alg. 1 (Sec. 4.4)
class OpEvo:
    """ask/tell form of Alg. 1.  `ask(n)` returns up to n new configurations
    (the first generation is lambda random ones, later ones rho children);
    `tell` enqueues evaluated (configuration, fitness) pairs into Q."""

    def __init__(self, space: Space, lam: int = 8, rho: int = 8, q: float = 0.5, seed: int = 0,
                 mutation: str = "walk"):
        assert lam >= 1 and rho >= 1 and 0.0 <= q < 1.0 and mutation in ("walk", "uniform")
        self.space, self.lam, self.rho, self.q = space, lam, rho, q
        # "walk": Sec. 4.3's q-random walk on every parameter (Alg. 1 as published);
        # "uniform": the plain-EA control, q then being the per-parameter resampling probability
        self._mutate = space.mutate if mutation == "walk" else space.mutate_uniform
        self.rng = SplitMix64(seed)
        self.Q: List[Tuple[Config, float]] = []   # in trial order
        self.sampled = set()                      # evaluated or pending (R-dup)
        self.started = False

    def _random_unsampled(self) -> Optional[Config]:
        n = self.space.size()
        if len(self.sampled) >= n:
            return None
        if n <= ENUM_LIMIT:
            taken = {self.space.rank(x) for x in self.sampled}
            free = [r for r in range(n) if r not in taken]
            return self.space.unrank(free[self.rng.next_below(len(free))])
        for _ in range(REJECT_TRIES):
            x = self.space.random(self.rng)
            if x not in self.sampled:
                return x
        return None

    def _fresh(self, x: Config, redraw: Callable[[Config], Config]) -> Optional[Config]:
        tries = 0
        while x in self.sampled:
            if tries == REMUTATE_CAP:
                return self._random_unsampled()
            x = redraw(x)
            tries += 1
        return x

    def ask(self, max_n: Optional[int] = None) -> List[Config]:
        want = self.lam if not self.started else self.rho
        if max_n is not None:
            want = min(want, max_n)
        out: List[Config] = []
        if not self.started:
            for _ in range(want):
                x = self._fresh(self.space.random(self.rng), lambda _x: self.space.random(self.rng))
                if x is None:
                    break
                self.sampled.add(x)
                out.append(x)
            self.started = True
            return out
        parents = [self.Q[t] for t in select_parents(self.Q, self.lam)]
        for _ in range(want):
            child = recombine(self.space, parents, self.rng)
            child = self._mutate(child, self.q, self.rng)
            child = self._fresh(child, lambda x: self._mutate(x, self.q, self.rng))
            if child is None:
                break
            self.sampled.add(child)
            out.append(child)
        return out

    def tell(self, configs: Sequence[Config], fitness: Sequence[float]) -> None:
        for x, f in zip(configs, fitness):
            self.sampled.add(x)
            self.Q.append((x, clamp_fitness(f)))

    def best(self) -> Tuple[Config, float, int]:
        t = select_parents(self.Q, 1)[0]
        return self.Q[t][0], self.Q[t][1], t


def run_opevo(space: Space, f: Callable[[Config], float], budget: int, lam: int = 8, rho: int = 8,
              q: float = 0.5, seed: int = 0, mutation: str = "walk") -> List[Tuple[Config, float]]:
    """Alg. 1 until `budget` configurations were evaluated (R-budget) or the space is exhausted."""
    tuner = OpEvo(space, lam, rho, q, seed, mutation)
    while len(tuner.Q) < budget:
        xs = tuner.ask(budget - len(tuner.Q))
        if not xs:
            break
        tuner.tell(xs, [f(x) for x in xs])
    return tuner.Q
