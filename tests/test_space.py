"""Configuration-space encoder and q-random walk of the library against the oracle (CPU)."""
from fractions import Fraction

import numpy as np
import pytest

import paper_2006_05664_amd as P
from oracle import search as S

SPECS = [
    ("factor", dict(type=P.OPEVO_FACTOR, C=8, nu=3), S.Factor(8, 3)),
    ("factor", dict(type=P.OPEVO_FACTOR, C=12, nu=3), S.Factor(12, 3)),
    ("factor", dict(type=P.OPEVO_FACTOR, C=56, nu=4), S.Factor(56, 4)),
    ("factor", dict(type=P.OPEVO_FACTOR, C=960, nu=2), S.Factor(960, 2)),
    ("factor", dict(type=P.OPEVO_FACTOR, C=1, nu=3), S.Factor(1, 3)),
    ("perm", dict(type=P.OPEVO_PERMUTATION, n_values=4), S.Permutation(4)),
    ("disc", dict(type=P.OPEVO_DISCRETE, values=[0.5, 2.0, 3.0, 10.0]), S.Discrete([0.5, 2.0, 3.0, 10.0])),
    ("cat", dict(type=P.OPEVO_CATEGORICAL, n_values=6), S.Categorical(6)),
    ("cat", dict(type=P.OPEVO_CATEGORICAL, n_values=1), S.Categorical(1)),
]


@pytest.mark.parametrize("kind,desc,oracle", SPECS)
def test_enumeration_and_neighbours_equal_oracle_in_order(kind, desc, oracle):
    sp = P.opevo_space_create([desc])
    try:
        V = [tuple(int(a) for a in v) for v in P.opevo_space_enumerate(sp, 0)]
        assert V == oracle.vertices()
        assert P.opevo_space_param_size(sp, 0) == len(V) == P.opevo_space_size(sp)
        for v in V:
            nb = [tuple(int(a) for a in u) for u in P.opevo_space_neighbors(sp, 0, v)]
            assert nb == oracle.neighbors(v)
            assert P.opevo_space_is_legal(sp, v)
    finally:
        P.opevo_space_destroy(sp)


def test_cfg_space_sizes_of_the_graded_workloads():
    want = {((512, 1024, 1024), P.OPEVO_MATMUL): 220 * 286 * 11 * 2,
            ((8192, 8192, 8192), P.OPEVO_MATMUL): 560 * 560 * 14 * 2,
            ((128, 128, 128, 64), P.OPEVO_BMM): 8 * 120 * 120 * 7 * 2,
            ((1, 64, 56, 56, 64, 3, 3, 1, 1), P.OPEVO_CONV2D): 1 * 84 * 80 * 80 * 21 * 2,
            ((32, 256, 14, 14, 256, 3, 3, 1, 1), P.OPEVO_CONV2D): 6 * 165 * 16 * 16 * 27 * 2}
    for (dims, kind), n in want.items():
        op = P.opevo_op_create(kind, dims, P.OPEVO_BF16)
        sp = P.opevo_op_space(op, P.OPEVO_TILE4)
        assert P.opevo_space_size(sp) == n
        P.opevo_space_destroy(sp); P.opevo_op_destroy(op)
    op = P.opevo_op_create(P.OPEVO_MATMUL, (64, 64, 64), P.OPEVO_F32)
    sp = P.opevo_op_space(op, P.OPEVO_TILE2)
    assert P.opevo_space_size(sp) == 343 and P.opevo_space_width(sp) == 6
    assert [P.opevo_space_param_name(sp, i) for i in range(3)] == ["M", "N", "K"]
    P.opevo_space_destroy(sp); P.opevo_op_destroy(op)


def _mixed():
    descs = [dict(type=P.OPEVO_FACTOR, C=12, nu=2, name="a"), dict(type=P.OPEVO_CATEGORICAL, n_values=2, name="f"),
             dict(type=P.OPEVO_PERMUTATION, n_values=3, name="p"), dict(type=P.OPEVO_DISCRETE, values=[1, 2, 4], name="d")]
    oracle = S.Space([S.Factor(12, 2), S.Categorical(2), S.Permutation(3), S.Discrete([1, 2, 4])])
    return P.opevo_space_create(descs), oracle


def test_legality_rank_unrank():
    sp, osp = _mixed()
    n = osp.size()
    assert P.opevo_space_size(sp) == n and P.opevo_space_width(sp) == 2 + 1 + 3 + 1
    assert P.opevo_space_param_slice(sp, 2) == (3, 3)
    for r in range(n):
        cfg = P.opevo_space_unrank(sp, r)
        assert list(cfg) == osp.flat(osp.unrank(r))
        assert P.opevo_space_rank(sp, cfg) == r and P.opevo_space_is_legal(sp, cfg)
    for bad in ([5, 2, 0, 0, 1, 2, 0], [12, 1, 2, 0, 1, 2, 0], [12, 1, 0, 0, 0, 2, 0], [12, 1, 0, 0, 1, 2, 3],
                [0, 0, 0, 0, 1, 2, 0], [-12, -1, 0, 0, 1, 2, 0]):
        assert not P.opevo_space_is_legal(sp, bad)
        with pytest.raises(P.OpevoError) as ei:
            P.opevo_space_rank(sp, bad)
        assert ei.value.status == P.OPEVO_E_ILLEGAL
    P.opevo_space_destroy(sp)


def test_random_walk_and_mutate_follow_the_oracle_draw_for_draw():
    sp, osp = _mixed()
    rng, orng = P.opevo_rng_create(2024), S.SplitMix64(2024)
    assert [P.opevo_rng_next_u64(rng) for _ in range(3)] == [orng.next_u64() for _ in range(3)]
    assert P.opevo_rng_next_double(rng) == orng.next_double()
    assert [P.opevo_rng_next_below(rng, 7) for _ in range(5)] == [orng.next_below(7) for _ in range(5)]
    for _ in range(200):
        x = P.opevo_space_random(sp, rng)
        ox = osp.random(orng)
        assert list(x) == osp.flat(ox)
        for q in (0.0, 0.5, 0.9):
            y = P.opevo_space_mutate(sp, q, rng, x)
            oy = osp.mutate(ox, q, orng)
            assert list(y) == osp.flat(oy)
    v = P.opevo_space_walk(sp, 0, 0.8, rng, [12, 1])
    assert tuple(v) == S.qwalk(osp.params[0], (12, 1), 0.8, orng)
    assert P.opevo_rng_next_u64(rng) == orng.next_u64()   # both consumed the same number of draws
    P.opevo_rng_destroy(rng); P.opevo_space_destroy(sp)


@pytest.mark.parametrize("desc,oracle,start", [
    (dict(type=P.OPEVO_FACTOR, C=8, nu=3), S.Factor(8, 3), (8, 1, 1)),
    (dict(type=P.OPEVO_FACTOR, C=56, nu=4), S.Factor(56, 4), (7, 2, 2, 2)),
    (dict(type=P.OPEVO_PERMUTATION, n_values=3), S.Permutation(3), (0, 1, 2)),
    (dict(type=P.OPEVO_DISCRETE, values=[1, 2, 3, 4]), S.Discrete([1, 2, 3, 4]), (0,)),
    (dict(type=P.OPEVO_CATEGORICAL, n_values=6), S.Categorical(6), (0,)),
    (dict(type=P.OPEVO_FACTOR, C=1, nu=2), S.Factor(1, 2), (1, 1)),
])
def test_exact_qwalk_law_matches_oracle_rationals(desc, oracle, start):
    sp = P.opevo_space_create([desc])
    for q in (Fraction(0), Fraction(1, 2), Fraction(7, 10), Fraction(19, 20)):
        law = oracle and S.qwalk_law(oracle, start, q)
        got = P.opevo_qrw_exact(sp, 0, start, float(q))
        want = np.array([float(law[v]) for v in oracle.vertices()])
        assert np.max(np.abs(got - want)) < 1e-13
        assert abs(got.sum() - 1.0) < 1e-13 and got.min() >= 0.0   # Thm 1 (App. A)
    P.opevo_space_destroy(sp)


def test_walk_histogram_matches_exact_law():
    sp = P.opevo_space_create([dict(type=P.OPEVO_FACTOR, C=8, nu=3)])
    rng = P.opevo_rng_create(5)
    law = P.opevo_qrw_exact(sp, 0, (8, 1, 1), 0.5)
    V = [tuple(v) for v in P.opevo_space_enumerate(sp, 0)]
    n = 60000
    counts = np.zeros(len(V))
    for _ in range(n):
        counts[V.index(tuple(P.opevo_space_walk(sp, 0, 0.5, rng, (8, 1, 1))))] += 1
    sigma = np.sqrt(law * (1 - law) / n)
    assert np.all(np.abs(counts / n - law) < 5 * sigma + 1e-9)
    P.opevo_rng_destroy(rng); P.opevo_space_destroy(sp)


def test_error_paths():
    for bad in ([dict(type=P.OPEVO_FACTOR, C=0, nu=2)], [dict(type=P.OPEVO_FACTOR, C=8, nu=0)],
                [dict(type=P.OPEVO_DISCRETE, values=[1, 1])], [dict(type=P.OPEVO_CATEGORICAL, n_values=0)],
                [dict(type=7)], []):
        with pytest.raises(P.OpevoError) as ei:
            P.opevo_space_create(bad)
        assert ei.value.status == P.OPEVO_E_ARG
    with pytest.raises(P.OpevoError) as ei:
        P.opevo_space_create([dict(type=P.OPEVO_FACTOR, C=2 ** 30, nu=12)])
    assert ei.value.status == P.OPEVO_E_TOO_LARGE
    sp = P.opevo_space_create([dict(type=P.OPEVO_FACTOR, C=8, nu=3)])
    rng = P.opevo_rng_create(1)
    for q in (1.0, -0.1, float("nan")):
        with pytest.raises(P.OpevoError) as ei:
            P.opevo_space_mutate(sp, q, rng, (8, 1, 1))
        assert ei.value.status == P.OPEVO_E_ARG
    with pytest.raises(P.OpevoError) as ei:
        P.opevo_space_mutate(sp, 0.5, rng, (8, 2, 1))
    assert ei.value.status == P.OPEVO_E_ILLEGAL
    with pytest.raises(P.OpevoError) as ei:
        P.opevo_space_neighbors(sp, 3, (8, 1, 1))
    assert ei.value.status == P.OPEVO_E_ARG
    P.opevo_rng_destroy(rng); P.opevo_space_destroy(sp)
