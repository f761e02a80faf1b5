"""Pins for oracle/plan_ref.py: brute-force enumeration, closed-form special cases and bounds."""
import itertools
import math
import random

import pytest

from oracle import plan_ref as P

random.seed(7)


# ------------------------------------------------------------------ Eq. 1
def test_oef_special_values():
    assert P.oef(3.0, 5.0, 5.0) == 1.0           # shorter operator completely hidden
    assert P.oef(3.0, 5.0, 8.0) == 0.0           # no gain over running back to back
    assert P.oef(3.0, 5.0, 9.5) == -0.5          # interference
    assert abs(P.oef(2.0, 4.0, 5.0) - 0.5) < 1e-15
    assert P.oef(3.0, 5.0, 6.0) == P.oef(5.0, 3.0, 6.0)


# ------------------------------------------------------------------ Eq. 2
def brute_paths(p_f, p_b, p_fb):
    """Minimum over every monotone lattice path with steps (1,0), (0,1), (1,1)."""
    nf, nb = len(p_f), len(p_b)
    best = [math.inf]

    def walk(i, j, acc):
        if i == nf and j == nb:
            best[0] = min(best[0], acc)
            return
        if i < nf:
            walk(i + 1, j, acc + p_f[i])
        if j < nb:
            walk(i, j + 1, acc + p_b[j])
        if i < nf and j < nb:
            walk(i + 1, j + 1, acc + p_fb[i][j])
    walk(0, 0, 0.0)
    return best[0]


@pytest.mark.parametrize("nf,nb", [(1, 1), (2, 3), (4, 4), (5, 3), (0, 3), (3, 0)])
def test_pair_dp_equals_brute_force(nf, nb):
    for _ in range(20):
        p_f = [random.uniform(1, 5) for _ in range(nf)]
        p_b = [random.uniform(1, 5) for _ in range(nb)]
        p_fb = [[random.uniform(0.5, 1.2) * max(p_f[i], p_b[j]) + random.uniform(0, 2) for j in range(nb)] for i in range(nf)]
        t, steps = P.pair_dp(p_f, p_b, p_fb)
        assert abs(t - brute_paths(p_f, p_b, p_fb)) < 1e-12
        # the reported steps cover each segment once, in order, and add up to the optimum
        acc, fi, bj = 0.0, 0, 0
        for i, j in steps:
            if i is not None:
                assert i == fi; fi += 1
            if j is not None:
                assert j == bj; bj += 1
            acc += p_fb[i][j] if (i is not None and j is not None) else (p_f[i] if i is not None else p_b[j])
        assert fi == nf and bj == nb and abs(acc - t) < 1e-12


def test_pair_dp_closed_forms_and_bounds():
    n = 5
    p_f = [random.uniform(1, 5) for _ in range(n)]
    p_b = [random.uniform(1, 5) for _ in range(n)]
    # no overlap at all: P(i,j) = P(i)+P(j)  ->  the plain sum
    t, _ = P.pair_dp(p_f, p_b, [[a + b for b in p_b] for a in p_f])
    assert abs(t - (sum(p_f) + sum(p_b))) < 1e-12
    # perfect overlap with equal per-index times -> the longer strand
    eq = [2.0] * n
    t, _ = P.pair_dp(eq, eq, [[2.0] * n for _ in range(n)])
    assert t == 2.0 * n
    # bounds max(sum) <= T_opt <= sum+sum whenever max <= P <= sum, and monotonicity in P
    p_fb = [[random.uniform(max(a, b), a + b) for b in p_b] for a in p_f]
    t, _ = P.pair_dp(p_f, p_b, p_fb)
    assert max(sum(p_f), sum(p_b)) - 1e-12 <= t <= sum(p_f) + sum(p_b) + 1e-12
    p_low = [[v * 0.9 for v in row] for row in p_fb]
    assert P.pair_dp(p_f, p_b, p_low)[0] <= t + 1e-12


# ------------------------------------------------------------------ segment cost (fluid model)
def table(nf, nb, fn):
    return [[fn(a, b) for b in range(nb)] for a in range(nf)]


def test_segment_cost_closed_forms():
    t_f = [1.0, 2.5, 0.7]; t_b = [2.0, 0.4, 1.1, 3.0]
    one = table(3, 4, lambda a, b: 1.0)
    # undisturbed co-run: the longer chain
    assert abs(P.segment_cost([0, 1, 2], [0, 1, 2, 3], t_f, t_b, one, one) - max(sum(t_f), sum(t_b))) < 1e-12
    # time slicing (rates add to 1): work conserving, the plain sum
    rf = table(3, 4, lambda a, b: 0.3 + 0.1 * ((a + b) % 3)); rb = [[1 - v for v in row] for row in rf]
    assert abs(P.segment_cost([0, 1, 2], [0, 1, 2, 3], t_f, t_b, rf, rb) - (sum(t_f) + sum(t_b))) < 1e-12
    # one side empty: solo time
    assert P.segment_cost([1, 2], [], t_f, t_b, rf, rb) == t_f[1] + t_f[2]
    assert P.segment_cost([], [3], t_f, t_b, rf, rb) == t_b[3]
    # single pair by hand: a needs 1/0.5 = 2, b needs 2/0.8 = 2.5 -> a ends at 2, b has 2-1.6 = 0.4 left
    assert abs(P.segment_cost([0], [0], t_f, t_b, table(3, 4, lambda a, b: 0.5), table(3, 4, lambda a, b: 0.8)) - 2.4) < 1e-12


def test_rates_round_trip_reproduces_profiled_pair_time():
    for _ in range(50):
        ta, tb = random.uniform(1, 5), random.uniform(1, 5)
        ra, rb = random.uniform(0.3, 1), random.uniform(0.3, 1)
        # synthesise finish times from the model, recover rates, re-simulate
        p = P.segment_cost([0], [0], [ta], [tb], [[ra]], [[rb]])
        t1 = min(ta / ra, tb / rb)
        end_a, end_b = (t1, p) if ta / ra <= tb / rb else (p, t1)
        qa, qb = P.rates_from_corun(ta, tb, end_a, end_b)
        assert abs(P.segment_cost([0], [0], [ta], [tb], [[qa]], [[qb]]) - max(end_a, end_b)) < 1e-12
        if ta / ra <= tb / rb:
            assert abs(qa - ra) < 1e-12 and abs(qb - rb) < 1e-12


# ------------------------------------------------------------------ barrier placement
def brute_cuts(seq_f, seq_b, t_f, t_b, rf, rb, bc):
    nf, nb = len(seq_f), len(seq_b)
    best = [math.inf]

    def walk(i, j, acc):
        if i == nf and j == nb:
            best[0] = min(best[0], acc)
            return
        for i2 in range(i, nf + 1):
            for j2 in range(j, nb + 1):
                if (i2, j2) != (i, j):
                    walk(i2, j2, acc + P.segment_cost(seq_f[i:i2], seq_b[j:j2], t_f, t_b, rf, rb) + bc)
    walk(0, 0, 0.0)
    return best[0]


@pytest.mark.parametrize("nf,nb,bc", [(2, 2, 0.0), (3, 4, 0.0), (4, 3, 0.05), (1, 4, 0.0)])
def test_search_cuts_equals_brute_force(nf, nb, bc):
    for _ in range(6):
        t_f = [random.uniform(0.5, 3) for _ in range(nf)]
        t_b = [random.uniform(0.5, 3) for _ in range(nb)]
        rf = table(nf, nb, lambda a, b: random.uniform(0.2, 1.0))
        rb = table(nf, nb, lambda a, b: random.uniform(0.2, 1.0))
        sf, sb = list(range(nf)), list(range(nb))
        m, pairs = P.search_cuts(sf, sb, t_f, t_b, rf, rb, bc)
        assert abs(m - brute_cuts(sf, sb, t_f, t_b, rf, rb, bc)) < 1e-12
        # pairs tile both sequences and re-add to the makespan
        acc, fi, bj = 0.0, 0, 0
        for f0, f1, b0, b1 in pairs:
            assert f0 == fi and b0 == bj and (f1 > f0 or b1 > b0)
            acc += P.segment_cost(sf[f0:f1], sb[b0:b1], t_f, t_b, rf, rb) + bc
            fi, bj = f1, b1
        assert fi == nf and bj == nb and abs(acc - m) < 1e-12
        # never worse than running the strands back to back or as one free-running pair
        assert m <= sum(t_f) + sum(t_b) + 2 * bc + 1e-12
        assert m <= P.segment_cost(sf, sb, t_f, t_b, rf, rb) + bc + 1e-12


def test_search_cuts_avoids_interfering_pair():
    # forward op 0 and backward op 0 thrash each other (rates 0.2): better to serialise them with a barrier
    t_f = [1.0]; t_b = [1.0]
    m, pairs = P.search_cuts([0], [0], t_f, t_b, [[0.2]], [[0.2]])
    assert abs(m - 2.0) < 1e-12 and len(pairs) == 2
    m, pairs = P.search_cuts([0], [0], t_f, t_b, [[0.9]], [[0.9]])
    assert abs(m - 1.0 / 0.9) < 1e-12 and len(pairs) == 1


# ------------------------------------------------------------------ sequencing
def test_topo_orders_counts():
    assert len(P.topo_orders(4, [])) == 24
    assert P.topo_orders(3, [(0, 1), (1, 2)]) == [[0, 1, 2]]
    # a chain 0->1->2 with a free node 3 hanging off node 0: it may sit in 3 places
    assert len(P.topo_orders(4, [(0, 1), (1, 2), (0, 3)])) == 3
    for o in P.topo_orders(5, [(0, 2), (1, 2), (2, 4)]):
        assert o.index(0) < o.index(2) and o.index(1) < o.index(2) and o.index(2) < o.index(4)


def test_search_uses_movable_operator():
    # backward: chain b0 -> b1 plus a movable "wgrad" b2 that only needs b0.
    # forward: one long communication-like operator that overlaps perfectly with b2 only.
    kinds_f, deps_f = [0], []
    kinds_b, deps_b = [0, 1, 2], [(0, 1), (0, 2)]
    t_f = [2.0]; t_b = [1.0, 1.0, 2.0]
    rate_f = [[0.5, 0.5, 1.0]]; rate_b = [[0.5, 0.5, 1.0]]
    m, of, ob, pairs = P.search(kinds_f, deps_f, kinds_b, deps_b, t_f, t_b, rate_f, rate_b)
    assert abs(m - 4.0) < 1e-12     # b0, b1 alone (2.0) + f0 || b2 (2.0), in either order
    tot = sum(t_f) + sum(t_b)
    assert m < tot
