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


# ------------------------------------------------------------------ lane model (more than two participants)
def rand_tab(nf, nb, lo=0.3):
    t_f = [random.uniform(0.5, 3) for _ in range(nf)]
    t_b = [random.uniform(0.5, 3) for _ in range(nb)]
    rf = [[random.uniform(lo, 1.0) for _ in range(nb)] for _ in range(nf)]
    rb = [[random.uniform(lo, 1.0) for _ in range(nb)] for _ in range(nf)]
    return t_f, t_b, rf, rb


def test_lane_cost_reduces_to_the_two_queue_model():
    """No stream of its own for any stand-in, nothing beside the strand: two lanes, i.e. segment_cost, whatever the
    operator graphs and kinds say."""
    for _ in range(50):
        t_f, t_b, rf, rb = rand_tab(5, 6)
        sf = random.sample(range(5), random.randrange(0, 6))
        sb = random.sample(range(6), random.randrange(0, 7))
        ref = P.segment_cost(sf, sb, t_f, t_b, rf, rb)
        got = P.lane_cost(sf, sb, t_f, t_b, rf, rb, deps_f=[(0, 1)], deps_b=[(2, 3)], comm_f={1: 1}, comm_b={2: 1, 4: 2},
                          lanes=(0, 0, 0))
        assert abs(got - ref) <= 1e-12 * max(1.0, ref)


def test_lane_cost_closed_forms():
    one = [[1.0] * 4 for _ in range(3)]
    t_f, t_b = [2.0, 5.0, 1.0], [1.0, 4.0, 3.0, 2.0]
    # backward strand alone: compute 0, collective 1 (own lane), independent compute 2, consumer 3 of the collective.
    # The collective starts after op 0; op 2 overlaps it; op 3 waits for both: 1 + max(4, 3) + 2
    kw = dict(deps_b=[(0, 1), (1, 3)], comm_b={1: 1}, lanes=(0, 1, 0))
    assert abs(P.lane_cost([], [0, 1, 2, 3], t_f, t_b, one, one, **kw) - (1 + 4 + 2)) < 1e-12
    # the same with the collective in the strand's own stream: everything in a row
    assert abs(P.lane_cost([], [0, 1, 2, 3], t_f, t_b, one, one, deps_b=kw["deps_b"], comm_b={1: 1}, lanes=(0, 0, 0)) - 10) < 1e-12
    # the independent operator issued BEFORE the collective cannot overlap it (streams run in issue order)
    assert abs(P.lane_cost([], [0, 2, 1, 3], t_f, t_b, one, one, **kw) - (1 + 3 + 4 + 2)) < 1e-12
    # both strands' collectives on one shared communication stream run one after the other in issue order;
    # on separate streams they overlap.  forward: compute 0 (2), collective 1 (5), consumer 2 (1);
    # backward: compute 0 (1), collective 1 (4), consumer 3 (2)
    f = dict(deps_f=[(0, 1), (1, 2)], comm_f={1: 1}, deps_b=[(0, 1), (1, 3)], comm_b={1: 1})
    shared = P.lane_cost([0, 1, 2], [0, 1, 3], t_f, t_b, one, one, lanes=(1, 1, 0), **f)
    # forward collective issued first: starts at 2, ends 7; backward's starts at 7 (its strand was ready at 1), ends 11, consumer 13
    assert abs(shared - 13.0) < 1e-12
    apart = P.lane_cost([0, 1, 2], [0, 1, 3], t_f, t_b, one, one, lanes=(1, 2, 0), **f)
    assert abs(apart - max(2 + 5 + 1, 1 + 4 + 2)) < 1e-12
    # an operator beside its strand runs in alpha's stream behind beta's issued work: beta 0 (1), side op 2 (3) on alpha
    # after alpha's op 0 (2) and beta's op 0, beta goes on with op 3 (2) meanwhile
    side = P.lane_cost([0], [0, 2, 3], t_f, t_b, one, one, side=(2,))
    assert abs(side - max(2 + 3, 1 + 2)) < 1e-12
    # slow-down of three participants multiplies: forward compute 0 against backward compute 0 and backward collective 1
    rf = [[0.5, 0.5, 1, 1]] + [[1.0] * 4] * 2
    tri = P.lane_cost([0], [1, 0], [4.0, 1, 1], [8.0, 8.0, 1, 1], rf, one, comm_b={1: 1}, lanes=(0, 2, 0))
    # backward issues op 1 (collective, own lane, 8) then op 0 (compute, 8): both run from t = 0 undisturbed; forward op 0
    # advances at 0.5 * 0.5: 2 of its 4 units are done at t = 8, the rest runs alone
    assert abs(tri - 10.0) < 1e-12


def brute_force_lanes(jobs_spec, dt=1e-3):
    """Independent check by time stepping.  jobs_spec: list of (stream, work, after, rate_fn) with rate_fn(k, running)."""
    left = [w for _, w, _, _ in jobs_spec]
    done = [False] * len(jobs_spec)
    t = 0.0
    while not all(done):
        running, seen = [], set()
        for k, (stream, _, after, _) in enumerate(jobs_spec):
            if done[k] or stream in seen:
                continue
            seen.add(stream)                       # the first unfinished job of a stream
            if all(done[a] for a in after):
                running.append(k)
        for k in running:
            left[k] -= jobs_spec[k][3](k, running) * dt
        for k in running:
            if left[k] <= 0:
                done[k] = True
        t += dt
    return t


def test_lane_cost_against_time_stepping():
    """Three lanes, pairwise rates multiplied: the event-driven result against plain time stepping."""
    for _ in range(6):
        t_f, t_b, rf, rb = rand_tab(2, 3, lo=0.5)
        # forward: ops 0, 1 in alpha's stream.  backward: op 0 compute, op 1 collective (own lane, like forward op 1),
        # op 2 compute independent of the collective
        like_b = {1: 1}
        got = P.lane_cost([0, 1], [0, 1, 2], t_f, t_b, rf, rb, deps_b=[(0, 1)], comm_b={1: 1}, lanes=(0, 2, 0), like_b=like_b)

        def rate(k, running):
            ident = {0: ("f", 0), 1: ("f", 1), 2: ("b", 0), 3: ("b", 1), 4: ("b", 2)}
            r = 1.0
            for o in running:
                if o == k:
                    continue
                (xd, xo), (yd, yo) = ident[k], ident[o]
                if xd == yd:
                    if yd == "b" and yo in like_b:
                        yd, yo = "f", like_b[yo]
                    elif xd == "b" and xo in like_b:
                        xd, xo = "f", like_b[xo]
                    else:
                        continue
                r *= rf[xo][yo] if xd == "f" else rb[yo][xo]
            return r
        spec = [("A", t_f[0], [], rate), ("A", t_f[1], [], rate), ("B", t_b[0], [], rate), ("CB", t_b[1], [2], rate),
                ("B", t_b[2], [], rate)]
        ref = brute_force_lanes(spec)
        assert abs(got - ref) <= 6e-3
