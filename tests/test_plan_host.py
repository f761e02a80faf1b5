"""Host-side planner of the library (C++) against the plan oracle (Python).  No GPU needed."""
import random

import pytest

from oracle import plan_ref as P
from paper_2411_15871_amd import dhelix as dh

random.seed(11)


def rand_table(nf, nb):
    t_f = [random.uniform(0.5, 3) for _ in range(nf)]
    t_b = [random.uniform(0.5, 3) for _ in range(nb)]
    rf = [[random.uniform(0.2, 1.0) for _ in range(nb)] for _ in range(nf)]
    rb = [[random.uniform(0.2, 1.0) for _ in range(nb)] for _ in range(nf)]
    return t_f, t_b, rf, rb


def test_oef_matches_eq1():
    for _ in range(20):
        a, b, p = random.uniform(1, 5), random.uniform(1, 5), random.uniform(1, 9)
        assert abs(dh.dh_oef(a, b, p) - P.oef(a, b, p)) < 1e-15


@pytest.mark.parametrize("nf,nb", [(1, 1), (3, 5), (6, 4), (0, 3), (4, 0)])
def test_pair_dp_matches_oracle(nf, nb):
    for _ in range(10):
        p_f = [random.uniform(1, 5) for _ in range(nf)]
        p_b = [random.uniform(1, 5) for _ in range(nb)]
        p_fb = [[random.uniform(max(a, b), a + b) for b in p_b] for a in p_f]
        t, steps = dh.dh_pair_dp(p_f, p_b, p_fb)
        t_ref, _ = P.pair_dp(p_f, p_b, p_fb)
        assert abs(t - t_ref) <= 1e-12 * max(1.0, t_ref)
        acc = sum(p_fb[i][j] if (i is not None and j is not None) else (p_f[i] if i is not None else p_b[j]) for i, j in steps)
        assert abs(acc - t) < 1e-9
        assert [i for i, _ in steps if i is not None] == list(range(nf))
        assert [j for _, j in steps if j is not None] == list(range(nb))


def test_segment_cost_matches_oracle():
    t_f, t_b, rf, rb = rand_table(6, 7)
    tab = dh.make_table(t_f, t_b, rf, rb)
    for _ in range(200):
        sf = [random.randrange(6) for _ in range(random.randrange(0, 6))]
        sb = [random.randrange(7) for _ in range(random.randrange(0, 6))]
        ref = P.segment_cost(sf, sb, t_f, t_b, rf, rb)
        assert abs(dh.dh_segment_cost(tab, sf, sb) - ref) <= 1e-12 * max(1.0, ref)
    with pytest.raises(dh.DhelixError):
        dh.dh_segment_cost(tab, [9], [0])
    rf[2][3] = 0.0
    with pytest.raises(dh.DhelixError):
        dh.dh_segment_cost(dh.make_table(t_f, t_b, rf, rb), [2], [3])


def test_plan_search_matches_oracle_on_small_graphs():
    # forward chain of 4, backward chain of 3 plus two movable nodes
    deps_f = [(0, 1), (1, 2), (2, 3)]
    deps_b = [(0, 1), (1, 2), (0, 3), (1, 4)]
    for _ in range(4):
        t_f, t_b, rf, rb = rand_table(4, 5)
        tab = dh.make_table(t_f, t_b, rf, rb)
        gf, gb = dh.make_graph(4, deps_f), dh.make_graph(5, deps_b)
        for bc in (0.0, 0.07):
            plan, mk = dh.dh_plan_search(gf, gb, tab, bc, 0)
            ref, _, _, _ = P.search(list(range(4)), deps_f, list(range(5)), deps_b, t_f, t_b, rf, rb, bc)
            assert abs(mk - ref) <= 1e-12 * max(1.0, ref)
            dh.dh_plan_validate(gf, gb, plan)
            fo, bo, pairs = dh.plan_to_py(plan)
            acc = sum(P.segment_cost(fo[a:b], bo[c:d], t_f, t_b, rf, rb) + bc for a, b, c, d in pairs)
            assert abs(acc - mk) <= 1e-9


def test_plan_validate_rejects_bad_plans():
    gf, gb = dh.make_graph(3, [(0, 1), (1, 2)]), dh.make_graph(2, [(0, 1)])
    ok = dh.make_plan([0, 1, 2], [0, 1], [(0, 2, 0, 1), (2, 3, 1, 2)])
    dh.dh_plan_validate(gf, gb, ok)
    bad = [dh.make_plan([0, 2, 1], [0, 1], [(0, 3, 0, 2)]),           # dependency violated
           dh.make_plan([0, 1, 1], [0, 1], [(0, 3, 0, 2)]),           # not a permutation
           dh.make_plan([0, 1, 2], [0, 1], [(0, 2, 0, 2)]),           # forward op 2 never runs
           dh.make_plan([0, 1, 2], [0, 1], [(0, 2, 0, 1), (1, 3, 1, 2)]),  # overlap
           dh.make_plan([0, 1], [0, 1], [(0, 2, 0, 2)])]              # wrong operator count
    for p in bad:
        with pytest.raises(dh.DhelixError) as e:
            dh.dh_plan_validate(gf, gb, p)
        assert e.value.code == dh.DH_ERR_PLAN_INVALID


def test_layer_graphs_and_sequential_plan():
    L = dh.dh_layer_create(arch=0, dtype=0, batch=1, seq=16, hidden=64, n_q_heads=2, n_kv_heads=1, head_dim=16, ffn=32,
                           eps=1e-5, rope_base=1e4, n_ranks=2)
    try:
        gf, gb = dh.dh_layer_op_graph(L, 0), dh.dh_layer_op_graph(L, 1)
        assert gf.n_ops == len(dh.FWD_OPS) and gb.n_ops == len(dh.BWD_OPS)
        assert [i for i in range(gf.n_ops) if gf.is_comm[i]] == [dh.FWD_OPS.index("F_AR1"), dh.FWD_OPS.index("F_AR2")]
        assert [i for i in range(gb.n_ops) if gb.is_comm[i]] == [dh.BWD_OPS.index("B_AR3"), dh.BWD_OPS.index("B_AR4")]
        seq = dh.dh_plan_sequential(L)
        dh.dh_plan_validate(gf, gb, seq)
        fo, bo, pairs = dh.plan_to_py(seq)
        assert pairs == [(0, gf.n_ops, 0, 0), (gf.n_ops, gf.n_ops, 0, gb.n_ops)]
        # the default backward order is a topological order with each wgrad right after its dgrad
        assert dh.dh_layer_saved_bytes(L) > 0
        assert dh.dh_layer_workspace_bytes(L, dh.DH_WS_SI) == dh.dh_layer_workspace_bytes(L, dh.DH_WS_FWD) + dh.dh_layer_workspace_bytes(L, dh.DH_WS_BWD)
        # weight-gradient GEMMs are the movable operators: with uniform perfect-overlap rates the search
        # must reach max(sum_f, sum_b) on the layer's own graphs
        nf, nb = gf.n_ops, gb.n_ops
        tab = dh.make_table([1.0] * nf, [1.0] * nb, [[1.0] * nb] * nf, [[1.0] * nb] * nf)
        plan, mk = dh.dh_plan_search(gf, gb, tab, 0.0, 8)
        assert abs(mk - max(nf, nb)) < 1e-12
        dh.dh_plan_validate(gf, gb, plan)
        # the round-robin comparison plan: default orders, one operator of each strand per pair
        rr = dh.dh_plan_round_robin(gf, gb)
        dh.dh_plan_validate(gf, gb, rr)
        fo, bo, pairs = dh.plan_to_py(rr)
        assert fo == list(range(nf)) and bo == list(range(nb)) and len(pairs) == max(nf, nb)
        assert pairs[0] == (0, 1, 0, 1) and pairs[-1] == (nf, nf, nb - 1, nb)
        # weight gradients left in their default places: one order per graph
        fixed, mk_fixed = dh.dh_plan_search(gf, gb, tab, 0.0, 1)
        assert dh.plan_to_py(fixed)[1] == list(range(nb)) and mk_fixed >= mk - 1e-12
    finally:
        dh.dh_layer_destroy(L)


def test_side_operators_are_validated():
    """Only operators the backward graph marks side_ok may be set to run beside their strand."""
    from paper_2411_15871_amd import dhelix as dh
    gf = dh.make_graph(2, [(0, 1)])
    gb = dh.make_graph(3, [(0, 1)], side_ok=(2,))
    ok = dh.make_plan([0, 1], [0, 1, 2], [(0, 2, 0, 3)], side=(2,))
    dh.dh_plan_validate(gf, gb, ok)
    for bad_op in (1, 5):
        bad = dh.make_plan([0, 1], [0, 1, 2], [(0, 2, 0, 3)], side=(bad_op,))
        with pytest.raises(dh.DhelixError) as e:
            dh.dh_plan_validate(gf, gb, bad)
        assert e.value.code == dh.DH_ERR_PLAN_INVALID
    q = dh.with_side(ok, ())
    assert list(q.bwd_side) == [0] * dh.DH_MAX_OPS and list(ok.bwd_side)[2] == 1
