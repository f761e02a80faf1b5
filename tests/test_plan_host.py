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


# ------------------------------------------------------------------ lane model and its search
def rand_case():
    """Small operator graphs with collectives, a movable operator and like operators; a random table."""
    nf, nb = 4, 6
    deps_f = [(0, 1), (1, 2), (2, 3)]                 # chain; op 1 is a collective
    deps_b = [(0, 1), (1, 2), (2, 3), (0, 4), (2, 5)]  # chain 0-1-2-3 with the collective at 1; 4 and 5 hang off (movable)
    comm_f, comm_b = {1: 1}, {1: 1}
    like_f, like_b = {1: 1, 2: 4}, {1: 1, 4: 2}
    t_f, t_b, rf, rb = rand_table(nf, nb)
    gf = dh.make_graph(nf, deps_f, comm=comm_f, like=like_f)
    gb = dh.make_graph(nb, deps_b, comm=comm_b, side_ok=(4, 5), like=like_b)
    okw = dict(deps_f=deps_f, deps_b=deps_b, comm_f=comm_f, comm_b=comm_b, like_f=like_f, like_b=like_b)
    return nf, nb, deps_f, deps_b, t_f, t_b, rf, rb, gf, gb, okw


def rand_order(n, deps):
    left, order = set(range(n)), []
    while left:
        ready = sorted(v for v in left if all(s not in left for s, d in deps if d == v))
        v = random.choice(ready)
        order.append(v)
        left.remove(v)
    return order


def test_plan_cost_matches_oracle_lane_model():
    for _ in range(30):
        nf, nb, deps_f, deps_b, t_f, t_b, rf, rb, gf, gb, okw = rand_case()
        tab = dh.make_table(t_f, t_b, rf, rb)
        fo, bo = rand_order(nf, deps_f), rand_order(nb, deps_b)
        cut_f, cut_b = random.randrange(nf + 1), random.randrange(nb + 1)
        pairs = [q for q in [(0, cut_f, 0, cut_b), (cut_f, nf, cut_b, nb)] if q[0] != q[1] or q[2] != q[3]]
        side = tuple(op for op in (4, 5) if random.random() < 0.5)
        plan = dh.make_plan(fo, bo, pairs, side)
        for lanes in [(0, 0, 0), (1, 1, 0), (1, 2, 0), (0, 2, 0)]:
            got = dh.dh_plan_cost(gf, gb, tab, plan, dh.lanes(*lanes), 0.01)
            ref = P.plan_cost_lanes(pairs, fo, bo, t_f, t_b, rf, rb, 0.01, lanes=lanes, side=side, **okw)
            assert abs(got - ref) <= 1e-11 * max(1.0, ref), (lanes, fo, bo, pairs, side)
    with pytest.raises(dh.DhelixError):
        dh.dh_plan_cost(gf, gb, tab, plan, dh.lanes(3, 0, 0), 0.0)


def test_plan_search_lanes_matches_brute_force_and_moves_the_weight_gradient():
    # brute force over all orders, side subsets and barrier placements with the oracle's lane model
    for trial in range(2):
        nf, nb, deps_f, deps_b, t_f, t_b, rf, rb, gf, gb, okw = rand_case()
        tab = dh.make_table(t_f, t_b, rf, rb)
        lanes = (1, 2, 0)
        plan, mk, info = dh.dh_plan_search_lanes(gf, gb, tab, dh.lanes(*lanes), 0.02, 0)
        assert info.truncated == 0 and info.orders_bwd_total == dh.dh_plan_count_orders(gb) == len(P.topo_orders(nb, deps_b))
        dh.dh_plan_validate(gf, gb, plan)
        fo, bo, pairs = dh.plan_to_py(plan)
        side = tuple(op for op in range(nb) if plan.bwd_side[op])
        again = P.plan_cost_lanes(pairs, fo, bo, t_f, t_b, rf, rb, 0.02, lanes=lanes, side=side, **okw)
        assert abs(again - mk) <= 1e-11 * max(1.0, mk)          # the reported time is the plan's time
        assert abs(dh.dh_plan_cost(gf, gb, tab, plan, dh.lanes(*lanes), 0.02) - mk) <= 1e-11 * max(1.0, mk)
        best = min(P.search_cuts_lanes(of, ob, t_f, t_b, rf, rb, 0.02, lanes=lanes, side=sd, **okw)[0]
                   for of in P.topo_orders(nf, deps_f) for ob in P.topo_orders(nb, deps_b)
                   for sd in [(), (4,), (5,), (4, 5)])
        assert mk >= best - 1e-11          # never better than the exhaustive optimum ...
        assert mk <= best * 1.03 + 1e-12   # ... and, on graphs this small, within the refinement's reach of it
    # a table on which the movable operator 4 (like the forward GEMM 2) pairs well only with the strand's own collective:
    # every forward operator halves it, the collective leaves it alone -> the search must issue it right after the collective
    nf, nb, deps_f, deps_b, _, _, _, _, gf, gb, okw = rand_case()
    t_f, t_b = [1.0] * nf, [1.0, 4.0, 1.0, 1.0, 4.0, 0.1]
    rf = [[1.0] * nb for _ in range(nf)]
    rb = [[1.0] * nb for _ in range(nf)]
    for i in range(nf):
        rb[i][4] = 0.25                       # operator 4 crawls beside any forward operator ...
    rb[1][4] = 1.0                            # ... except beside a collective (forward collective 1 is the like of backward 1)
    rf[2][1] = 1.0
    tab = dh.make_table(t_f, t_b, rf, rb)
    plan, mk, _ = dh.dh_plan_search_lanes(gf, gb, tab, dh.lanes(0, 2, 0), 0.0, 0)
    fo, bo, pairs = dh.plan_to_py(plan)
    assert bo.index(4) > bo.index(1) and bo.index(4) < bo.index(2)  # after the collective is issued, before its consumer
    default = dh.make_plan(list(range(nf)), list(range(nb)), [(0, nf, 0, nb)])
    assert mk < dh.dh_plan_cost(gf, gb, tab, default, dh.lanes(0, 2, 0), 0.0) - 0.5


def test_count_orders_and_full_enumeration():
    L = dh.dh_layer_create(arch=0, dtype=0, batch=1, seq=16, hidden=64, n_q_heads=2, n_kv_heads=1, head_dim=16, ffn=32,
                           eps=1e-5, rope_base=1e4, n_ranks=2)
    try:
        gf, gb = dh.dh_layer_op_graph(L, 0), dh.dh_layer_op_graph(L, 1)
        assert dh.dh_plan_count_orders(gf) == 1 and dh.dh_plan_count_orders(gb) == 5760
        assert dh.dh_plan_count_orders(gb, 100) == 100       # counting stops at the cap
        # like operators: the backward all-reduces and weight gradients name their forward counterparts
        assert gb.like_other[dh.BWD_OPS.index("B_AR3")] == dh.FWD_OPS.index("F_AR1") + 1
        assert gb.like_other[dh.BWD_OPS.index("B_FC1_WGRAD")] == dh.FWD_OPS.index("F_FC1") + 1
        assert gb.like_other[dh.BWD_OPS.index("B_ATTN")] == 0
        # a table where the down-projection weight gradient pairs well only late (beside the last forward operators):
        # the search must move it there -- with the enumeration cut to the first orders it could not
        nf, nb = gf.n_ops, gb.n_ops
        w = dh.BWD_OPS.index("B_FC2_WGRAD")
        rf = [[0.5] * nb for _ in range(nf)]
        rb = [[0.5] * nb for _ in range(nf)]
        for i in (nf - 2, nf - 1):
            rf[i][w] = rb[i][w] = 1.0
        tab = dh.make_table([1.0] * nf, [1.0] * nb, rf, rb)
        plan, mk = dh.dh_plan_search(gf, gb, tab, 0.3, 0)   # (barriers cost something: aligning by barriers alone loses)
        bo = dh.plan_to_py(plan)[1]
        assert bo.index(w) >= 8, bo
    finally:
        dh.dh_layer_destroy(L)


ARCH_CFGS = {
    "llama": dict(arch=0, n_ranks=2),
    "gpt": dict(arch=1, n_ranks=2, n_kv_heads=2),
    "moe": dict(arch=2, n_ranks=1, n_experts=4, n_local_experts=2),
    "llama_cp": dict(arch=3, n_ranks=2, cp_ranks=2, cp_rank=1),
}


@pytest.mark.parametrize("name", list(ARCH_CFGS))
def test_lane_search_on_every_architecture_graph(name):
    """dh_plan_search_lanes on the layer's own operator graphs with random tables (some operators at the profiler's floor
    time, some pairs undisturbed), under every placement of the stand-ins and a small order cap: the plan is valid, its
    bwd_side marks only side_ok operators, dh_plan_cost reproduces the makespan the search reports, and no plan is worse
    than the sequential or the default free-running one costed the same way."""
    cfg = dict(dtype=0, batch=1, seq=64, hidden=64, n_q_heads=2, n_kv_heads=1, head_dim=32, ffn=64, eps=1e-5, rope_base=1e4)
    cfg.update(ARCH_CFGS[name])
    L = dh.dh_layer_create(**cfg)
    rng = random.Random(5)
    try:
        gf, gb = dh.dh_layer_op_graph(L, 0), dh.dh_layer_op_graph(L, 1)
        nf, nb = gf.n_ops, gb.n_ops
        assert dh.dh_plan_count_orders(gb, 10 ** 6) >= 1
        seq = dh.dh_plan_sequential(L)
        free = dh.make_plan(list(seq.fwd_order[:nf]), list(seq.bwd_order[:nb]), [(0, nf, 0, nb)])
        for trial in range(3):
            t_f = [1e-7 if rng.random() < 0.1 else rng.uniform(1e-6, 2e-4) for _ in range(nf)]
            t_b = [1e-7 if rng.random() < 0.1 else rng.uniform(1e-6, 2e-4) for _ in range(nb)]
            rf = [[1.0 if rng.random() < 0.2 else rng.uniform(0.02, 1.0) for _ in range(nb)] for _ in range(nf)]
            rb = [[1.0 if rng.random() < 0.2 else rng.uniform(0.02, 1.0) for _ in range(nb)] for _ in range(nf)]
            tab = dh.make_table(t_f, t_b, rf, rb)
            bc = 5e-6 if trial & 1 else 0.0
            for lanes in [(0, 0, 0), (1, 1, 0), (1, 2, 0), (1, 1, 1), (1, 2, 1)]:
                ln = dh.lanes(*lanes)
                plan, mk, info = dh.dh_plan_search_lanes(gf, gb, tab, ln, bc, 40)
                dh.dh_plan_validate(gf, gb, plan)
                assert all(gb.side_ok[o] for o in range(nb) if plan.bwd_side[o])
                assert info.orders_bwd_tried <= 40 and info.orders_fwd_tried <= 40
                again = dh.dh_plan_cost(gf, gb, tab, plan, ln, bc)
                assert abs(again - mk) <= 1e-9 * mk
                assert mk <= dh.dh_plan_cost(gf, gb, tab, seq, ln, bc) * (1 + 1e-9)
                assert mk <= dh.dh_plan_cost(gf, gb, tab, free, ln, bc) * (1 + 1e-9)
    finally:
        dh.dh_layer_destroy(L)
