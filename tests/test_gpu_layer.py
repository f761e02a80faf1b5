"""GPU parity of the layer forward/backward and of the SI step against the fp64 oracle, plus the SI
invariant: interleaved execution gives bitwise the same per-strand results as sequential execution."""
import random

import numpy as np
import pytest
import torch

from oracle import layer_ref as R
from paper_2411_15871_amd import harness as H

pytestmark = pytest.mark.gpu

CASES = {
    "c1_tiny_fp32": (H.CONFIGS["c1_tiny_fp32"], 1e-5),
    "fp32_ragged": (dict(batch=2, seq=75, hidden=136, nq=4, nkv=2, d=32, ffn=200, n_ranks=3, bf16=False), 1e-5),
    "bf16_mid_ragged": (dict(batch=2, seq=330, hidden=520, nq=4, nkv=1, d=128, ffn=1000, n_ranks=4, bf16=True), 2e-2),
    "bf16_d64_mha": (dict(batch=1, seq=257, hidden=256, nq=4, nkv=4, d=64, ffn=344, n_ranks=1, bf16=True), 2e-2),
    "fp32_rope_adjacent": (dict(batch=2, seq=75, hidden=136, nq=4, nkv=2, d=32, ffn=200, n_ranks=3, bf16=False, rope_pairing=1), 1e-5),
    "bf16_rope_adjacent": (dict(batch=2, seq=330, hidden=520, nq=4, nkv=1, d=128, ffn=1000, n_ranks=4, bf16=True, rope_pairing=1), 2e-2),
    "cp_fp32_rope_adjacent": (dict(arch="llama_cp", batch=2, seq=37, hidden=136, nq=4, nkv=2, d=32, ffn=200, n_ranks=2, bf16=False,
                                   cp_ranks=3, cp_rank=1, rope_pairing=1), 1e-5),
    "gpt_fp32_gelu_erf": (dict(arch="gpt", batch=2, seq=40, hidden=136, nq=4, nkv=4, d=32, ffn=200, n_ranks=4, bf16=False, gelu_form=1), 1e-5),
    "gpt_bf16_gelu_erf": (dict(arch="gpt", batch=2, seq=264, hidden=520, nq=4, nkv=4, d=128, ffn=1000, n_ranks=4, bf16=True, gelu_form=1), 2e-2),
    "c2_llama8b_tp8": (H.CONFIGS["c2_llama8b_tp8"], 2e-2),
    "gpt_fp32_small": (dict(arch="gpt", batch=2, seq=40, hidden=136, nq=4, nkv=4, d=32, ffn=200, n_ranks=4, bf16=False), 1e-5),
    "gpt_bf16_mid": (dict(arch="gpt", batch=2, seq=264, hidden=520, nq=4, nkv=4, d=128, ffn=1000, n_ranks=4, bf16=True), 2e-2),
    "gpt_fp32_one_rank": (dict(arch="gpt", batch=1, seq=33, hidden=64, nq=2, nkv=1, d=32, ffn=72, n_ranks=1, bf16=False), 1e-5),
    "moe_fp32_small": (dict(arch="moe", batch=2, seq=75, hidden=136, nq=4, nkv=2, d=32, ffn=96, n_ranks=1, bf16=False,
                            n_experts=8, n_local=2), 1e-5),
    "moe_bf16_mid": (dict(arch="moe", batch=1, seq=600, hidden=520, nq=4, nkv=2, d=128, ffn=328, n_ranks=1, bf16=True,
                          n_experts=16, n_local=2), 2e-2),
    "moe_bf16_all_local": (dict(arch="moe", batch=1, seq=130, hidden=128, nq=2, nkv=2, d=64, ffn=64, n_ranks=1, bf16=True,
                                n_experts=4, n_local=4), 2e-2),
    "cp_fp32_small": (dict(arch="llama_cp", batch=2, seq=37, hidden=136, nq=4, nkv=2, d=32, ffn=200, n_ranks=2, bf16=False,
                           cp_ranks=3, cp_rank=1), 1e-5),
    "cp_fp32_first_rank": (dict(arch="llama_cp", batch=1, seq=50, hidden=64, nq=2, nkv=1, d=32, ffn=72, n_ranks=1, bf16=False,
                                cp_ranks=2, cp_rank=0), 1e-5),
    "cp_fp32_alone": (dict(arch="llama_cp", batch=1, seq=21, hidden=64, nq=2, nkv=2, d=16, ffn=40, n_ranks=1, bf16=False,
                           cp_ranks=1, cp_rank=0), 1e-5),
    "cp_bf16_mid": (dict(arch="llama_cp", batch=1, seq=384, hidden=520, nq=4, nkv=1, d=128, ffn=1000, n_ranks=4, bf16=True,
                         cp_ranks=4, cp_rank=2), 2e-2),
    "cp_bf16_last_d64": (dict(arch="llama_cp", batch=2, seq=128, hidden=256, nq=4, nkv=2, d=64, ffn=344, n_ranks=1, bf16=True,
                              cp_ranks=2, cp_rank=1), 2e-2),
    "c3_gpt_tp8_sp": (H.CONFIGS["c3_gpt_tp8_sp"], 2e-2),
    "c5_phimoe_ep8": (H.CONFIGS["c5_phimoe_ep8"], 2e-2),
    "c6_llama8b_tp8_cp4": (H.CONFIGS["c6_llama8b_tp8_cp4"], 2e-2),
    "c4_llama70b_tp8": (H.CONFIGS["c4_llama70b_tp8"], 2e-2),
}
GPT_NAMES = dict(Wgu="W1", Wd="W2", bfc1="bf1", bfc2="bf2")  # harness / C-struct name -> oracle name


def rel(a, b):
    return np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-30)


# A whole-tensor norm hides a wrong row or a dropped chunk, so every [rows, features] result is also checked row by row,
# and every weight gradient in blocks of 32 columns: the error norm of a row (block) against that row's (block's) own
# oracle norm, with a floor at the tensor's root-mean-square row (block) norm so that near-zero rows are measured
# against the tensor's scale.  bf16 rounding of a stored element is 2^-9 relative, of an intermediate activation a few
# times that: 3e-2 per row in bf16 mode, 2e-5 in fp32 mode.
ROW_TOL = {1e-5: 2e-5, 2e-2: 3e-2}


def row_err(got, ref):
    got, ref = np.atleast_2d(got), np.atleast_2d(ref)
    got, ref = got.reshape(-1, got.shape[-1]), ref.reshape(-1, ref.shape[-1])
    d, n = np.linalg.norm(got - ref, axis=1), np.linalg.norm(ref, axis=1)
    floor = max(float(np.sqrt(np.mean(n * n))), 1e-30)
    return float((d / np.maximum(n, floor)).max())


def colblock_err(got, ref, width=32):
    got, ref = np.atleast_2d(got), np.atleast_2d(ref)
    got, ref = got.reshape(-1, got.shape[-1]), ref.reshape(-1, ref.shape[-1])
    edges = list(range(0, got.shape[1], width))
    d = np.array([np.linalg.norm(got[:, c:c + width] - ref[:, c:c + width]) for c in edges])
    n = np.array([np.linalg.norm(ref[:, c:c + width]) for c in edges])
    floor = max(float(np.sqrt(np.mean(n * n))), 1e-30)
    return float((d / np.maximum(n, floor)).max())


class Worst:
    """Collects (name, whole-tensor error, per-row or per-block error) of a case and prints the largest."""

    def __init__(self, case, tol):
        self.case, self.tol, self.rows = case, tol, []

    def check(self, name, got, ref, blocks=False):
        g = rel(got, ref)
        r = colblock_err(got, ref) if blocks else row_err(got, ref)
        self.rows.append((name, g, r))
        assert g <= self.tol, (name, g)
        assert r <= ROW_TOL[self.tol], (name, "per block" if blocks else "per row", r)

    def report(self):
        wg, wr = max(self.rows, key=lambda t: t[1]), max(self.rows, key=lambda t: t[2])
        print("worst errors of %s: whole tensor %.3e (%s), per row/block %.3e (%s)" % (self.case, wg[1], wg[0], wr[2], wr[0]),
              flush=True)


def oracle_run(run, s):
    c = run.cfg
    cfg = R.LayerCfg(batch=c["batch"], seq=c["seq"], H=c["hidden"], nq=c["nq"], nkv=c["nkv"], d=c["d"], F=c["ffn"],
                     eps=c["eps"], rope_base=c["rope_base"], rope_pairing=c.get("rope_pairing", 0), gelu_form=c.get("gelu_form", 0))
    W = {k: v.astype(np.float64) for k, v in run.w_np.items()}
    x, dout = s.x_np.astype(np.float64), s.dout_np.astype(np.float64)
    if c["arch"] == "gpt":
        W = {GPT_NAMES.get(k, k): v for k, v in W.items()}
        pf = {"ag1": s.peers_np["ag1"], "ag2": s.peers_np["ag2"], "rs1": s.peers_np["ar1"], "rs2": s.peers_np["ar2"]}
        pb = {"ag3": s.peers_np["ag3"], "ag4": s.peers_np["ag4"], "rs3": s.peers_np["ar3"], "rs4": s.peers_np["ar4"]}
        if c["n_ranks"] == 1:
            pf = pb = None
        out, saved = R.gpt_fwd(cfg, W, x, pf)
        dx, grads, _ = R.gpt_bwd(cfg, W, saved, dout, pb)
        back = {v: k for k, v in GPT_NAMES.items()}
        grads = {"d" + back.get(k[1:], k[1:]): v for k, v in grads.items()}
        return out, dx, grads
    if c["arch"] == "moe":
        out, saved = R.moe_layer_fwd(cfg, W, x, s.logits_np.astype(np.float64), c["n_local"])
        dx, grads = R.moe_layer_bwd(cfg, W, saved, dout, c["n_local"])
        return out, dx, grads
    if c["arch"] == "llama_cp":
        out, saved = R.llama_cp_fwd(cfg, W, x, c["cp_rank"], s.peers_np)
        dx, grads, inter = R.llama_cp_bwd(cfg, W, saved, dout, c["cp_rank"], s.peers_np)
        if c["cp_rank"] > 0:  # what the rank sends back to the earlier ranks is a result too
            grads["dkv_peers"] = inter["dkv_peers"]
        return out, dx, grads
    out, saved = R.llama_fwd(cfg, W, x, s.peers_np)
    dx, grads, _ = R.llama_bwd(cfg, W, saved, dout, s.peers_np)
    return out, dx, grads


def check_grads(run, s, grads, tol, worst=None):
    worst = worst or Worst("-", tol)
    got = run.grads_np()
    assert sorted(got) == sorted(k for k in grads if k not in ("dlogits", "dkv_peers"))
    for k, v in got.items():
        if v.ndim >= 2:
            worst.check(k, v, grads[k], blocks=True)  # weight gradients: per 32-column block
        else:
            assert rel(v, grads[k]) <= tol, k         # gain / bias gradients: one row
    if "dlogits" in grads:
        worst.check("dlogits", H.to_np(s.dlogits), grads["dlogits"])
    if "dkv_peers" in grads:
        worst.check("dkv_peers", H.to_np(s.dkv_peers), grads["dkv_peers"])
    return got


@pytest.mark.parametrize("name", list(CASES))
def test_layer_fwd_bwd_matches_oracle(name):
    cfg, tol = CASES[name]
    run = H.LayerRun(cfg)
    try:
        s = run.strand(0)
        print("case", name, flush=True)
        run.fwd(s)
        run.bwd(s)
        torch.cuda.synchronize()
        out, dx, grads = oracle_run(run, s)
        worst = Worst(name, tol)
        try:
            worst.check("out", H.to_np(s.out), out)
            worst.check("dx", H.to_np(s.dx), dx)
            got = check_grads(run, s, grads, tol, worst)
        finally:
            worst.report()
        # gradient buffers accumulate: a second backward doubles them
        run.bwd(s)
        torch.cuda.synchronize()
        got2 = run.grads_np()
        for k in got:
            assert rel(got2[k], 2 * got[k]) <= 1e-6, k
    finally:
        run.close()


def snapshot(run, alpha, beta):
    torch.cuda.synchronize()
    extra = [t.clone() for t in (beta.dlogits, beta.dkv_peers) if t is not None]
    return [alpha.out.clone(), alpha.saved.clone(), beta.dx.clone()] + extra + [g.clone() for g in run.g.values()]


def random_legal_plan(dh, run, rng):
    gf, gb = dh.dh_layer_op_graph(run.layer, 0), dh.dh_layer_op_graph(run.layer, 1)

    def rand_topo(g):
        deps = [(g.dep_src[e], g.dep_dst[e]) for e in range(g.n_deps)]
        left, order = set(range(g.n_ops)), []
        while left:
            ready = [v for v in left if all(s not in left for s, d in deps if d == v)]
            v = rng.choice(sorted(ready))
            order.append(v)
            left.remove(v)
        return order
    fo, bo = rand_topo(gf), rand_topo(gb)
    pairs, fi, bj = [], 0, 0
    while fi < len(fo) or bj < len(bo):
        f2 = min(len(fo), fi + rng.randint(0, 3))
        b2 = min(len(bo), bj + rng.randint(0, 4))
        if (f2, b2) == (fi, bj):
            continue
        pairs.append((fi, f2, bj, b2))
        fi, bj = f2, b2
    side = [op for op in range(gb.n_ops) if gb.side_ok[op] and rng.random() < 0.5]  # weight gradients beside the strand
    plan = dh.make_plan(fo, bo, pairs, side)
    dh.dh_plan_validate(gf, gb, plan)
    return plan


@pytest.mark.parametrize("name", ["c1_tiny_fp32", "bf16_mid_ragged", "gpt_fp32_small", "gpt_bf16_mid", "moe_fp32_small",
                                  "moe_bf16_mid", "cp_fp32_small", "cp_bf16_mid"])
def test_si_step_bitwise_equals_sequential_and_matches_oracle(name):
    from paper_2411_15871_amd import dhelix as dh
    cfg, tol = CASES[name]
    run = H.LayerRun(cfg)
    comm, cross, comm_b = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
    try:
        alpha, beta = run.strand(0), run.strand(1)
        sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
        # beta's forward (untimed prerequisite of its backward)
        run.fwd(beta)
        torch.cuda.synchronize()
        # reference: plain sequential calls on one stream
        alpha.out.zero_(); alpha.saved.zero_(); beta.dx.zero_()
        run.zero_grads()
        run.fwd(alpha)
        run.bwd(beta)
        ref = snapshot(run, alpha, beta)
        out_o, _, _ = oracle_run(run, alpha)
        _, dx_o, grads_o = oracle_run(run, beta)
        worst = Worst(name, tol)
        try:
            worst.check("out", H.to_np(alpha.out), out_o)
            worst.check("dx", H.to_np(beta.dx), dx_o)
            check_grads(run, beta, grads_o, tol, worst)
        finally:
            worst.report()
        gf, gb = dh.dh_layer_op_graph(run.layer, 0), dh.dh_layer_op_graph(run.layer, 1)
        nf, nb = gf.n_ops, gb.n_ops
        rng = random.Random(5)
        plans = {
            "sequential": dh.dh_plan_sequential(run.layer),
            "one_pair": dh.make_plan(list(range(nf)), list(range(nb)), [(0, nf, 0, nb)]),
            "op_by_op": dh.make_plan(list(range(nf)), list(range(nb)),
                                     [(min(i, nf), min(i + 1, nf), min(i, nb), min(i + 1, nb)) for i in range(max(nf, nb))]),
            "all_beside": dh.make_plan(list(range(nf)), list(range(nb)), [(0, nf, 0, nb)],
                                       [op for op in range(nb) if gb.side_ok[op]]),
            "random_a": random_legal_plan(dh, run, rng),
            "random_b": random_legal_plan(dh, run, rng),
        }
        for pname, plan in plans.items():
            variants = [(sa, sb, comm, None), (sa, sb, None, None)]
            if cfg.get("arch") == "llama_cp":  # Send/Recv stand-ins on a cross-node stream of their own
                variants += [(sa, sb, comm, cross), (sa, sb, None, cross)]
            variants = [v + (None,) for v in variants] + [(sa, sb, comm, None, comm_b)]  # beta's collectives on a stream of their own
            for *streams, xs, cb in variants:
                print("plan", pname, "comm" if streams[2] else "nocomm", "cross" if xs else "", "beta-comm" if cb else "", flush=True)
                alpha.out.zero_(); alpha.saved.zero_(); beta.dx.zero_()
                if beta.dkv_peers is not None:
                    beta.dkv_peers.zero_()
                run.zero_grads()
                torch.cuda.synchronize()
                dh.dh_layer_set_cross_stream(run.layer, xs)
                dh.dh_layer_set_beta_comm_stream(run.layer, cb)
                run.si_step(alpha, beta, plan, *streams)
                got = snapshot(run, alpha, beta)
                dh.dh_layer_set_beta_comm_stream(run.layer, None)
                for a, b in zip(got, ref):
                    assert torch.equal(a, b), pname
        # stand-ins that launch nothing (the timing-only mode) leave the schedule runnable, and the normal mode comes back
        dh.dh_layer_set_comm_blocks(run.layer, -1)
        run.si_step(alpha, beta, plans["random_a"], sa, sb, comm)
        torch.cuda.synchronize()
        dh.dh_layer_set_comm_blocks(run.layer, 3)   # a few blocks: the result does not depend on the block count
        alpha.out.zero_(); alpha.saved.zero_(); beta.dx.zero_()
        if beta.dkv_peers is not None:
            beta.dkv_peers.zero_()
        run.zero_grads()
        run.si_step(alpha, beta, plans["random_a"], sa, sb, comm)
        for a, b in zip(snapshot(run, alpha, beta), ref):
            assert torch.equal(a, b), "after the no-op mode"
        dh.dh_layer_set_comm_blocks(run.layer, 0)
        with pytest.raises(dh.DhelixError):
            dh.dh_layer_set_comm_blocks(run.layer, -2)
        # invalid plans are rejected before anything is enqueued
        bad = dh.make_plan(list(range(nf)), list(range(nb)), [(0, nf, 0, nb - 1)])
        with pytest.raises(dh.DhelixError) as e:
            run.si_step(alpha, beta, bad, sa, sb, comm)
        assert e.value.code == dh.DH_ERR_PLAN_INVALID
        with pytest.raises(dh.DhelixError) as e:
            dh.dh_si_step(run.layer, alpha.fwd_args, beta.bwd_args, plans["one_pair"], run.ws, 1024, sa, sb, None)
        assert e.value.code == dh.DH_ERR_WORKSPACE_TOO_SMALL
    finally:
        run.close()


@pytest.mark.parametrize("name", ["c2_llama8b_tp8", "c3_gpt_tp8_sp", "c5_phimoe_ep8", "c6_llama8b_tp8_cp4"])
def test_si_step_bitwise_equals_sequential_at_full_size(name):
    """The invariant holds at any size: at the benchmark shapes, in the configurations bench.py times (stand-ins in the
    strand streams or on a communication stream, a searched plan, eager and graph replay), the interleaved step
    leaves bitwise what alpha's forward followed by beta's backward leaves."""
    from paper_2411_15871_amd import dhelix as dh
    cfg, _ = CASES[name]
    run = H.LayerRun(cfg)
    comm = torch.cuda.Stream()
    try:
        alpha, beta = run.strand(0), run.strand(1)
        sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
        run.fwd(beta)
        torch.cuda.synchronize()
        alpha.out.zero_(); alpha.saved.zero_(); beta.dx.zero_()
        run.zero_grads()
        run.fwd(alpha)
        run.bwd(beta)
        ref = snapshot(run, alpha, beta)
        # SwiGLU inside the GEMM epilogues (on by default where the shapes fit) against the separate operators: the same bits
        fused = dh.dh_layer_set_fused_activation(run.layer, True)
        print("fused activation mask", fused, flush=True)
        if name in ("c2_llama8b_tp8", "c6_llama8b_tp8_cp4"):
            assert fused == 3
        if fused:
            assert dh.dh_layer_set_fused_activation(run.layer, False) == 0
            run.fwd(beta)
            torch.cuda.synchronize()
            alpha.out.zero_(); alpha.saved.zero_(); beta.dx.zero_()
            if beta.dkv_peers is not None:
                beta.dkv_peers.zero_()
            run.zero_grads()
            run.fwd(alpha)
            run.bwd(beta)
            for a, b in zip(snapshot(run, alpha, beta), ref):
                assert torch.equal(a, b), "separate activation operators"
            assert dh.dh_layer_set_fused_activation(run.layer, True) == fused
        gf, gb = dh.dh_layer_op_graph(run.layer, 0), dh.dh_layer_op_graph(run.layer, 1)
        table = dh.dh_profile_pairs(run.layer, alpha.fwd_args, beta.bwd_args, run.ws, run.ws_bytes, sa, sb, comm, 1)
        searched, _ = dh.dh_plan_search(gf, gb, table, 5e-6, 64)
        plans = {"searched": searched, "random": random_legal_plan(dh, run, random.Random(11))}

        def reset():
            alpha.out.zero_(); alpha.saved.zero_(); beta.dx.zero_()
            if beta.dkv_peers is not None:
                beta.dkv_peers.zero_()
            run.zero_grads()
            torch.cuda.synchronize()
        for pname, plan in plans.items():
            for c in (None, comm):
                print("plan", pname, "comm" if c else "nocomm", flush=True)
                reset()
                run.si_step(alpha, beta, plan, sa, sb, c)
                for a, b in zip(snapshot(run, alpha, beta), ref):
                    assert torch.equal(a, b), pname
        if name in ("c2_llama8b_tp8", "c6_llama8b_tp8_cp4"):
            # the backward all-reduces carried by their strand's weight-gradient GEMMs (one launch each; stand-ins on a block
            # budget): sequentially and interleaved, the same bits
            dh.dh_layer_set_comm_blocks(run.layer, 64)
            assert dh.dh_layer_set_fused_collective(run.layer, 3) == 3
            try:
                reset()
                run.fwd(alpha)
                run.bwd(beta)
                for a, b in zip(snapshot(run, alpha, beta), ref):
                    assert torch.equal(a, b), "fused collectives, sequential"
                for pname, plan in plans.items():
                    for c in (None, comm):
                        print("fused collectives: plan", pname, "comm" if c else "nocomm", flush=True)
                        reset()
                        run.si_step(alpha, beta, plan, sa, sb, c)
                        for a, b in zip(snapshot(run, alpha, beta), ref):
                            assert torch.equal(a, b), pname + " (fused collectives)"
            finally:
                dh.dh_layer_set_fused_collective(run.layer, 0)
                dh.dh_layer_set_comm_blocks(run.layer, cfg.get("comm_blocks", 0))
            graph = dh.dh_si_graph_create(run.layer, alpha.fwd_args, beta.bwd_args, plan, run.ws, run.ws_bytes, sa, sb)
            try:
                for _ in range(2):
                    reset()
                    dh.dh_si_graph_launch(graph, sa)
                    for a, b in zip(snapshot(run, alpha, beta), ref):
                        assert torch.equal(a, b), pname + " (graph)"
            finally:
                dh.dh_si_graph_destroy(graph)
    finally:
        run.close()


def test_empty_micro_batch_is_a_no_op():
    run = H.LayerRun(dict(batch=0, seq=16, hidden=64, nq=2, nkv=1, d=32, ffn=64, n_ranks=2, bf16=False))
    try:
        s = run.strand(0)
        run.fwd(s)
        run.bwd(s)
        torch.cuda.synchronize()
        assert all(float(g.abs().sum()) == 0.0 for g in run.g.values())
    finally:
        run.close()


@pytest.mark.parametrize("name", ["c1_tiny_fp32", "gpt_bf16_mid", "moe_bf16_mid", "cp_bf16_mid"])
def test_captured_si_step_replays_bitwise(name):
    """The SI step recorded into a HIP graph gives, on every replay, bitwise what the eager step gives; replays are
    separated by eager work and synchronisations of the program's own."""
    from paper_2411_15871_amd import dhelix as dh
    cfg, _ = CASES[name]
    run = H.LayerRun(cfg)
    try:
        alpha, beta = run.strand(0), run.strand(1)
        sa, sb, sc = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
        run.fwd(beta)
        torch.cuda.synchronize()
        rng = random.Random(11)
        for plan in (dh.dh_plan_sequential(run.layer), random_legal_plan(dh, run, rng)):
            alpha.out.zero_(); alpha.saved.zero_(); beta.dx.zero_(); run.zero_grads()
            run.si_step(alpha, beta, plan, sa, sb, sc)
            ref = snapshot(run, alpha, beta)
            graph = dh.dh_si_graph_create(run.layer, alpha.fwd_args, beta.bwd_args, plan, run.ws, run.ws_bytes, sa, sb)
            try:
                for rep in range(3):
                    print("replay", rep, flush=True)
                    alpha.out.zero_(); alpha.saved.zero_(); beta.dx.zero_(); run.zero_grads()
                    torch.cuda.synchronize()
                    dh.dh_si_graph_launch(graph, sa)
                    got = snapshot(run, alpha, beta)
                    for a, b in zip(got, ref):
                        assert torch.equal(a, b), rep
                    run.si_step(alpha, beta, plan, sa, sb, sc)  # eager work between the replays
                    torch.cuda.synchronize()
            finally:
                dh.dh_si_graph_destroy(graph)
        with pytest.raises(dh.DhelixError):
            dh.dh_si_graph_create(run.layer, alpha.fwd_args, beta.bwd_args, plan, run.ws, run.ws_bytes, sa, sa)
    finally:
        run.close()
