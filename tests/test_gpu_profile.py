"""The pair profiler's table (Sec. 3.2, Eq. 1) checked entry by entry: what dh_profile_pairs returns is what the planner
consumes, so every derived field must follow from the measured ones by the oracle's formulas (Eq. 1 for the overlap
factor, the two-queue model of Sec. 4.2's P for the pair time), and the measured ones must be sane."""
import math

import pytest
import torch

from oracle import plan_ref as P
from paper_2411_15871_amd import harness as H

pytestmark = pytest.mark.gpu

CASES = {
    "llama_bf16_mid": dict(arch="llama", batch=1, seq=1024, hidden=1024, nq=4, nkv=1, d=128, ffn=1408, n_ranks=4, bf16=True),
    "gpt_bf16_mid": dict(arch="gpt", batch=2, seq=512, hidden=1024, nq=4, nkv=4, d=128, ffn=2048, n_ranks=4, bf16=True),
    # shapes at which SwiGLU runs inside the neighbouring GEMMs' epilogues: F_ACT and B_ACT launch nothing
    "llama_bf16_fused_act": dict(arch="llama", batch=2, seq=2048, hidden=512, nq=4, nkv=1, d=128, ffn=1024, n_ranks=2, bf16=True),
    # rank 0 of a context-parallel group sends nothing back: B_CP_SEND launches no kernel and measures ~0
    "cp_first_rank": dict(arch="llama_cp", batch=1, seq=256, hidden=512, nq=4, nkv=1, d=128, ffn=512, n_ranks=2, bf16=True,
                          cp_ranks=2, cp_rank=0),
}


@pytest.mark.parametrize("name", list(CASES))
def test_profile_table_entries(name):
    from paper_2411_15871_amd import dhelix as dh
    run = H.LayerRun(CASES[name])
    try:
        alpha, beta = run.strand(0), run.strand(1)
        sa, sb, comm = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
        run.fwd(alpha); run.fwd(beta); run.bwd(beta)
        torch.cuda.synchronize()
        print("case", name, "profiling", flush=True)
        t = dh.dh_profile_pairs(run.layer, alpha.fwd_args, beta.bwd_args, run.ws, run.ws_bytes, sa, sb, comm, 3)
        gf, gb = dh.dh_layer_op_graph(run.layer, 0), dh.dh_layer_op_graph(run.layer, 1)
        nf, nb = t.n_fwd, t.n_bwd
        assert (nf, nb) == (gf.n_ops, gb.n_ops)
        t_f, t_b = [t.t_fwd[i] for i in range(nf)], [t.t_bwd[j] for j in range(nb)]
        rf = [[t.rate_fwd[i][j] for j in range(nb)] for i in range(nf)]
        rb = [[t.rate_bwd[i][j] for j in range(nb)] for i in range(nf)]
        # measured fields: positive, finite solo times below a second; rates inside the clamp
        for v in t_f + t_b:
            assert math.isfinite(v) and 1e-7 <= v < 1.0
        names_b = dh.op_names(H.ARCH[run.cfg["arch"]], 1)
        if name == "cp_first_rank":
            assert t_b[names_b.index("B_CP_SEND")] <= 5e-6  # an operator that launches nothing sits at (about) the floor
        if name == "llama_bf16_fused_act":
            names_f = dh.op_names(H.ARCH[run.cfg["arch"]], 0)
            c = run.cfg
            assert dh.dh_gemm_swiglu_fwd_fits(c["batch"] * c["seq"], c["ffn"], c["hidden"])
            assert dh.dh_gemm_swiglu_bwd_fits(c["batch"] * c["seq"], c["ffn"], c["hidden"])
            assert t_f[names_f.index("F_ACT")] <= 5e-6 and t_b[names_b.index("B_ACT")] <= 5e-6
        for i in range(nf):
            for j in range(nb):
                assert 0.02 <= rf[i][j] <= 1.0 and 0.02 <= rb[i][j] <= 1.0
                # derived fields: the pair time under the two-queue model and Eq. 1, from the table's own numbers
                p = P.segment_cost([i], [j], t_f, t_b, rf, rb)
                assert abs(t.p_pair[i][j] - p) <= 1e-12 * max(1.0, p)
                assert abs(t.oef[i][j] - P.oef(t_f[i], t_b[j], p)) <= 1e-9
                assert math.isfinite(t.oef[i][j])
                # a co-run is never shorter than the longer operator (rates <= 1); contention can make it longer than
                # one operator after the other, but the clamp of the rates bounds it
                assert max(t_f[i], t_b[j]) * (1 - 1e-9) <= t.p_pair[i][j] <= (t_f[i] + t_b[j]) / 0.02
                if gf.is_comm[i] == 1 and gb.is_comm[j] == 1:  # two collectives share the one communication stream
                    # they serialise: nothing is hidden but what the lower clamp of the rates (0.02) lets through
                    lo, hi = min(t_f[i], t_b[j]), max(t_f[i], t_b[j])
                    assert abs(t.p_pair[i][j] - (t_f[i] + t_b[j])) <= 0.0201 * hi and abs(t.oef[i][j]) <= 0.0201 * hi / lo
        # the solo times against event timing of the test's own: the strand run operator by operator takes the sum
        run.fwd(alpha); run.fwd(beta); run.bwd(beta)   # the profiler ran operators in place: restore valid inputs
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        best_f = best_b = float("inf")
        for _ in range(5):
            with torch.cuda.stream(sa):
                e0.record(sa); run.fwd(alpha, sa); e1.record(sa)
            torch.cuda.synchronize()
            best_f = min(best_f, e0.elapsed_time(e1) * 1e-3)
            with torch.cuda.stream(sa):
                e0.record(sa); run.bwd(beta, sa); e1.record(sa)
            torch.cuda.synchronize()
            best_b = min(best_b, e0.elapsed_time(e1) * 1e-3)
        print("solo us, forward:", [round(v * 1e6, 1) for v in t_f], "backward:", [round(v * 1e6, 1) for v in t_b], flush=True)
        print("forward: sum of solo %.1f us, strand %.1f us; backward: %.1f us, %.1f us" %
              (sum(t_f) * 1e6, best_f * 1e6, sum(t_b) * 1e6, best_b * 1e6), flush=True)
        # launch gaps make the strand a little longer than the sum of back-to-back repetitions, clock ramps either way
        if name != "cp_first_rank":  # (that case's operators are shorter than a launch: the strand measures launch rate)
            assert 0.5 * best_f <= sum(t_f) <= 2.0 * best_f
            assert 0.5 * best_b <= sum(t_b) <= 2.0 * best_b
    finally:
        run.close()
