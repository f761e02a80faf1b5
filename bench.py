#!/usr/bin/env python3
"""Benchmark of one Strand-Interleaving layer step (alpha forward || beta backward) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c2_llama8b_tp8]

A step = one dh_si_step over one micro-batch per strand with all inputs resident in HBM.  Prints one
JSON line: model TFLOP/s of the step (2MNK per GEMM, causal attention at half dense, backward =
2x forward), SI speedup over sequential alpha-then-beta through the same executor, the fraction of
collective stand-in time hidden, the roofline of the dominant kernel and the CPU oracle baseline.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

BF16_MFMA_PEAK_TFLOPS = 2500.0  # MI355X dense bf16
# HBM bytes per launch of the dominant GEMM from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs (scaled by a copy kernel of
# known size: `bench.py --traffic-probe`); the summary with the commands is profiles/gemm_gateup_c2_hbm_traffic.txt.
# Re-measure when the GEMM changes.
HBM_TRAFFIC_BYTES = {"c2_llama8b_tp8": (176.3 + 28.3) * 2 ** 20}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def time_steps(fn, steps, warmup, torch):
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps


def cpu_baseline(cfg, flops):
    """Times the fp64 oracle (as it stands) on one strand's full forward+backward at the same shapes."""
    import numpy as np
    from oracle import layer_ref as R
    from paper_2411_15871_amd import inputs as gen
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count()
    arch, bf = cfg["arch"], cfg["bf16"]
    T, H = cfg["batch"] * cfg["seq"], cfg["hidden"]
    rows = T // cfg["n_ranks"] if arch == "gpt" else T
    n_qkv = (cfg["nq"] + 2 * cfg["nkv"]) * cfg["d"]
    ocfg = R.LayerCfg(batch=cfg["batch"], seq=cfg["seq"], H=H, nq=cfg["nq"], nkv=cfg["nkv"], d=cfg["d"], F=cfg["ffn"])
    x = gen.strand_input(0, rows, H, bf).astype(np.float64)
    dout = gen.strand_upstream_grad(0, rows, H, bf).astype(np.float64)
    f64 = lambda w: {k: v.astype(np.float64) for k, v in w.items()}
    if arch == "gpt":
        names = dict(Wgu="W1", Wd="W2", bfc1="bf1", bfc2="bf2")
        W = {names.get(k, k): v for k, v in f64(gen.gpt_weights(H, n_qkv, cfg["nq"] * cfg["d"], cfg["ffn"], bf)).items()}
        peers = lambda n: {k: np.zeros((cfg["n_ranks"] - 1, rows, H)) for k in n}

        def once():
            _, saved = R.gpt_fwd(ocfg, W, x, peers(("ag1", "ag2", "rs1", "rs2")))
            R.gpt_bwd(ocfg, W, saved, dout, peers(("ag3", "ag4", "rs3", "rs4")))
    elif arch == "moe":
        W = f64(gen.moe_weights(H, n_qkv, cfg["nq"] * cfg["d"], cfg["ffn"], cfg["n_local"], bf))
        logits = gen.router_logits(T, cfg["n_experts"]).astype(np.float64)

        def once():
            _, saved = R.moe_layer_fwd(ocfg, W, x, logits, cfg["n_local"])
            R.moe_layer_bwd(ocfg, W, saved, dout, cfg["n_local"])
    elif arch == "llama_cp":
        W = f64(gen.llama_weights(H, n_qkv, cfg["nq"] * cfg["d"], cfg["ffn"], bf))
        Wkv = 2 * cfg["nkv"] * cfg["d"]
        kv = gen.peer_partials(170, cfg["cp_ranks"] - 1, T, Wkv, bf, 1.0)
        dkv = gen.peer_partials(270, cfg["cp_ranks"] - 1, T, Wkv, bf, 1e-2)

        def once():
            _, saved = R.llama_cp_fwd(ocfg, W, x, cfg["cp_rank"], {"kv": kv})
            R.llama_cp_bwd(ocfg, W, saved, dout, cfg["cp_rank"], {"dkv": dkv})
    else:
        W = f64(gen.llama_weights(H, n_qkv, cfg["nq"] * cfg["d"], cfg["ffn"], bf))

        def once():
            _, saved = R.llama_fwd(ocfg, W, x)
            R.llama_bwd(ocfg, W, saved, dout)
    t0 = time.perf_counter()
    reps = 0
    while reps < 1 or (time.perf_counter() - t0 < 10.0 and reps < 20):
        once()
        reps += 1
    dt = (time.perf_counter() - t0) / reps
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": int(threads), "kind": "oracle",
            "sample": "%d x one full layer forward+backward of one strand at the benchmark shapes (peer partials absent or zero), "
                      "%.1f s each" % (reps, dt)}


def write_pair_table(path, args, table, fnames, bnames, t_f, t_b):
    """The profiler's output as text: solo times, then for every forward/backward operator pair the rate each keeps
    while the other runs (percent of its solo rate) and the overlap effectiveness factor of Eq. 1,
    (t_i + t_j - P_ij) / min(t_i, t_j): 1 = the shorter operator is hidden completely, 0 = nothing gained."""
    nf, nb = len(t_f), len(t_b)
    with open(path, "w") as f:
        f.write("operator-pair table, workload %s, %d repetitions per measurement\n" % (args.workload, args.profile_reps))
        f.write("solo us, forward : " + "  ".join("%s %.1f" % (fnames[i], t_f[i] * 1e6) for i in range(nf)) + "\n")
        f.write("solo us, backward: " + "  ".join("%s %.1f" % (bnames[j], t_b[j] * 1e6) for j in range(nb)) + "\n\n")
        f.write("cell: rate kept while co-running forward%/backward%, then OEF (Eq. 1); rows: forward operator of strand alpha, "
                "columns: backward operator of strand beta\n")
        f.write("%-8s" % "" + "".join("%-14s" % n[2:] for n in bnames[:nb]) + "\n")
        for i in range(nf):
            cells = ["%3.0f/%-3.0f %4.2f" % (100 * table.rate_fwd[i][j], 100 * table.rate_bwd[i][j], table.oef[i][j]) for j in range(nb)]
            f.write("%-8s" % fnames[i][2:] + "".join("%-14s" % c for c in cells) + "\n")


def stack_bench(args, torch, dh, H):
    """L stacked layers (Llama shapes only): a steady-state phase = forward sweep of one micro-batch co-run with the
    backward sweep of the previous one; reports its rate and the activation arena against two unshared sets."""
    from paper_2411_15871_amd import inputs as gen
    c = H.CONFIGS[args.workload]
    if c["arch"] != "llama":
        sys.exit("bench.py --layers: only the Llama workloads can be stacked")
    L, bf = args.layers, c["bf16"]
    T, Hd = c["batch"] * c["seq"], c["hidden"]
    n_qkv = (c["nq"] + 2 * c["nkv"]) * c["d"]
    stack = dh.dh_stack_create(L, arch=dh.DH_ARCH_LLAMA, dtype=dh.DH_BF16 if bf else dh.DH_F32, batch=c["batch"], seq=c["seq"],
                               hidden=Hd, n_q_heads=c["nq"], n_kv_heads=c["nkv"], head_dim=c["d"], ffn=c["ffn"], eps=1e-5,
                               rope_base=10000.0, n_ranks=c["n_ranks"], comm_blocks=args.comm_blocks, n_experts=0, n_local_experts=0)
    keep = []
    for l in range(L):
        w_np = gen.llama_weights(Hd, n_qkv, c["nq"] * c["d"], c["ffn"], bf, seed=gen.SEED_WEIGHTS + 100 * l)
        w = {k: H.to_dev(v, bf) for k, v in w_np.items()}
        g = {"d" + k: torch.zeros(v.shape, dtype=torch.float32, device="cuda") for k, v in w_np.items()}
        dh.dh_layer_bind_weights(dh.dh_stack_layer(stack, l), **w)
        dh.dh_layer_bind_wgrads(dh.dh_stack_layer(stack, l), **g)
        keep.append((w, g))
    n_peers = c["n_ranks"] - 1
    peers = [H.to_dev(gen.peer_partials(300 + 10 * i, n_peers, T, Hd, bf), bf) if n_peers else None for i in range(4)]
    xs = [H.to_dev(gen.strand_input(m, T, Hd, bf), bf) for m in range(2)]
    douts = [H.to_dev(gen.strand_upstream_grad(m, T, Hd, bf), bf) for m in range(2)]
    outs = [torch.empty_like(xs[0]) for _ in range(2)]
    dxs = [torch.empty_like(xs[0]) for _ in range(2)]
    arena_bytes, ws_bytes = dh.dh_stack_arena_bytes(stack), dh.dh_stack_workspace_bytes(stack)
    arena = torch.empty(arena_bytes, dtype=torch.uint8, device="cuda")
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    sa, sb, sc = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
    layer0 = dh.dh_stack_layer(stack, 0)
    gf, gb = dh.dh_layer_op_graph(layer0, 0), dh.dh_layer_op_graph(layer0, 1)
    plan = dh.make_plan(list(range(gf.n_ops)), list(range(gb.n_ops)), [(0, gf.n_ops, 0, gb.n_ops)])
    fwd = lambda m: (xs[m], outs[m], peers[0], peers[1])
    bwd = lambda m: (douts[m], dxs[m], peers[2], peers[3])
    comm = {"s": sc}
    phase = lambda a, b, p: dh.dh_stack_phase(stack, a, b, p, arena, arena_bytes, ws, ws_bytes, sa, sb, comm["s"])
    phase(fwd(0), None, None)
    state = {"m": 1}

    def steady():
        m = state["m"]
        phase(fwd(m & 1), bwd((m - 1) & 1), plan)
        state["m"] = m + 1
    # stand-ins on the shared communication stream or in their strand's streams: keep the faster (an even number of
    # probe phases, so that the micro-batch parity carries over)
    probe = 2 * max(2, args.steps // 10)
    t_shared = time_steps(steady, probe, 2, torch)
    comm["s"] = None
    t_own = time_steps(steady, probe, 2, torch)
    log("stack phase: stand-ins on the communication stream %.1f us, in their strand's streams %.1f us" % (t_shared * 1e6, t_own * 1e6))
    if t_shared < t_own:
        comm["s"] = sc
    t_phase = time_steps(steady, args.steps, args.warmup, torch)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    phase(None, bwd((state["m"] - 1) & 1), None)   # cool-down
    torch.cuda.synchronize()
    # sequential reference: the same two sweeps one after the other
    def seq():
        phase(fwd(0), None, None)
        phase(None, bwd(0), None)
    t_seq = time_steps(seq, max(3, args.steps // 3), 2, torch)
    flops = L * H.model_flops(c)
    value = flops / t_phase / 1e12
    out = {"metric": "SI phase over %d stacked layers, fwd sweep || bwd sweep, TFLOP/s per MI355X" % L, "value": value, "unit": "TFLOP/s",
           "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": t_phase * 1e3, "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "bf16" if bf else "f32", "data": "synthetic",
           "config": {"workload": args.workload, "layers": L, "tokens_per_strand": T,
                      "standins_on": "communication stream" if comm["s"] is not None else "strand streams"},
           "pct_bf16_peak": 100.0 * value / BF16_MFMA_PEAK_TFLOPS, "speedup_vs_sequential": t_seq / t_phase,
           "ms_sequential": t_seq * 1e3, "arena_bytes": arena_bytes, "unshared_bytes": dh.dh_stack_unshared_bytes(stack),
           "single_strand_bytes": dh.dh_stack_unshared_bytes(stack) // 2}
    dh.dh_stack_destroy(stack)
    print(json.dumps(out), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="c2_llama8b_tp8")
    ap.add_argument("--comm-blocks", type=int, default=0, help="thread blocks per collective stand-in (0 = cover payload)")
    ap.add_argument("--cross-blocks", type=int, default=0, help="thread blocks per cross-node Send/Recv stand-in (0 = 8, about one 400 Gb/s port)")
    ap.add_argument("--profile-reps", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--layers", type=int, default=0, help="stack this many layers: alpha sweeps forward while beta sweeps backward")
    ap.add_argument("--traffic-probe", action="store_true", help="only launch a calibration copy and the dominant GEMM (for rocprofv3 --pmc)")
    ap.add_argument("--sequential-probe", action="store_true",
                    help="only run alpha's forward then beta's backward, one kernel at a time, --steps times (for rocprofv3: every kernel's solo "
                         "duration and counters at the workload's shapes)")
    ap.add_argument("--pair-table", default=None, metavar="PATH",
                    help="also write the measured operator-pair table (solo times, co-run rates, Eq. 1 overlap factors) to this text file")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (the SI step is a per-GPU schedule); use --gpus 1")

    import torch
    from paper_2411_15871_amd import dhelix as dh
    from paper_2411_15871_amd import harness as H

    if args.traffic_probe:
        # For `rocprofv3 --pmc FETCH_SIZE` / `--pmc WRITE_SIZE` runs: a plain copy of known size (the stand-in kernel with
        # one partial: reads 256 MiB, writes 256 MiB) calibrates the counters, then the dominant GEMM is launched alone.
        c = H.CONFIGS[args.workload]
        T, Hd = c["batch"] * c["seq"], c["hidden"]
        T = T if c["arch"] != "moe" else 2 * T // c["n_local"]
        F2 = c["ffn"] if c["arch"] == "gpt" else 2 * c["ffn"]
        src = torch.empty(128 << 20, dtype=torch.bfloat16, device="cuda").normal_()
        dst = torch.empty_like(src)
        a_mat = torch.empty(T, Hd, dtype=torch.bfloat16, device="cuda").normal_()
        b_mat = torch.empty(Hd, F2, dtype=torch.bfloat16, device="cuda").normal_(0, 0.02)
        c_mat = torch.empty(T, F2, dtype=torch.bfloat16, device="cuda")
        wsb = dh.dh_gemm_workspace_bytes(dh.DH_BF16, 0, 0, T, F2, Hd)
        gws = torch.empty(max(wsb, 256), dtype=torch.uint8, device="cuda")
        torch.cuda.synchronize()
        for _ in range(3):
            dh.dh_comm_standin(dh.DH_COMM_ALLREDUCE, [src], dst, src.numel(), dh.DH_BF16)
        for _ in range(3):
            dh.dh_gemm(dh.DH_BF16, 0, 0, T, F2, Hd, a_mat, b_mat, c_mat, False, gws, wsb)
        torch.cuda.synchronize()
        print("traffic probe: 3 x copy of %d KiB, 3 x GEMM %dx%dx%d" % (src.numel() * 2 // 1024, T, F2, Hd))
        return

    if args.layers > 0:
        return stack_bench(args, torch, dh, H)

    cfg = dict(H.CONFIGS[args.workload])
    cfg["comm_blocks"] = args.comm_blocks
    cfg["cross_blocks"] = args.cross_blocks
    flops = H.model_flops(cfg)
    run = H.LayerRun(cfg)
    alpha, beta = run.strand(0), run.strand(1)
    run.fwd(beta)   # beta's forward produced its saved activations earlier (untimed)
    run.fwd(alpha)
    run.bwd(beta)
    torch.cuda.synchronize()
    if args.sequential_probe:
        # a plain copy of known size first (the stand-in kernel with one partial: 256 MiB read, 256 MiB written): the
        # scale of the HBM byte counters in the same run
        src = torch.empty(128 << 20, dtype=torch.bfloat16, device="cuda").normal_()
        dst = torch.empty_like(src)
        dh.dh_comm_standin(dh.DH_COMM_ALLREDUCE, [src], dst, src.numel(), dh.DH_BF16)
        for _ in range(args.steps):
            run.fwd(alpha)
            run.bwd(beta)
        torch.cuda.synchronize()
        print("sequential probe: %d x (forward of one strand, backward of the other), workload %s" % (args.steps, args.workload))
        run.close()
        return
    sa, sb, sc = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
    sx = None
    if cfg["arch"] == "llama_cp":  # Sec. 5: cross-node transfers get a stream of their own
        sx = torch.cuda.Stream()
        dh.dh_layer_set_cross_stream(run.layer, sx)

    # offline part of the method: pairwise profiling and plan search (Sec. 3.2, 4.2)
    t0 = time.perf_counter()
    table = dh.dh_profile_pairs(run.layer, alpha.fwd_args, beta.bwd_args, run.ws, run.ws_bytes, sa, sb, sc, args.profile_reps)
    t_prof = time.perf_counter() - t0
    gf, gb = dh.dh_layer_op_graph(run.layer, 0), dh.dh_layer_op_graph(run.layer, 1)
    t0 = time.perf_counter()
    plan, predicted = dh.dh_plan_search(gf, gb, table, 5e-6, 256)
    t_search = time.perf_counter() - t0
    fo, bo, pairs = dh.plan_to_py(plan)
    t_f = [table.t_fwd[i] for i in range(gf.n_ops)]
    t_b = [table.t_bwd[j] for j in range(gb.n_ops)]
    log("profile %.2fs, search %.2fs, predicted makespan %.1f us, sum solo %.1f us" % (t_prof, t_search, predicted * 1e6, (sum(t_f) + sum(t_b)) * 1e6))
    fnames, bnames = dh.op_names(H.ARCH[cfg["arch"]], 0), dh.op_names(H.ARCH[cfg["arch"]], 1)
    log("fwd solo us:", {fnames[i]: round(t_f[i] * 1e6, 1) for i in range(gf.n_ops)})
    log("bwd solo us:", {bnames[j]: round(t_b[j] * 1e6, 1) for j in range(gb.n_ops)})
    log("plan:", [([fnames[o] for o in fo[a:b]], [bnames[o] for o in bo[c:d]]) for a, b, c, d in pairs])
    if args.pair_table:
        write_pair_table(args.pair_table, args, table, fnames, bnames, t_f, t_b)

    nf, nb = gf.n_ops, gb.n_ops
    seq_plan = dh.dh_plan_sequential(run.layer)
    free_plan = dh.make_plan(list(seq_plan.fwd_order[:nf]), list(seq_plan.bwd_order[:nb]), [(0, nf, 0, nb)])
    # Last offline step: the cost model ranks plans, measurement picks among its best few.  Candidates: the searched
    # plan at several barrier prices (dearer barriers -> fewer, longer segment pairs), each also with its operator orders
    # kept but all barriers dropped, and the default orders without barriers.
    cands, seen = [("default order, one pair", free_plan)], {dh.plan_to_py(free_plan).__repr__()}
    for bc in (0.0, 3e-7, 1e-6, 2.5e-6, 5e-6, 1.5e-5, 3e-5, 6e-5, 2e-4):
        p_bc, _ = dh.dh_plan_search(gf, gb, table, bc, 512)
        fo_c, bo_c, pairs_c = dh.plan_to_py(p_bc)
        for name, q in (("searched, barrier %.1e, %d pairs" % (bc, len(pairs_c)), p_bc),
                        ("searched orders (barrier %.1e), one pair" % bc, dh.make_plan(fo_c, bo_c, [(0, nf, 0, nb)]))):
            key = dh.plan_to_py(q).__repr__()
            if key not in seen:  # different barrier prices often give the same plan
                seen.add(key)
                cands.append((name, q))
    # Transfers that wait for nothing (the context-parallel key/value exchange) can start the step: the same candidates
    # again with such operators moved to the front of the forward order.
    free_comm = [op for op in range(nf) if gf.is_comm[op] and not any(gf.dep_dst[e] == op for e in range(gf.n_deps))]
    if free_comm:
        for name, q in list(cands):
            fo_c, bo_c, pairs_c = dh.plan_to_py(q)
            if len(pairs_c) != 1:
                continue  # segment boundaries are positions in the order: only hoist in single-pair plans
            hoisted = free_comm + [op for op in fo_c if op not in free_comm]
            cands.append((name + ", exchange first", dh.make_plan(hoisted, bo_c, pairs_c)))
    # Where the collective stand-ins go is part of the schedule too: on one shared communication stream (their order
    # there is the host's issue order, so a strand's collective can wait behind the other strand's) or each in its own
    # strand's stream.
    probe_steps = max(5, args.steps // 5)
    sc_stream = sc
    timed = [(time_steps(lambda p=p, c=c: run.si_step(alpha, beta, p, sa, sb, c), probe_steps, 2, torch), name, p, c)
             for name, p in cands for c in (sc_stream, None)]
    for t, name, _, c in timed:
        log("  candidate %-48s stand-ins on %-20s %.1f us" % (name, "the comm stream" if c is not None else "strand streams", t * 1e6))
    t_best, best_name, best_plan, sc = min(timed, key=lambda x: x[0])
    comm_placement = "communication stream" if sc is not None else "strand streams"
    # Weight-gradient operators may run beside the backward strand (on the forward strand's stream, which is the
    # shorter one): try a few subsets on the chosen plan.
    side_ok = sorted((op for op in range(nb) if gb.side_ok[op]), key=lambda o: -t_b[o])
    in_strand_plan, side_ops = best_plan, []
    for label, ops in (("all", side_ok), ("two largest", side_ok[:2]), ("largest", side_ok[:1]), ("all but the largest", side_ok[1:])):
        if not ops:
            continue
        q = dh.with_side(in_strand_plan, ops)
        t = time_steps(lambda q=q: run.si_step(alpha, beta, q, sa, sb, sc), probe_steps, 2, torch)
        log("  weight gradients beside the strand (%s: %s): %.1f us" % (label, [bnames[o] for o in ops], t * 1e6))
        if t < t_best:
            t_best, best_plan, side_ops = t, q, ops
    if side_ops:
        best_name += ", beside the strand: " + "+".join(bnames[o] for o in side_ops)
    fo, bo, pairs = dh.plan_to_py(best_plan)
    log("chosen plan:", best_name, [([fnames[o] for o in fo[a:b]], [bnames[o] for o in bo[c:d]]) for a, b, c, d in pairs])
    t_seq = time_steps(lambda: run.si_step(alpha, beta, seq_plan, sa, sb, sc), args.steps, args.warmup, torch)
    t_free = time_steps(lambda: run.si_step(alpha, beta, free_plan, sa, sb, sc), args.steps, args.warmup, torch)
    t_si = time_steps(lambda: run.si_step(alpha, beta, best_plan, sa, sb, sc), args.steps, args.warmup, torch)
    t_in_strand = time_steps(lambda: run.si_step(alpha, beta, in_strand_plan, sa, sb, sc), probe_steps, 2, torch) if side_ops else t_si
    # ablations of Sec. 6.1 / 6.4 through the same executor: round-robin interleaving ("Wavelet+"), and the searched plan
    # with the weight-gradient operators left in their default places
    rr_plan = dh.dh_plan_round_robin(gf, gb)
    fixed_plan, _ = dh.dh_plan_search(gf, gb, table, 5e-6, 1)
    probe = max(5, args.steps // 3)
    t_rr = time_steps(lambda: run.si_step(alpha, beta, rr_plan, sa, sb, sc), probe, 2, torch)
    t_fixed = time_steps(lambda: run.si_step(alpha, beta, fixed_plan, sa, sb, sc), probe, 2, torch)
    log("ablations: round-robin %.1f us, weight gradients fixed %.1f us" % (t_rr * 1e6, t_fixed * 1e6))
    t_shared = None
    if sx is not None:  # ablation of Sec. 6.4 ("Communication and Communication Overlap"): both kinds of transfer on one stream
        dh.dh_layer_set_cross_stream(run.layer, None)
        t_shared = time_steps(lambda: run.si_step(alpha, beta, best_plan, sa, sb, sc_stream), probe, 2, torch)
        dh.dh_layer_set_cross_stream(run.layer, sx)
        t_cross = sum(t_f[i] for i in range(nf) if gf.is_comm[i] == 2) + sum(t_b[j] for j in range(nb) if gb.is_comm[j] == 2)
        log("cross-node stand-ins solo %.1f us; SI step with them on the collectives' stream %.1f us" % (t_cross * 1e6, t_shared * 1e6))
    # the same step replayed from a HIP graph (one launch per step instead of one per operator)
    graph = dh.dh_si_graph_create(run.layer, alpha.fwd_args, beta.bwd_args, best_plan, run.ws, run.ws_bytes, sa, sb)
    t_graph = time_steps(lambda: dh.dh_si_graph_launch(graph, sa), args.steps, args.warmup, torch)
    t_comm = sum(t_f[i] for i in range(nf) if gf.is_comm[i]) + sum(t_b[j] for j in range(nb) if gb.is_comm[j])
    log("T_seq %.1f us, T_free-running %.1f us, T_SI(plan) %.1f us, T_SI(plan, graph replay) %.1f us, stand-ins solo %.1f us"
        % (t_seq * 1e6, t_free * 1e6, t_si * 1e6, t_graph * 1e6, t_comm * 1e6))

    # The step is timed both ways it can be issued (operator by operator, or as one replay of its recorded graph: same
    # kernels, bitwise the same results); the faster one is the step time, and config.execution says which.
    t_eager = t_si
    execution = "eager (one launch per operator)"
    if t_graph < t_si:
        t_si, execution = t_graph, "graph replay (dh_si_graph_launch)"
    value = flops / t_si / 1e12
    # Spread of the step time: events between consecutive steps on strand alpha's stream (every step forks from it
    # and joins it), same plan and execution as `value`.
    step_fn = ((lambda: dh.dh_si_graph_launch(graph, sa)) if execution.startswith("graph")
               else (lambda: run.si_step(alpha, beta, best_plan, sa, sb, sc)))
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    for _ in range(3):
        step_fn()
    marks[0].record(sa)
    for i in range(args.steps):
        step_fn()
        marks[i + 1].record(sa)
    torch.cuda.synchronize()
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))
    pct = lambda q: per_step[min(len(per_step) - 1, int(q * len(per_step)))]
    # roofline of the dominant kernel: the first FFN GEMM (gate/up projection; largest share of the FLOPs), timed
    # alone with events on the stream it is launched on.  MoE: one local expert's balanced share of the rows.
    Hd = cfg["hidden"]
    T = run.T if cfg["arch"] != "moe" else 2 * run.T // cfg["n_local"]
    F2 = cfg["ffn"] if cfg["arch"] == "gpt" else 2 * cfg["ffn"]
    a_mat = torch.empty(T, Hd, dtype=torch.bfloat16, device="cuda").normal_()
    b_mat = torch.empty(Hd, F2, dtype=torch.bfloat16, device="cuda").normal_(0, 0.02)
    c_mat = torch.empty(T, F2, dtype=torch.bfloat16, device="cuda")
    wsb = dh.dh_gemm_workspace_bytes(dh.DH_BF16, 0, 0, T, F2, Hd)
    gws = torch.empty(max(wsb, 256), dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    reps = 50
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for _ in range(5):
        dh.dh_gemm(dh.DH_BF16, 0, 0, T, F2, Hd, a_mat, b_mat, c_mat, False, gws, wsb, sa)
    e0.record(sa)
    for _ in range(reps):
        dh.dh_gemm(dh.DH_BF16, 0, 0, T, F2, Hd, a_mat, b_mat, c_mat, False, gws, wsb, sa)
    e1.record(sa)
    torch.cuda.synchronize()
    gemm_s = e0.elapsed_time(e1) * 1e-3 / reps
    gemm_tflops = 2.0 * T * F2 * Hd / gemm_s / 1e12
    log("dominant GEMM [%d x %d x %d]: %.1f us, %.1f TFLOP/s" % (T, F2, Hd, gemm_s * 1e6, gemm_tflops))

    # Composition of the stand-in (communication) time in the manner of Table 7: the share SI hides, the visible share
    # that launch intervals cost (what the graph replay of the same plan saves over eager launches), the visible rest
    # (kernel slowdown under co-execution).  Hidden is capped at the whole: SI also overlaps work that is not communication.
    comp = None
    if t_comm > 0:
        hidden = min(1.0, max(0.0, (t_seq - t_eager) / t_comm))
        launch = min(1.0 - hidden, max(0.0, (t_eager - t_graph) / t_comm))
        comp = {"hidden": hidden, "visible_launch_interval": launch, "visible_slowdown": 1.0 - hidden - launch}
    out = {
        "metric": "SI layer fwd+bwd TFLOP/s per MI355X (% bf16 peak); speedup vs sequential",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": t_si * 1e3, "ms_per_step_events": {"p10": pct(0.1), "median": pct(0.5), "p90": pct(0.9)},
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg["bf16"] else "f32", "data": "synthetic",
        "config": {"workload": args.workload, "arch": cfg["arch"], "tokens_per_strand": run.T, "comm_blocks": args.comm_blocks,
                   "cp": [cfg["cp_rank"], cfg["cp_ranks"]] if cfg["arch"] == "llama_cp" else None, "plan_pairs": len(pairs), "plan": best_name, "execution": execution, "standins_on": comm_placement},
        "pct_bf16_peak": 100.0 * value / BF16_MFMA_PEAK_TFLOPS,
        "tflops_full_attention_convention": H.model_flops(cfg, full_attention=True) / t_si / 1e12,
        "tokens_per_s": run.T / t_si,
        "speedup_vs_sequential": t_seq / t_si,
        "ms_sequential": t_seq * 1e3, "ms_free_running": t_free * 1e3, "ms_eager": t_eager * 1e3, "ms_graph_replay": t_graph * 1e3,
        "ms_round_robin": t_rr * 1e3, "ms_wgrad_fixed": t_fixed * 1e3, "ms_wgrad_in_strand": t_in_strand * 1e3,
        "ms_one_comm_stream": t_shared * 1e3 if t_shared is not None else None,
        "comm_hidden_frac": (t_seq - t_si) / t_comm if t_comm > 0 else None,
        "comm_composition": comp,
        "roofline": {"bound": "mfma", "achieved": gemm_tflops, "peak": BF16_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": gemm_tflops / BF16_MFMA_PEAK_TFLOPS, "traffic": HBM_TRAFFIC_BYTES.get(args.workload),
                     "traffic_unit": "bytes/launch", "algorithmic_bytes": 2.0 * (T * Hd + Hd * F2 + T * F2),
                     "kernel": "gemm_bf16_kernel (first FFN projection %dx%dx%d)" % (T, F2, Hd)},
    }
    dh.dh_si_graph_destroy(graph)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, flops)
    run.close()
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
