#!/usr/bin/env python3
"""Benchmark of one Strand-Interleaving layer step (alpha forward || beta backward) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c2_llama8b_tp8]

A step = one dh_si_step over one micro-batch per strand with all inputs resident in HBM.  Prints one
JSON line: model TFLOP/s of the step (2MNK per GEMM, causal attention at half dense, backward =
2x forward; the step time is the median of per-step event times), SI speedup over sequential
alpha-then-beta through the same executor, the share of the collective stand-ins' time that is hidden
(1 - (T_SI - T_SI without communication) / sum of the stand-ins' solo times), the same again with the
stand-ins at a link-like rate (`link_rate`), predicted against measured step time, the roofline of
every operator and of the one with the largest share of the solo time, and the CPU oracle baseline.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)
# The step uses up to five streams at once (two strands, a communication stream per strand, the cross-node stream).  The
# HIP runtime spreads a process's streams over GPU_MAX_HW_QUEUES hardware queues (4 unless told otherwise) and two streams
# on one queue run one after the other; eight queues give every stream its own.  Read when the runtime starts.
if int(os.environ.get("GPU_MAX_HW_QUEUES", "0") or 0) < 8:
    os.environ["GPU_MAX_HW_QUEUES"] = "8"

BF16_MFMA_PEAK_TFLOPS = 2500.0  # MI355X dense bf16
HBM_PEAK_GBS = 8000.0           # MI355X HBM3E
# kernels behind an operator name (for the roofline's description)
OP_KERNELS = {"ATTN": "attention kernels and their merge launches", "FC1": "gemm_bf16_kernel", "FC2": "gemm_bf16_kernel",
              "QKV": "gemm_bf16_kernel", "PROJ": "gemm_bf16_kernel"}


def read_traffic(workload, op):
    """HBM bytes per launch of an operator from profiles/roofline_traffic.txt (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs
    scaled by a copy kernel of known size; the file names its sources).  None if the file has no line for it."""
    path = os.path.join(ROOT, "profiles", "roofline_traffic.txt")
    try:
        for line in open(path):
            f = line.split()
            if len(f) >= 3 and f[0] == workload and f[1] == op:
                return float(f[2])
    except OSError:
        pass
    return None


def op_work(cfg, name):
    """Algorithmic work of one launch of an operator: ("mfma", flops) for the dense contractions (2MNK; causal attention at
    half the dense count, backward twice the forward), ("hbm", bytes) for the memory-bound operators (every operand read
    once, every result written once).  None for operators without a formula here."""
    arch = cfg["arch"]
    T, Hd, nq, nkv, d, F = cfg["batch"] * cfg["seq"], cfg["hidden"], cfg["nq"], cfg["nkv"], cfg["d"], cfg["ffn"]
    es = 2 if cfg["bf16"] else 4
    nqkv, no, R = (nq + 2 * nkv) * d, nq * d, cfg["n_ranks"]
    Tf = 2 * T if arch == "moe" else T                 # rows entering the FFN GEMMs
    Fin = F if arch == "gpt" else 2 * F
    Ts = T // R if arch == "gpt" else T
    attn = 0.5 * 4.0 * cfg["batch"] * cfg["seq"] ** 2 * d * nq
    if arch == "llama_cp":
        attn += 4.0 * cfg["batch"] * cfg["seq"] ** 2 * cfg["cp_rank"] * d * nq
    direction, op = name.split("_", 1)
    gemm = {"QKV": 2.0 * T * Hd * nqkv, "PROJ": 2.0 * T * Hd * no, "FC1": 2.0 * Tf * Hd * Fin, "FC2": 2.0 * Tf * Hd * F}
    for k, v in gemm.items():
        if op in (k, k + "_DGRAD", k + "_WGRAD"):
            return "mfma", v
    if op == "ATTN":
        return "mfma", attn * (2.0 if direction == "B" else 1.0)
    row = Ts * Hd * es
    if op in ("AR1", "AR2", "AR3", "AR4"):
        return "hbm", (R + 1.0) * T * Hd * es
    if op in ("RS1", "RS2", "RS3", "RS4"):
        return "hbm", (R + 1.0) * row
    if op in ("AG1", "AG2", "AG3", "AG4"):
        return "hbm", 2.0 * T * Hd * es
    if op in ("A2A_DISPATCH", "A2A_COMBINE", "PERMUTE") and arch == "moe":
        return "hbm", 2.0 * Tf * Hd * es
    if op == "NORM1":
        return "hbm", (2.0 if direction == "F" else 4.0) * row
    if op == "NORM2":
        return "hbm", 4.0 * row
    if op == "ROPE":
        return "hbm", 2.0 * T * (nq + nkv) * d * es
    if op == "ACT":
        return "hbm", Tf * es * ((Fin + F) if direction == "F" else (Fin + F + Fin))
    if op == "BDA2":
        return "hbm", 3.0 * row
    return None


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
    ap.add_argument("--profile-reps", type=int, default=10)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--layers", type=int, default=0, help="stack this many layers: alpha sweeps forward while beta sweeps backward")
    ap.add_argument("--sequential-probe", action="store_true",
                    help="only run alpha's forward then beta's backward, one kernel at a time, --steps times (for rocprofv3: every kernel's solo "
                         "duration and counters at the workload's shapes)")
    ap.add_argument("--link-blocks", type=int, default=64,
                    help="thread blocks per stand-in of the second, link-rate regime (0 = skip it)")
    ap.add_argument("--barrier-cost", type=float, default=5e-6, help="seconds a cross-strand barrier is priced at in the plan search")
    ap.add_argument("--plan-table", default=None, metavar="PATH",
                    help="also write the predicted-vs-measured table of the plan candidates to this text file")
    ap.add_argument("--pair-table", default=None, metavar="PATH",
                    help="also write the measured operator-pair table (solo times, co-run rates, Eq. 1 overlap factors) to this text file")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (the SI step is a per-GPU schedule); use --gpus 1")

    import torch
    from paper_2411_15871_amd import dhelix as dh
    from paper_2411_15871_amd import harness as H

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
    sa, sb, sc, scb = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
    sx = None
    if cfg["arch"] == "llama_cp":  # Sec. 5: cross-node transfers get a stream of their own
        sx = torch.cuda.Stream()
        dh.dh_layer_set_cross_stream(run.layer, sx)
    gf, gb = dh.dh_layer_op_graph(run.layer, 0), dh.dh_layer_op_graph(run.layer, 1)
    nf, nb = gf.n_ops, gb.n_ops
    fnames, bnames = dh.op_names(H.ARCH[cfg["arch"]], 0), dh.op_names(H.ARCH[cfg["arch"]], 1)
    seq_plan = dh.dh_plan_sequential(run.layer)
    free_plan = dh.make_plan(list(seq_plan.fwd_order[:nf]), list(seq_plan.bwd_order[:nb]), [(0, nf, 0, nb)])
    # where the stand-ins go is part of the schedule (Sec. 5: one stream per kind of work): in their strand's stream, on
    # one communication stream, or on a communication stream per strand
    placements = {"strand streams": (dh.lanes(0, 0, 1 if sx else 0), None, None),
                  "one communication stream": (dh.lanes(1, 1, 1 if sx else 0), sc, None),
                  "a communication stream per strand": (dh.lanes(1, 2, 1 if sx else 0), sc, scb)}

    def describe(plan):
        fo, bo, pairs = dh.plan_to_py(plan)
        side = [bnames[o] for o in range(nb) if plan.bwd_side[o]]
        return [([fnames[o] for o in fo[a:b]], [bnames[o] for o in bo[c:d]]) for a, b, c, d in pairs], side

    def event_times(fn, steps, warmup):
        """Per-step durations from events recorded between consecutive steps on strand alpha's stream (every step forks
        from that stream and joins it)."""
        for _ in range(warmup):
            fn()
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
        marks[0].record(sa)
        for i in range(steps):
            fn()
            marks[i + 1].record(sa)
        torch.cuda.synchronize()
        return sorted(marks[i].elapsed_time(marks[i + 1]) * 1e-3 for i in range(steps))

    def median(v):
        return v[len(v) // 2]

    def regime(label, comm_blocks, steps, warmup, table_path=None):
        """Offline part of the method (Sec. 3.2, 4.2) and the timed step, with the stand-ins at one cost."""
        dh.dh_layer_set_comm_blocks(run.layer, comm_blocks)
        dh.dh_layer_set_beta_comm_stream(run.layer, scb)   # the profile co-runs the two strands' collectives on two streams
        t0 = time.perf_counter()
        table = dh.dh_profile_pairs(run.layer, alpha.fwd_args, beta.bwd_args, run.ws, run.ws_bytes, sa, sb, sc, args.profile_reps)
        t_prof = time.perf_counter() - t0
        t_f = [table.t_fwd[i] for i in range(nf)]
        t_b = [table.t_bwd[j] for j in range(nb)]
        t_comm = sum(t_f[i] for i in range(nf) if gf.is_comm[i]) + sum(t_b[j] for j in range(nb) if gb.is_comm[j])
        log("[%s] profile %.2fs; sum of solo times %.1f us, of which stand-ins %.1f us" % (label, t_prof, (sum(t_f) + sum(t_b)) * 1e6, t_comm * 1e6))
        log("[%s] fwd solo us:" % label, {fnames[i]: round(t_f[i] * 1e6, 1) for i in range(nf)})
        log("[%s] bwd solo us:" % label, {bnames[j]: round(t_b[j] * 1e6, 1) for j in range(nb)})
        if args.pair_table:
            write_pair_table(args.pair_table if label == "default" else args.pair_table + "." + label.replace(" ", "_"), args, table,
                             fnames, bnames, t_f, t_b)
        rows = []   # (name, placement, predicted, measured, plan)
        probe = max(15, steps // 3)

        def measure(plan, placement):
            lanes, c, cb = placements[placement]
            dh.dh_layer_set_beta_comm_stream(run.layer, cb)
            return median(event_times(lambda: run.si_step(alpha, beta, plan, sa, sb, c), probe, 6))
        t0 = time.perf_counter()
        for placement, (lanes, c, cb) in placements.items():
            plan, predicted, info = dh.dh_plan_search_lanes(gf, gb, table, lanes, args.barrier_cost, 0)
            rows.append(["searched", placement, predicted, None, plan, info])
            for name, q in (("default orders, one pair", free_plan), ("sequential", seq_plan)):
                rows.append([name, placement, dh.dh_plan_cost(gf, gb, table, q, lanes, args.barrier_cost), None, q, None])
        t_search = time.perf_counter() - t0
        info = rows[0][5]
        log("[%s] search %.2fs over %d x %d operator orders (%s), %d refined by barrier placement" %
            (label, t_search, info.orders_fwd_tried, info.orders_bwd_tried, "truncated" if info.truncated else "all of them", info.refined))
        for r in rows:
            r[3] = measure(r[4], r[1])
        # Every plan that runs comes from dh_plan_search_lanes, one per placement of the stand-ins; which of the three
        # placements to use is a property of the machine (how its queues and caches take a third and fourth stream) that
        # the pairwise table does not hold, so that one choice is made by measurement.  The other rows are measured too,
        # so that the table shows what the model is worth.
        searched = [r for r in rows if r[0] == "searched"]
        best = min(searched, key=lambda r: r[3])
        lines = ["predicted (lane model) vs measured step time, workload %s, stand-ins on %s blocks" % (args.workload, comm_blocks or "payload-sized"),
                 "%-28s %-36s %12s %12s %8s" % ("plan", "stand-ins on", "predicted us", "measured us", "ratio")]
        for name, placement, pred, meas, _, _ in rows:
            lines.append("%-28s %-36s %12.1f %12.1f %8.3f%s" % (name, placement, pred * 1e6, meas * 1e6, pred / meas,
                                                                   "   <- chosen" if (name, placement) == (best[0], best[1]) else ""))
        for ln in lines:
            log("[%s] " % label + ln)
        if table_path:
            with open(table_path, "a") as f:
                f.write("\n".join(lines) + "\n\n")
        plan, placement = best[4], best[1]
        lanes, c, cb = placements[placement]
        segs, side = describe(plan)
        log("[%s] chosen plan (stand-ins on %s), beside the strand %s:" % (label, placement, side), segs)
        dh.dh_layer_set_beta_comm_stream(run.layer, cb)
        step = lambda q=plan: run.si_step(alpha, beta, q, sa, sb, c)
        ts_si = event_times(step, steps, warmup)
        ts_seq = event_times(lambda: run.si_step(alpha, beta, seq_plan, sa, sb, c), max(10, steps // 2), 3)
        # the same two schedules with every stand-in launching nothing (events and dependencies stay): what the
        # communication costs each of them
        dh.dh_layer_set_comm_blocks(run.layer, -1)
        ts_si_nc = event_times(step, max(10, steps // 2), 3)
        ts_seq_nc = event_times(lambda: run.si_step(alpha, beta, seq_plan, sa, sb, c), max(10, steps // 2), 3)
        dh.dh_layer_set_comm_blocks(run.layer, comm_blocks)
        t_si, t_seq, t_si_nc, t_seq_nc = median(ts_si), median(ts_seq), median(ts_si_nc), median(ts_seq_nc)
        visible = max(0.0, t_si - t_si_nc)
        rec = {"comm_blocks": comm_blocks, "standins_on": placement, "plan_pairs": len(segs), "beside_strand": side,
               "ms_si": t_si * 1e3, "ms_sequential": t_seq * 1e3, "ms_si_no_comm": t_si_nc * 1e3, "ms_sequential_no_comm": t_seq_nc * 1e3,
               "ms_standins_solo": t_comm * 1e3, "speedup_vs_sequential": t_seq / t_si,
               "comm_visible_ms": visible * 1e3, "comm_hidden_frac": (1.0 - visible / t_comm) if t_comm > 0 else None,
               "comm_hidden_frac_sequential": (1.0 - max(0.0, t_seq - t_seq_nc) / t_comm) if t_comm > 0 else None,
               "predicted_ms": best[2] * 1e3, "predicted_over_measured": best[2] / t_si,
               "orders_searched": [info.orders_fwd_tried, info.orders_bwd_tried], "orders_truncated": bool(info.truncated)}
        log("[%s] T_seq %.1f us, T_SI %.1f us (predicted %.1f), without communication: T_seq %.1f, T_SI %.1f; stand-ins solo %.1f us; hidden %.2f" %
            (label, t_seq * 1e6, t_si * 1e6, best[2] * 1e6, t_seq_nc * 1e6, t_si_nc * 1e6, t_comm * 1e6, rec["comm_hidden_frac"] or 0.0))
        if comm_blocks > 0 and dh.dh_layer_set_fused_collective(run.layer, 3):
            # The backward all-reduces carried by their strand's weight-gradient GEMMs, one launch each (Sec. 6.3's closing
            # remark on Table 7: computation and communication in one kernel): profile, search and timing anew under the
            # placement chosen above; the pair's makespan against the two kernels co-running on two streams (pair table).
            dh.dh_layer_set_beta_comm_stream(run.layer, scb)
            table_f = dh.dh_profile_pairs(run.layer, alpha.fwd_args, beta.bwd_args, run.ws, run.ws_bytes, sa, sb, sc, args.profile_reps)
            plan_f, pred_f, _ = dh.dh_plan_search_lanes(gf, gb, table_f, lanes, args.barrier_cost, 0)
            dh.dh_layer_set_beta_comm_stream(run.layer, cb)
            t_si_f = median(event_times(lambda: run.si_step(alpha, beta, plan_f, sa, sb, c), steps, warmup))
            pairs_f = {}
            for ar_f, ar_b, wg in (("F_AR1", "B_AR3", "B_FC1_WGRAD"), ("F_AR2", "B_AR4", "B_QKV_WGRAD")):
                if ar_f in fnames and ar_b in bnames and wg in bnames and table_f.t_bwd[bnames.index(wg)] < 1e-6:
                    i, j = fnames.index(ar_f), bnames.index(wg)
                    pairs_f[ar_b + "+" + wg] = {"one_launch_us": table_f.t_bwd[bnames.index(ar_b)] * 1e6,
                                                "two_kernels_corun_us": table.p_pair[i][j] * 1e6,
                                                "allreduce_solo_us": t_b[bnames.index(ar_b)] * 1e6, "gemm_solo_us": t_b[j] * 1e6}
            dh.dh_layer_set_fused_collective(run.layer, 0)
            rec["fused_collective"] = {"ms_si": t_si_f * 1e3, "predicted_ms": pred_f * 1e3, "pairs": pairs_f,
                                       "comm_hidden_frac": (1.0 - max(0.0, t_si_f - t_si_nc) / t_comm) if t_comm > 0 else None}
            log("[%s] all-reduces carried by weight-gradient GEMMs: T_SI %.1f us (predicted %.1f); %s" % (label, t_si_f * 1e6, pred_f * 1e6, pairs_f))
        return rec, plan, (c, cb), table, ts_si

    if args.plan_table and os.path.exists(args.plan_table):
        os.remove(args.plan_table)
    rec, best_plan, (c_best, cb_best), table, ts_si = regime("default", args.comm_blocks, args.steps, args.warmup, args.plan_table)
    t_si = median(ts_si)
    pct = lambda q: ts_si[min(len(ts_si) - 1, int(q * len(ts_si)))]
    dh.dh_layer_set_beta_comm_stream(run.layer, cb_best)
    step_fn = lambda: run.si_step(alpha, beta, best_plan, sa, sb, c_best)
    t_wall = time_steps(step_fn, args.steps, 3, torch)   # the same steps back to back against the host clock

    # ablations of Sec. 6.1 / 6.4 through the same executor: round-robin interleaving ("Wavelet+"), the searched plan with
    # the weight-gradient operators left in their default places, the default orders free-running, and the replay of
    # the chosen plan from a HIP graph (one launch per step instead of one per operator)
    probe = max(5, args.steps // 5)
    rr_plan = dh.dh_plan_round_robin(gf, gb)
    lanes_best = placements[rec["standins_on"]][0]
    fixed_plan, _, _ = dh.dh_plan_search_lanes(gf, gb, table, lanes_best, args.barrier_cost, 1)
    t_rr = median(event_times(lambda: run.si_step(alpha, beta, rr_plan, sa, sb, c_best), probe, 2))
    t_fixed = median(event_times(lambda: run.si_step(alpha, beta, fixed_plan, sa, sb, c_best), probe, 2))
    t_free = median(event_times(lambda: run.si_step(alpha, beta, free_plan, sa, sb, c_best), probe, 2))
    graph = dh.dh_si_graph_create(run.layer, alpha.fwd_args, beta.bwd_args, best_plan, run.ws, run.ws_bytes, sa, sb)
    t_graph = median(event_times(lambda: dh.dh_si_graph_launch(graph, sa), probe, 2))
    dh.dh_si_graph_destroy(graph)
    t_shared = None
    if sx is not None:  # ablation of Sec. 6.4 ("Communication and Communication Overlap"): both kinds of transfer on one stream
        dh.dh_layer_set_cross_stream(run.layer, None)
        t_shared = median(event_times(lambda: run.si_step(alpha, beta, best_plan, sa, sb, sc), probe, 2))
        dh.dh_layer_set_cross_stream(run.layer, sx)
    log("ablations: round-robin %.1f us, weight gradients fixed %.1f us, default orders free-running %.1f us, graph replay %.1f us" %
        (t_rr * 1e6, t_fixed * 1e6, t_free * 1e6, t_graph * 1e6))
    # SwiGLU inside the GEMM epilogues against the separate activation operators: the same plan, same results (bitwise)
    t_unfused = t_seq_unfused = None
    if dh.dh_layer_set_fused_activation(run.layer, True):
        dh.dh_layer_set_fused_activation(run.layer, False)
        n_ab = max(15, args.steps // 2)
        t_unfused = median(event_times(lambda: run.si_step(alpha, beta, best_plan, sa, sb, c_best), n_ab, 3))
        t_seq_unfused = median(event_times(lambda: run.si_step(alpha, beta, seq_plan, sa, sb, c_best), n_ab, 3))
        dh.dh_layer_set_fused_activation(run.layer, True)
        t_again = median(event_times(lambda: run.si_step(alpha, beta, best_plan, sa, sb, c_best), n_ab, 3))
        log("activation as separate operators: T_SI %.1f us, T_seq %.1f us (fused, timed again right after: T_SI %.1f us)" %
            (t_unfused * 1e6, t_seq_unfused * 1e6, t_again * 1e6))

    # the same workload with the stand-ins at a link-like rate (64 thread blocks: a 32 MiB all-reduce then takes what an
    # 8-GPU xGMI ring takes): profile, search and timing anew
    link = None
    if args.link_blocks > 0 and rec["ms_standins_solo"] > 0:
        link, _, _, _, _ = regime("link rate", args.link_blocks, max(10, args.steps // 2), 3, args.plan_table)
        dh.dh_layer_set_comm_blocks(run.layer, args.comm_blocks)
        dh.dh_layer_set_beta_comm_stream(run.layer, cb_best)

    # Roofline of every operator: algorithmic flops or bytes over its solo launch time, timed with events on the stream it
    # runs on (dh_profile_solo); the headline roofline is the operator with the largest share of the step's solo time.
    dh.dh_layer_set_beta_comm_stream(run.layer, scb)
    tf20, tb20 = dh.dh_profile_solo(run.layer, alpha.fwd_args, beta.bwd_args, run.ws, run.ws_bytes, sa, sb, sc, 20)
    dh.dh_layer_set_beta_comm_stream(run.layer, cb_best)
    ops, fused = [], []
    total_solo = sum(tf20[:nf]) + sum(tb20[:nb])
    for names, ts in ((fnames, tf20), (bnames, tb20)):
        for k, name in enumerate(names):
            w = op_work(cfg, name)
            if w is None:
                continue
            kind, amount = w
            if ts[k] < 1e-6:   # launches nothing: SwiGLU merged into the neighbouring GEMM's epilogue
                fused.append(name)
                continue
            peak = BF16_MFMA_PEAK_TFLOPS if kind == "mfma" else HBM_PEAK_GBS
            ach = amount / ts[k] / (1e12 if kind == "mfma" else 1e9)
            ops.append({"op": name, "bound": kind, "solo_us": ts[k] * 1e6, "share_of_solo": ts[k] / total_solo,
                        "work": amount, "work_unit": "flop" if kind == "mfma" else "bytes", "achieved": ach,
                        "unit": "TFLOP/s" if kind == "mfma" else "GB/s", "peak": peak, "frac": ach / peak})
    dom = max(ops, key=lambda o: o["solo_us"])
    log("operator rooflines (solo):", ", ".join("%s %.1fus %.0f%%" % (o["op"], o["solo_us"], 100 * o["frac"]) for o in ops))
    traffic = read_traffic(args.workload, dom["op"])
    roofline = {"bound": dom["bound"], "achieved": dom["achieved"], "peak": dom["peak"], "unit": dom["unit"], "frac": dom["frac"],
                "traffic": traffic, "traffic_unit": "bytes/launch", "algorithmic_work": dom["work"], "work_unit": dom["work_unit"],
                "kernel": "%s (the operator with the largest share, %.1f %%, of the step's summed solo time; %s)" %
                          (dom["op"], 100 * dom["share_of_solo"], OP_KERNELS.get(dom["op"].split("_")[1] if "_" in dom["op"] else dom["op"], "its kernels")),
                "solo_us": dom["solo_us"]}

    value = flops / t_si / 1e12
    # Composition of the stand-in (communication) time in the manner of Table 7: the share SI hides, the visible share
    # that launch intervals cost (what the graph replay of the same plan saves over eager launches), the visible rest
    # (kernel slowdown under co-execution).
    comp = None
    if rec["comm_hidden_frac"] is not None:
        hidden = min(1.0, max(0.0, rec["comm_hidden_frac"]))
        launch = min(1.0 - hidden, max(0.0, (t_si - t_graph) / (rec["ms_standins_solo"] * 1e-3)))
        comp = {"hidden": hidden, "visible_launch_interval": launch, "visible_slowdown": 1.0 - hidden - launch}
    segs, side = describe(best_plan)
    out = {
        "metric": "SI layer fwd+bwd TFLOP/s per MI355X (% bf16 peak); speedup vs sequential",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": t_si * 1e3, "ms_per_step_events": {"p10": pct(0.1) * 1e3, "median": t_si * 1e3, "p90": pct(0.9) * 1e3},
        "ms_per_step_host_clock": t_wall * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg["bf16"] else "f32", "data": "synthetic",
        "config": {"workload": args.workload, "arch": cfg["arch"], "tokens_per_strand": run.T, "comm_blocks": args.comm_blocks,
                   "cp": [cfg["cp_rank"], cfg["cp_ranks"]] if cfg["arch"] == "llama_cp" else None, "plan_pairs": len(segs),
                   "plan": "dh_plan_search_lanes (lane model, all operator orders), beside the strand: %s" % ("+".join(side) or "none"),
                   "execution": "eager (one launch per operator)", "standins_on": rec["standins_on"]},
        "pct_bf16_peak": 100.0 * value / BF16_MFMA_PEAK_TFLOPS,
        "tflops_full_attention_convention": H.model_flops(cfg, full_attention=True) / t_si / 1e12,
        "tokens_per_s": run.T / t_si,
        "speedup_vs_sequential": rec["speedup_vs_sequential"],
        "ms_sequential": rec["ms_sequential"], "ms_si_no_comm": rec["ms_si_no_comm"], "ms_sequential_no_comm": rec["ms_sequential_no_comm"],
        "ms_free_running": t_free * 1e3, "ms_graph_replay": t_graph * 1e3, "ms_round_robin": t_rr * 1e3, "ms_wgrad_fixed": t_fixed * 1e3,
        "ms_one_comm_stream": t_shared * 1e3 if t_shared is not None else None,
        "ms_separate_activation": t_unfused * 1e3 if t_unfused is not None else None,
        "ms_sequential_separate_activation": t_seq_unfused * 1e3 if t_seq_unfused is not None else None,
        "comm_hidden_frac": rec["comm_hidden_frac"], "comm_composition": comp,
        "predicted_ms": rec["predicted_ms"], "predicted_over_measured": rec["predicted_over_measured"],
        "link_rate": link,
        "roofline": roofline, "roofline_ops": ops, "ops_without_launch": fused,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, flops)
    run.close()
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
