"""Several layers under SI on one GPU (forward sweep of one micro-batch co-run with the backward sweep of the
previous one, activations in the shared two-triangle arena) against the fp64 oracle applied layer by layer."""
import numpy as np
import pytest
import torch

from oracle import layer_ref as R
from paper_2411_15871_amd import harness as H
from paper_2411_15871_amd import inputs as gen

pytestmark = pytest.mark.gpu


def rel(a, b):
    return np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-30)


@pytest.mark.parametrize("bf16,n_layers,n_mb", [(False, 3, 3), (True, 4, 2), (False, 1, 2)])
def test_stack_phases_match_oracle(bf16, n_layers, n_mb):
    from paper_2411_15871_amd import dhelix as dh
    c = dict(batch=2, seq=75, hidden=136, nq=4, nkv=2, d=32, ffn=200, n_ranks=3) if not bf16 else \
        dict(batch=1, seq=330, hidden=264, nq=2, nkv=1, d=128, ffn=328, n_ranks=2)
    T, Hd, tol = c["batch"] * c["seq"], c["hidden"], (2e-2 if bf16 else 1e-5)
    n_qkv = (c["nq"] + 2 * c["nkv"]) * c["d"]
    cfgkw = dict(arch=dh.DH_ARCH_LLAMA, dtype=dh.DH_BF16 if bf16 else dh.DH_F32, batch=c["batch"], seq=c["seq"], hidden=Hd,
                 n_q_heads=c["nq"], n_kv_heads=c["nkv"], head_dim=c["d"], ffn=c["ffn"], eps=1e-5, rope_base=10000.0,
                 n_ranks=c["n_ranks"], comm_blocks=0, n_experts=0, n_local_experts=0)
    stack = dh.dh_stack_create(n_layers, **cfgkw)
    try:
        w_np = [gen.llama_weights(Hd, n_qkv, c["nq"] * c["d"], c["ffn"], bf16, seed=gen.SEED_WEIGHTS + 100 * l) for l in range(n_layers)]
        w = [{k: H.to_dev(v, bf16) for k, v in wl.items()} for wl in w_np]
        g = [{"d" + k: torch.zeros(v.shape, dtype=torch.float32, device="cuda") for k, v in wl.items()} for wl in w_np]
        for l in range(n_layers):
            dh.dh_layer_bind_weights(dh.dh_stack_layer(stack, l), **w[l])
            dh.dh_layer_bind_wgrads(dh.dh_stack_layer(stack, l), **g[l])
        n_peers = c["n_ranks"] - 1
        peers_np = {k: gen.peer_partials(300 + 10 * i, n_peers, T, Hd, bf16) for i, k in enumerate(("ar1", "ar2", "ar3", "ar4"))}
        peers = {k: H.to_dev(v, bf16) for k, v in peers_np.items()}
        xs_np = [gen.strand_input(m, T, Hd, bf16) for m in range(n_mb)]
        douts_np = [gen.strand_upstream_grad(m, T, Hd, bf16) for m in range(n_mb)]
        xs = [H.to_dev(a, bf16) for a in xs_np]; douts = [H.to_dev(a, bf16) for a in douts_np]
        outs = [torch.empty_like(xs[0]) for _ in range(n_mb)]; dxs = [torch.empty_like(xs[0]) for _ in range(n_mb)]
        arena_bytes, ws_bytes = dh.dh_stack_arena_bytes(stack), dh.dh_stack_workspace_bytes(stack)
        assert arena_bytes < dh.dh_stack_unshared_bytes(stack) or n_layers == 1
        arena = torch.empty(arena_bytes, dtype=torch.uint8, device="cuda"); ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
        sa, sb, sc = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
        layer0 = dh.dh_stack_layer(stack, 0)
        gf, gb = dh.dh_layer_op_graph(layer0, 0), dh.dh_layer_op_graph(layer0, 1)
        plan = dh.make_plan(list(range(gf.n_ops)), list(range(gb.n_ops)), [(0, 5, 0, 6), (5, gf.n_ops, 6, gb.n_ops)])
        fwd = lambda m: (xs[m], outs[m], peers["ar1"], peers["ar2"])
        bwd = lambda m: (douts[m], dxs[m], peers["ar3"], peers["ar4"])
        with pytest.raises(dh.DhelixError):  # nothing to run backward yet
            dh.dh_stack_phase(stack, None, bwd(0), plan, arena, arena_bytes, ws, ws_bytes, sa, sb, sc)
        print("warm-up", flush=True)
        dh.dh_stack_phase(stack, fwd(0), None, None, arena, arena_bytes, ws, ws_bytes, sa, sb, sc)
        for m in range(1, n_mb):
            print("phase", m, flush=True)
            dh.dh_stack_phase(stack, fwd(m), bwd(m - 1), plan, arena, arena_bytes, ws, ws_bytes, sa, sb, sc)
        with pytest.raises(dh.DhelixError):  # the last micro-batch still waits for its backward
            dh.dh_stack_phase(stack, fwd(0), None, None, arena, arena_bytes, ws, ws_bytes, sa, sb, sc)
        print("cool-down", flush=True)
        dh.dh_stack_phase(stack, None, bwd(n_mb - 1), None, arena, arena_bytes, ws, ws_bytes, sa, sb, sc)
        torch.cuda.synchronize()
        # oracle, layer by layer
        cfg = R.LayerCfg(batch=c["batch"], seq=c["seq"], H=Hd, nq=c["nq"], nkv=c["nkv"], d=c["d"], F=c["ffn"])
        W = [{k: v.astype(np.float64) for k, v in wl.items()} for wl in w_np]
        gsum = [dict() for _ in range(n_layers)]
        for m in range(n_mb):
            h, saved = xs_np[m].astype(np.float64), []
            for l in range(n_layers):
                h, sv = R.llama_fwd(cfg, W[l], h, peers_np)
                saved.append(sv)
            assert rel(H.to_np(outs[m]), h) <= tol, ("out", m)
            d = douts_np[m].astype(np.float64)
            for l in reversed(range(n_layers)):
                d, gr, _ = R.llama_bwd(cfg, W[l], saved[l], d, peers_np)
                for k, v in gr.items():
                    gsum[l][k] = gsum[l].get(k, 0) + v
            assert rel(H.to_np(dxs[m]), d) <= tol, ("dx", m)
        for l in range(n_layers):
            for k, v in gsum[l].items():
                assert rel(H.to_np(g[l][k]), v) <= tol, (l, k)
    finally:
        dh.dh_stack_destroy(stack)
