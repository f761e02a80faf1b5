"""Device-memory plumbing around libdhelix for tests, the smoke check and the benchmark.

PyTorch is used for allocation, host<->device copies and streams only; every step of the layer
runs in the library's HIP kernels through the ctypes binding.
"""
import numpy as np
import torch

from . import dhelix as dh
from . import inputs as gen

CONFIGS = {
    "c1_tiny_fp32": dict(arch="llama", batch=1, seq=128, hidden=256, nq=4, nkv=4, d=64, ffn=688, n_ranks=2, bf16=False),
    "c2_llama8b_tp8": dict(arch="llama", batch=1, seq=4096, hidden=4096, nq=4, nkv=1, d=128, ffn=1792, n_ranks=8, bf16=True),
    "c3_gpt_tp8_sp": dict(arch="gpt", batch=2, seq=2048, hidden=8192, nq=8, nkv=8, d=128, ffn=4096, n_ranks=8, bf16=True),
    "c4_llama70b_tp8": dict(arch="llama", batch=1, seq=8192, hidden=8192, nq=8, nkv=1, d=128, ffn=3584, n_ranks=8, bf16=True),
    "c5_phimoe_ep8": dict(arch="moe", batch=1, seq=4096, hidden=4096, nq=32, nkv=8, d=128, ffn=6400, n_ranks=1, bf16=True,
                          n_experts=16, n_local=2),
    # Llama-8B TP8 shard at a 16K context cut over 4 context-parallel ranks; this GPU holds the third chunk
    "c6_llama8b_tp8_cp4": dict(arch="llama_cp", batch=1, seq=4096, hidden=4096, nq=4, nkv=1, d=128, ffn=1792, n_ranks=8, bf16=True,
                               cp_ranks=4, cp_rank=2),
}
ARCH = {"llama": dh.DH_ARCH_LLAMA, "gpt": dh.DH_ARCH_GPT, "moe": dh.DH_ARCH_MOE, "llama_cp": dh.DH_ARCH_LLAMA_CP}


def model_flops(cfg, full_attention=False):
    """Model FLOPs of one forward+backward of the layer share: 2*M*N*K per GEMM, causal attention at
    half of the dense 4*s^2*d per head, backward = 2 x forward (no recompute credit)."""
    T, H, nq, nkv, d, F = cfg["batch"] * cfg["seq"], cfg["hidden"], cfg["nq"], cfg["nkv"], cfg["d"], cfg["ffn"]
    arch = cfg.get("arch", "llama")
    attn_gemm = 2.0 * T * H * ((nq + 2 * nkv) * d + nq * d)
    if arch == "gpt":
        ffn = 2.0 * T * H * 2 * F
    elif arch == "moe":
        ffn = 2.0 * (2 * T) * H * 3 * F  # every token visits two experts
    else:
        ffn = 2.0 * T * H * 3 * F
    attn = 0.5 * 4.0 * cfg["batch"] * cfg["seq"] ** 2 * d * nq
    if full_attention:  # the convention that counts the masked half of the score matrix too (Sec. 6.1 follows Megatron-LM's count)
        attn *= 2.0
    if arch == "llama_cp":  # the rank's queries also read cp_rank full chunks of earlier keys
        attn += 4.0 * cfg["batch"] * cfg["seq"] ** 2 * cfg["cp_rank"] * d * nq
    return 3.0 * (attn_gemm + ffn + attn)


def to_dev(a, bf16):
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    return t.to(torch.bfloat16) if bf16 else t


def to_np(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


class Strand:
    """One micro-batch strand's buffers: input, output, saved-activation slot, frozen peer buffers."""

    def __init__(self, run, seed):
        c = run.cfg
        arch, H, bf = c["arch"], c["hidden"], c["bf16"]
        rows = run.Ts  # rows of the layer input/output (the sequence shard for the GPT layer)
        self.x_np = gen.strand_input(seed, rows, H, bf)
        self.dout_np = gen.strand_upstream_grad(seed, rows, H, bf)
        n_peers = c["n_ranks"] - 1
        self.peers_np = {k: gen.peer_partials(base + 10 * i + 1000 * seed, n_peers, rows, H, bf)
                         for i, (k, base) in enumerate([("ar1", gen.SEED_PEER_FWD), ("ar2", gen.SEED_PEER_FWD),
                                                        ("ar3", gen.SEED_PEER_BWD), ("ar4", gen.SEED_PEER_BWD)])}
        if arch == "gpt":
            for i, (k, base, std) in enumerate([("ag1", gen.SEED_PEER_FWD, 1.0), ("ag2", gen.SEED_PEER_FWD, 1.0),
                                                ("ag3", gen.SEED_PEER_BWD, 1e-2), ("ag4", gen.SEED_PEER_BWD, 1e-2)]):
                self.peers_np[k] = gen.peer_partials(base + 50 + 10 * i + 1000 * seed, n_peers, rows, H, bf, std)
        if arch == "llama_cp":
            W, ncp = 2 * c["nkv"] * c["d"], c["cp_ranks"] - 1
            self.peers_np["kv"] = gen.peer_partials(gen.SEED_PEER_FWD + 70 + 1000 * seed, ncp, rows, W, bf, 1.0)
            self.peers_np["dkv"] = gen.peer_partials(gen.SEED_PEER_BWD + 70 + 1000 * seed, ncp, rows, W, bf, 1e-2)
        self.x = to_dev(self.x_np, bf)
        self.dout = to_dev(self.dout_np, bf)
        self.peers = {k: (to_dev(v, bf) if len(v) else None) for k, v in self.peers_np.items()}
        self.dkv_peers = None
        if arch == "llama_cp" and c["cp_rank"] > 0:
            self.dkv_peers = torch.zeros(c["cp_rank"], rows, 2 * c["nkv"] * c["d"], dtype=self.x.dtype, device="cuda")
        self.out = torch.empty_like(self.x)
        self.dx = torch.empty_like(self.x)
        self.saved = torch.empty(dh.dh_layer_saved_bytes(run.layer), dtype=torch.uint8, device="cuda")
        self.logits_np = self.logits = self.dlogits = None
        if arch == "moe":
            self.logits_np = gen.router_logits(run.T, c["n_experts"], gen.SEED_ROUTER + seed)
            self.logits = torch.from_numpy(self.logits_np).cuda()
            self.dlogits = torch.zeros_like(self.logits)
        p = self.peers
        self.fwd_args = dh.fwd_args(self.x, self.out, self.saved, p["ar1"], p["ar2"], p.get("ag1"), p.get("ag2"), self.logits,
                                    p.get("kv"))
        self.bwd_args = dh.bwd_args(self.dout, self.dx, self.x, self.saved, p["ar3"], p["ar4"], p.get("ag3"), p.get("ag4"),
                                    self.dlogits, p.get("dkv"), self.dkv_peers)


class LayerRun:
    def __init__(self, cfg):
        self.cfg = dict(cfg)
        c = self.cfg
        c.setdefault("arch", "llama")
        c.setdefault("eps", 1e-5)
        c.setdefault("rope_base", 10000.0)
        self.T = c["batch"] * c["seq"]
        self.Ts = self.T // c["n_ranks"] if c["arch"] == "gpt" else self.T
        bf = c["bf16"]
        self.layer = dh.dh_layer_create(arch=ARCH[c["arch"]], dtype=dh.DH_BF16 if bf else dh.DH_F32, batch=c["batch"],
                                        seq=c["seq"], hidden=c["hidden"], n_q_heads=c["nq"], n_kv_heads=c["nkv"],
                                        head_dim=c["d"], ffn=c["ffn"], eps=c["eps"], rope_base=c["rope_base"],
                                        n_ranks=c["n_ranks"], comm_blocks=c.get("comm_blocks", 0),
                                        n_experts=c.get("n_experts", 0), n_local_experts=c.get("n_local", 0),
                                        cp_ranks=c.get("cp_ranks", 0), cp_rank=c.get("cp_rank", 0),
                                        cross_blocks=c.get("cross_blocks", 0), rope_pairing=c.get("rope_pairing", 0),
                                        gelu_form=c.get("gelu_form", 0))
        n_qkv = (c["nq"] + 2 * c["nkv"]) * c["d"]
        if c["arch"] == "gpt":
            self.w_np = gen.gpt_weights(c["hidden"], n_qkv, c["nq"] * c["d"], c["ffn"], bf)
        elif c["arch"] == "moe":
            self.w_np = gen.moe_weights(c["hidden"], n_qkv, c["nq"] * c["d"], c["ffn"], c["n_local"], bf)
        else:
            self.w_np = gen.llama_weights(c["hidden"], n_qkv, c["nq"] * c["d"], c["ffn"], bf)
        self.w = {k: to_dev(v, bf) for k, v in self.w_np.items()}
        self.g = {"d" + k: torch.zeros(v.shape, dtype=torch.float32, device="cuda") for k, v in self.w_np.items()}
        dh.dh_layer_bind_weights(self.layer, **self.w)
        dh.dh_layer_bind_wgrads(self.layer, **self.g)
        self.ws_bytes = dh.dh_layer_workspace_bytes(self.layer, dh.DH_WS_SI)
        self.ws = torch.empty(max(self.ws_bytes, 256), dtype=torch.uint8, device="cuda")
        self.fwd_ws_bytes = dh.dh_layer_workspace_bytes(self.layer, dh.DH_WS_FWD)

    def close(self):
        if self.layer is not None:
            dh.dh_layer_destroy(self.layer)
            self.layer = None

    def zero_grads(self):
        for t in self.g.values():
            t.zero_()

    def grads_np(self):
        return {k: to_np(v) for k, v in self.g.items()}

    def strand(self, seed):
        return Strand(self, seed)

    def fwd(self, s, stream=None):
        dh.dh_layer_fwd(self.layer, s.fwd_args, self.ws, self.ws_bytes, stream)

    def bwd(self, s, stream=None):
        # the backward region of the SI workspace, so forward and backward never share transients
        dh.dh_layer_bwd(self.layer, s.bwd_args, self.ws.data_ptr() + self.fwd_ws_bytes,
                        self.ws_bytes - self.fwd_ws_bytes, stream)

    def si_step(self, alpha, beta, plan, s_alpha, s_beta, s_comm=None):
        dh.dh_si_step(self.layer, alpha.fwd_args, beta.bwd_args, plan, self.ws, self.ws_bytes, s_alpha, s_beta, s_comm)
