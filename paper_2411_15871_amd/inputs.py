"""Seeded synthetic inputs for the Strand-Interleaving layer step.

This module only draws random numbers and rounds them to a storage type; it holds none of
the method's arithmetic and is shared by the tests' oracle side and GPU side so that both
see bit-identical inputs.

Recipe (the paper trains on unspecified token streams and reports throughput only, so all
inputs are synthetic): weights and biases ~ N(0, 0.02), norm gains 1 + N(0, 0.02), layer inputs
~ N(0, 1), upstream gradients ~ N(0, 1e-2), frozen peer partials ~ N(0, 1e-2) (peer shards entering a
forward all-gather are normalised activations, ~ N(0, 1)), router logits ~ N(0, 1).  Values are drawn in float64 from numpy's Philox generator, cast to float32 and, for
the bf16 configurations, rounded to the nearest-even bf16 value (still held as float32).
"""
import numpy as np

SEED_WEIGHTS = 42
SEED_ALPHA = 0
SEED_BETA = 1
SEED_PEER_FWD = 100
SEED_PEER_BWD = 200
SEED_ROUTER = 7


def round_bf16(a):
    """Round float32 values to the nearest bf16 (ties to even); result stays float32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    r = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + r) & np.uint32(0xFFFF0000)).view(np.float32)


def normal(seed, shape, std=1.0, mean=0.0, bf16=False):
    g = np.random.Generator(np.random.Philox(seed))
    a = (mean + std * g.standard_normal(shape)).astype(np.float32)
    return round_bf16(a) if bf16 else a


def llama_weights(H, n_qkv, n_o, F, bf16, seed=SEED_WEIGHTS):
    """Weights of one Llama-style layer shard, stored [in, out]."""
    return {
        "g1": normal(seed + 0, (H,), 0.02, 1.0, bf16),
        "Wqkv": normal(seed + 1, (H, n_qkv), 0.02, 0.0, bf16),
        "Wo": normal(seed + 2, (n_o, H), 0.02, 0.0, bf16),
        "g2": normal(seed + 3, (H,), 0.02, 1.0, bf16),
        "Wgu": normal(seed + 4, (H, 2 * F), 0.02, 0.0, bf16),
        "Wd": normal(seed + 5, (F, H), 0.02, 0.0, bf16),
    }


def gpt_weights(H, n_qkv, n_o, F, bf16, seed=SEED_WEIGHTS):
    """Weights of one GPT-style layer shard: LayerNorm gains/shifts, two-matrix GeLU MLP (Wgu = first matrix [H,F],
    Wd = second [F,H]) and a bias per linear."""
    return {
        "g1": normal(seed + 0, (H,), 0.02, 1.0, bf16), "b1": normal(seed + 6, (H,), 0.02, 0.0, bf16),
        "Wqkv": normal(seed + 1, (H, n_qkv), 0.02, 0.0, bf16), "bqkv": normal(seed + 7, (n_qkv,), 0.02, 0.0, bf16),
        "Wo": normal(seed + 2, (n_o, H), 0.02, 0.0, bf16), "bo": normal(seed + 8, (H,), 0.02, 0.0, bf16),
        "g2": normal(seed + 3, (H,), 0.02, 1.0, bf16), "b2": normal(seed + 9, (H,), 0.02, 0.0, bf16),
        "Wgu": normal(seed + 4, (H, F), 0.02, 0.0, bf16), "bfc1": normal(seed + 10, (F,), 0.02, 0.0, bf16),
        "Wd": normal(seed + 5, (F, H), 0.02, 0.0, bf16), "bfc2": normal(seed + 11, (H,), 0.02, 0.0, bf16),
    }


def moe_weights(H, n_qkv, n_o, F, n_local, bf16, seed=SEED_WEIGHTS):
    """Weights of one MoE layer share: attention as the Llama layer, n_local SwiGLU experts."""
    w = llama_weights(H, n_qkv, n_o, 8, bf16, seed)
    w["Wgu"] = normal(seed + 4, (n_local, H, 2 * F), 0.02, 0.0, bf16)
    w["Wd"] = normal(seed + 5, (n_local, F, H), 0.02, 0.0, bf16)
    return w


def strand_input(seed, T, H, bf16):
    return normal(1000 + seed, (T, H), 1.0, 0.0, bf16)


def strand_upstream_grad(seed, T, H, bf16):
    return normal(2000 + seed, (T, H), 1e-2, 0.0, bf16)


def peer_partials(seed_base, n_peers, T, H, bf16, std=1e-2):
    """Frozen contributions of the other ranks of a collective: [n_peers, T, H]."""
    if n_peers == 0:
        return np.zeros((0, T, H), dtype=np.float32)
    return np.stack([normal(seed_base + r, (T, H), std, 0.0, bf16) for r in range(1, n_peers + 1)])


def router_logits(T, E, seed=SEED_ROUTER):
    """Router logits [T, E], float32 whatever the activation type (an input of the MoE layer)."""
    return normal(seed, (T, E), 1.0, 0.0, False)
