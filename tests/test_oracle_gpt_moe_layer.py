"""Pins for the GPT-style (tensor + sequence parallel) and MoE layer references in oracle/layer_ref.py.

1. A true R-rank model: the whole unsharded layer is written with torch fp64 operations and differentiated by
   autograd; rank 0's oracle call, fed the other ranks' real contributions as "peer" buffers, must reproduce
   rank 0's slice of the full layer's output, input gradient and sharded weight gradients.  This fixes what
   all-gather / reduce-scatter mean, in both directions.
2. With frozen forward peers and zero backward peers the oracle's backward is the plain gradient of a
   differentiable function; autograd of a torch transcription of the definitions gives every gradient,
   including LayerNorm parameters and the row-parallel biases.
3. The MoE layer against a per-token dense formulation (no permutation, no all-to-all) under autograd.
"""
import math
import numpy as np
import torch

from oracle import layer_ref as R

rng = np.random.default_rng(77)
t64 = lambda a, g=False: torch.tensor(np.asarray(a), dtype=torch.float64, requires_grad=g)


def relerr(a, b):
    return np.linalg.norm(np.asarray(a) - np.asarray(b)) / max(np.linalg.norm(np.asarray(b)), 1e-300)


def t_layernorm(x, g, b, eps):
    mu = x.mean(-1, keepdim=True)
    var = ((x - mu) ** 2).mean(-1, keepdim=True)
    return (x - mu) / torch.sqrt(var + eps) * g + b


def t_attention(q, k, v, batch, seq):
    """q[T,nq,d], k,v[T,nkv,d]; causal softmax attention per sequence, query head h reads kv head h // (nq/nkv)."""
    T, nq, d = q.shape
    nkv = k.shape[1]
    out = []
    mask = torch.tril(torch.ones(seq, seq, dtype=torch.bool))
    for b in range(batch):
        sl = slice(b * seq, (b + 1) * seq)
        heads = []
        for h in range(nq):
            kv = h // (nq // nkv)
            s = q[sl, h] @ k[sl, kv].T / math.sqrt(d)
            s = s.masked_fill(~mask, float("-inf"))
            heads.append(torch.softmax(s, dim=-1) @ v[sl, kv])
        out.append(torch.stack(heads, dim=1))
    return torch.cat(out, dim=0)


def t_rope(x, seq, base):
    T, nh, d = x.shape
    pos = (torch.arange(T) % seq).to(torch.float64)
    theta = base ** (-2.0 * torch.arange(d // 2, dtype=torch.float64) / d)
    ang = pos[:, None] * theta[None, :]
    c, s = torch.cos(ang)[:, None, :], torch.sin(ang)[:, None, :]
    a, b = x[..., : d // 2], x[..., d // 2:]
    return torch.cat([a * c - b * s, a * s + b * c], dim=-1)


def gpt_rank_weights(H, nq, nkv, d, F):
    n_qkv = (nq + 2 * nkv) * d
    return dict(Wqkv=rng.standard_normal((H, n_qkv)) * 0.3, bqkv=rng.standard_normal(n_qkv) * 0.1,
                Wo=rng.standard_normal((nq * d, H)) * 0.3, W1=rng.standard_normal((H, F)) * 0.3,
                bf1=rng.standard_normal(F) * 0.1, W2=rng.standard_normal((F, H)) * 0.3)


def test_gpt_sp_shard_reproduces_rank0_of_a_true_multi_rank_layer():
    Rk, batch, seq, H, nq, nkv, d, F = 4, 2, 8, 12, 2, 1, 4, 10
    T, Ts = batch * seq, batch * seq // Rk
    cfg = R.LayerCfg(batch=batch, seq=seq, H=H, nq=nq, nkv=nkv, d=d, F=F)
    shared = dict(g1=1 + 0.1 * rng.standard_normal(H), b1=0.1 * rng.standard_normal(H), g2=1 + 0.1 * rng.standard_normal(H),
                  b2=0.1 * rng.standard_normal(H), bo=0.1 * rng.standard_normal(H), bf2=0.1 * rng.standard_normal(H))
    ranks = [gpt_rank_weights(H, nq, nkv, d, F) for _ in range(Rk)]
    x = rng.standard_normal((T, H)); dout = rng.standard_normal((T, H)) * 0.1
    # ---- the full layer in torch
    xs = t64(x, True)
    sh = {k: t64(v, True) for k, v in shared.items()}
    rk = [{k: t64(v, True) for k, v in w.items()} for w in ranks]
    h1 = t_layernorm(xs, sh["g1"], sh["b1"], cfg.eps)
    qkv, o_part = [], []
    for w in rk:
        z = h1 @ w["Wqkv"] + w["bqkv"]; z.retain_grad(); qkv.append(z)
        o = t_attention(z[:, : nq * d].reshape(T, nq, d), z[:, nq * d:(nq + nkv) * d].reshape(T, nkv, d),
                        z[:, (nq + nkv) * d:].reshape(T, nkv, d), batch, seq).reshape(T, nq * d)
        o_part.append(o @ w["Wo"])
    x2 = xs + sum(o_part) + sh["bo"]; x2.retain_grad()
    h2 = t_layernorm(x2, sh["g2"], sh["b2"], cfg.eps)
    fs, z_part = [], []
    for w in rk:
        f = h2 @ w["W1"] + w["bf1"]; f.retain_grad(); fs.append(f)
        z_part.append(torch.nn.functional.gelu(f, approximate="tanh") @ w["W2"])
    out = x2 + sum(z_part) + sh["bf2"]
    (out * t64(dout)).sum().backward()
    n = lambda t: t.detach().numpy()
    shard = lambda a, r: a[r * Ts:(r + 1) * Ts]
    peer_shards = lambda a: np.stack([shard(a, r) for r in range(1, Rk)])
    # ---- rank 0 through the oracle
    W0 = dict(shared); W0.update(ranks[0])
    fp = dict(ag1=peer_shards(n(h1)), ag2=peer_shards(n(h2)),
              rs1=np.stack([n(o_part[r])[:Ts] for r in range(1, Rk)]),
              rs2=np.stack([n(z_part[r])[:Ts] for r in range(1, Rk)]))
    out_s, saved = R.gpt_fwd(cfg, W0, x[:Ts], fp)
    assert relerr(out_s, n(out)[:Ts]) < 1e-12
    bp = dict(ag3=peer_shards(dout), ag4=peer_shards(n(x2.grad)),
              rs3=np.stack([(n(fs[r].grad) @ ranks[r]["W1"].T)[:Ts] for r in range(1, Rk)]),
              rs4=np.stack([(n(qkv[r].grad) @ ranks[r]["Wqkv"].T)[:Ts] for r in range(1, Rk)]))
    dx_s, grads, _ = R.gpt_bwd(cfg, W0, saved, dout[:Ts], bp)
    assert relerr(dx_s, n(xs.grad)[:Ts]) < 1e-11
    for name in ("Wqkv", "bqkv", "Wo", "W1", "bf1", "W2"):
        key = "d" + name
        assert relerr(grads[key], n(rk[0][name].grad)) < 1e-11, name


def test_gpt_sp_backward_is_the_gradient_of_the_frozen_peer_function():
    Rk, batch, seq, H, nq, nkv, d, F = 2, 1, 6, 8, 2, 2, 4, 6
    T, Ts = batch * seq, batch * seq // Rk
    cfg = R.LayerCfg(batch=batch, seq=seq, H=H, nq=nq, nkv=nkv, d=d, F=F)
    W = dict(g1=1 + 0.1 * rng.standard_normal(H), b1=0.1 * rng.standard_normal(H), g2=1 + 0.1 * rng.standard_normal(H),
             b2=0.1 * rng.standard_normal(H), bo=0.1 * rng.standard_normal(H), bf2=0.1 * rng.standard_normal(H))
    W.update(gpt_rank_weights(H, nq, nkv, d, F))
    x_s = rng.standard_normal((Ts, H)); dout_s = rng.standard_normal((Ts, H)) * 0.1
    fp = {k: rng.standard_normal((Rk - 1, Ts, H)) * 0.2 for k in ("ag1", "ag2", "rs1", "rs2")}
    out_s, saved = R.gpt_fwd(cfg, W, x_s, fp)
    zero = {k: np.zeros((Rk - 1, Ts, H)) for k in ("ag3", "ag4", "rs3", "rs4")}
    dx_s, grads, _ = R.gpt_bwd(cfg, W, saved, dout_s, zero)
    # torch transcription of the definitions
    tw = {k: t64(v, True) for k, v in W.items()}
    xs = t64(x_s, True)
    cat = lambda own, peers: torch.cat([own] + [t64(p) for p in peers], dim=0)
    h1 = cat(t_layernorm(xs, tw["g1"], tw["b1"], cfg.eps), fp["ag1"])
    z = h1 @ tw["Wqkv"] + tw["bqkv"]
    o = t_attention(z[:, : nq * d].reshape(T, nq, d), z[:, nq * d:(nq + nkv) * d].reshape(T, nkv, d),
                    z[:, (nq + nkv) * d:].reshape(T, nkv, d), batch, seq).reshape(T, nq * d)
    x2 = xs + (o @ tw["Wo"])[:Ts] + t64(fp["rs1"].sum(0)) + tw["bo"]
    h2 = cat(t_layernorm(x2, tw["g2"], tw["b2"], cfg.eps), fp["ag2"])
    a = torch.nn.functional.gelu(h2 @ tw["W1"] + tw["bf1"], approximate="tanh")
    out = x2 + (a @ tw["W2"])[:Ts] + t64(fp["rs2"].sum(0)) + tw["bf2"]
    assert relerr(out_s, out.detach().numpy()) < 1e-12
    (out * t64(dout_s)).sum().backward()
    assert relerr(dx_s, xs.grad.numpy()) < 1e-11
    names = dict(dWqkv="Wqkv", dbqkv="bqkv", dWo="Wo", dbo="bo", dW1="W1", dbf1="bf1", dW2="W2", dbf2="bf2",
                 dg1="g1", db1="b1", dg2="g2", db2="b2")
    for key, name in names.items():
        assert relerr(grads[key], tw[name].grad.numpy()) < 1e-11, key


def test_gpt_sp_backward_peers_enter_linearly():
    Rk, batch, seq, H, nq, nkv, d, F = 2, 1, 4, 8, 1, 1, 4, 6
    Ts = batch * seq // Rk
    cfg = R.LayerCfg(batch=batch, seq=seq, H=H, nq=nq, nkv=nkv, d=d, F=F)
    W = dict(g1=np.ones(H), b1=np.zeros(H), g2=np.ones(H), b2=np.zeros(H), bo=np.zeros(H), bf2=np.zeros(H))
    W.update(gpt_rank_weights(H, nq, nkv, d, F))
    x_s = rng.standard_normal((Ts, H)); dout_s = rng.standard_normal((Ts, H))
    fp = {k: rng.standard_normal((Rk - 1, Ts, H)) for k in ("ag1", "ag2", "rs1", "rs2")}
    _, saved = R.gpt_fwd(cfg, W, x_s, fp)
    bp = {k: rng.standard_normal((Rk - 1, Ts, H)) for k in ("ag3", "ag4", "rs3", "rs4")}
    zero = {k: np.zeros((Rk - 1, Ts, H)) for k in bp}
    full, gf, _ = R.gpt_bwd(cfg, W, saved, dout_s, bp)
    a, ga, _ = R.gpt_bwd(cfg, W, saved, dout_s, zero)
    b, gb, _ = R.gpt_bwd(cfg, W, saved, np.zeros_like(dout_s), bp)
    assert relerr(full, a + b) < 1e-12
    for k in gf:
        assert relerr(gf[k], ga[k] + gb[k]) < 1e-12, k


def test_moe_layer_matches_dense_per_token_autograd():
    batch, seq, H, nq, nkv, d, F, E, n_local = 2, 6, 8, 4, 2, 4, 6, 6, 2
    T = batch * seq
    cfg = R.LayerCfg(batch=batch, seq=seq, H=H, nq=nq, nkv=nkv, d=d, F=F)
    n_qkv = (nq + 2 * nkv) * d
    W = dict(g1=1 + 0.1 * rng.standard_normal(H), g2=1 + 0.1 * rng.standard_normal(H),
             Wqkv=rng.standard_normal((H, n_qkv)) * 0.3, Wo=rng.standard_normal((nq * d, H)) * 0.3,
             Wgu=rng.standard_normal((n_local, H, 2 * F)) * 0.3, Wd=rng.standard_normal((n_local, F, H)) * 0.3)
    x = rng.standard_normal((T, H)); dout = rng.standard_normal((T, H)) * 0.1
    logits = rng.standard_normal((T, E))
    out, saved = R.moe_layer_fwd(cfg, W, x, logits, n_local)
    dx, grads = R.moe_layer_bwd(cfg, W, saved, dout, n_local)
    idx = saved["moe"]["idx"]
    # every token's two experts are its two largest logits
    for t in range(T):
        assert set(idx[t]) == set(np.argsort(-logits[t], kind="stable")[:2])
    tw = {k: t64(v, True) for k, v in W.items()}
    xs, tl = t64(x, True), t64(logits, True)
    rms = lambda v, g: v / torch.sqrt((v * v).mean(-1, keepdim=True) + cfg.eps) * g
    h1 = rms(xs, tw["g1"])
    z = h1 @ tw["Wqkv"]
    q = t_rope(z[:, : nq * d].reshape(T, nq, d), seq, cfg.rope_base)
    k = t_rope(z[:, nq * d:(nq + nkv) * d].reshape(T, nkv, d), seq, cfg.rope_base)
    o = t_attention(q, k, z[:, (nq + nkv) * d:].reshape(T, nkv, d), batch, seq).reshape(T, nq * d)
    x2 = xs + o @ tw["Wo"]
    h2 = rms(x2, tw["g2"])
    rows = []
    for t in range(T):
        p = torch.softmax(tl[t, torch.tensor(idx[t])], dim=0)
        acc = 0
        for kk in range(2):
            le = int(idx[t, kk]) % n_local
            gu = h2[t] @ tw["Wgu"][le]
            acc = acc + p[kk] * ((torch.nn.functional.silu(gu[:F]) * gu[F:]) @ tw["Wd"][le])
        rows.append(acc)
    ref = x2 + torch.stack(rows)
    assert relerr(out, ref.detach().numpy()) < 1e-12
    (ref * t64(dout)).sum().backward()
    assert relerr(dx, xs.grad.numpy()) < 1e-11
    assert relerr(grads["dlogits"], tl.grad.numpy()) < 1e-11
    for key in ("Wqkv", "Wo", "Wgu", "Wd", "g1", "g2"):
        assert relerr(grads["d" + key if key[0] == "W" else "d" + key], tw[key].grad.numpy()) < 1e-11, key
