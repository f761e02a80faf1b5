"""Plain fp64 reference of one transformer layer's forward and backward pass.

TEST INFRASTRUCTURE ONLY -- never imported by the product path.

Strand Interleaving does not change what is computed (paper Sec. 6.1, "Metrics":
training semantics are unmodified; Sec. 4.2: the two strands have no data
dependence), so what a strand must produce is the plain definition of a pre-norm
transformer layer (the operators of Table 2: GEMM, FlashAttention, LayerNorm,
fused bias-dropout-add with p=0, and the collectives, which on one GPU become
fixed-order sums with frozen peer partials) and its exact chain-rule backward.
Every function below writes that definition out with numpy in float64.  numpy's
matmul is the only library primitive used as a step; there is no tiling, fusion or
reordering.

Conventions (readings of points the paper leaves open; listed in the design notes):
  * weights are stored [in, out]; y = x @ W
  * qkv columns are [q heads | k heads | v heads], head-major, head_dim minor
  * gate/up columns are [gate F | up F]
  * RoPE pairs element i with i + d/2 ("rotate-half"), theta_i = base**(-2i/d),
    position restarts at 0 for every sequence
  * attention is causal; q head h reads kv head h // (nq // nkv)
  * a stand-in "collective" = partial 0 (this shard's GEMM output) + frozen peer
    partials, summed in index order
"""
from dataclasses import dataclass
import numpy as np


@dataclass
class LayerCfg:
    batch: int
    seq: int
    H: int
    nq: int
    nkv: int
    d: int
    F: int
    eps: float = 1e-5
    rope_base: float = 10000.0
    rope_pairing: int = 0   # 0: pair (i, i + d/2), 1: pair (2i, 2i + 1)
    gelu_form: int = 0      # 0: tanh form, 1: erf form

    @property
    def T(self):
        return self.batch * self.seq

    @property
    def n_qkv(self):
        return (self.nq + 2 * self.nkv) * self.d


# --------------------------------------------------------------------------- norms
def rmsnorm_fwd(x, gamma, eps):
    """h = gamma * x * rstd, rstd = (mean_j x_j^2 + eps)^(-1/2)  (LayerNorm base of Table 2,
    RMS form used by the Llama models of Sec. 6.1)."""
    rstd = 1.0 / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps)
    return gamma * x * rstd, rstd


def rmsnorm_bwd(dy, x, gamma, rstd):
    """Closed-form backward of rmsnorm_fwd: with xh = x*rstd, gh = gamma*dy,
    dx = rstd * (gh - xh * mean_j(gh*xh)); dgamma = sum_t dy*xh."""
    xh = x * rstd
    gh = gamma * dy
    dx = rstd * (gh - xh * np.mean(gh * xh, axis=-1, keepdims=True))
    dgamma = np.sum(dy * xh, axis=0)
    return dx, dgamma


def layernorm_fwd(x, gamma, beta, eps):
    """h = gamma * (x - mu) * rstd + beta with biased variance (LayerNorm of Table 2)."""
    mu = np.mean(x, axis=-1, keepdims=True)
    xc = x - mu
    rstd = 1.0 / np.sqrt(np.mean(xc * xc, axis=-1, keepdims=True) + eps)
    return gamma * xc * rstd + beta, mu, rstd


def layernorm_bwd(dy, x, gamma, mu, rstd):
    """dx = rstd * (gh - mean(gh) - xh*mean(gh*xh)); dgamma = sum dy*xh; dbeta = sum dy."""
    xh = (x - mu) * rstd
    gh = gamma * dy
    dx = rstd * (gh - np.mean(gh, axis=-1, keepdims=True)
                 - xh * np.mean(gh * xh, axis=-1, keepdims=True))
    return dx, np.sum(dy * xh, axis=0), np.sum(dy, axis=0)


# --------------------------------------------------------------------------- RoPE
def rope(t, seq, base, inverse=False, pos0=0, pairing=0):
    """Rotate head vectors t[T, nh, d] (T = batch*seq, sequence-major) by position*theta.

    Pair i at position p turns by angle p*base**(-2i/d); inverse=True turns by the
    negative angle, which is the backward of the forward rotation (a rotation's transpose).
    pairing 0: pair i is elements (i, i+d/2); pairing 1: elements (2i, 2i+1).
    pos0: position of each sequence's first row (a context-parallel rank holds a later chunk).
    """
    T, nh, d = t.shape
    half = d // 2
    pos = (pos0 + np.arange(T) % seq).astype(np.float64)
    theta = base ** (-2.0 * np.arange(half, dtype=np.float64) / d)
    ang = pos[:, None] * theta[None, :]
    c = np.cos(ang)[:, None, :]
    s = np.sin(ang)[:, None, :]
    if inverse:
        s = -s
    if pairing == 1:
        out = np.empty_like(t, dtype=np.float64)
        a = t[..., 0::2]
        b = t[..., 1::2]
        out[..., 0::2] = a * c - b * s
        out[..., 1::2] = a * s + b * c
        return out
    a = t[..., :half]
    b = t[..., half:]
    return np.concatenate([a * c - b * s, a * s + b * c], axis=-1)


# --------------------------------------------------------------------------- attention
def attention_fwd(q, k, v, batch, seq):
    """Causal softmax attention with grouped KV heads (FlashAttention base of Table 2 computes
    exactly this).  q[T,nq,d], k,v[T,nkv,d] -> o[T,nq,d], lse[nq,T] (natural-log sum-exp of the
    scaled, masked scores)."""
    T, nq, d = q.shape
    nkv = k.shape[1]
    g = nq // nkv
    scale = 1.0 / np.sqrt(d)
    o = np.zeros_like(q)
    lse = np.zeros((nq, T))
    future = np.triu(np.ones((seq, seq), dtype=bool), 1)
    for b in range(batch):
        sl = slice(b * seq, (b + 1) * seq)
        for h in range(nq):
            S = (q[sl, h, :] @ k[sl, h // g, :].T) * scale
            S[future] = -np.inf
            m = np.max(S, axis=1, keepdims=True)
            E = np.exp(S - m)
            Z = np.sum(E, axis=1, keepdims=True)
            o[sl, h, :] = (E / Z) @ v[sl, h // g, :]
            lse[h, sl] = (m + np.log(Z))[:, 0]
    return o, lse


def attention_bwd(do, q, k, v, batch, seq):
    """Chain rule of attention_fwd.  P is recomputed; dV = P^T dO, dP = dO V^T,
    dS = P * (dP - rowsum(dP*P)), dQ = dS K * scale, dK = dS^T Q * scale; dK,dV of a kv head
    sum over the q heads that read it."""
    T, nq, d = q.shape
    nkv = k.shape[1]
    g = nq // nkv
    scale = 1.0 / np.sqrt(d)
    dq = np.zeros_like(q)
    dk = np.zeros_like(k)
    dv = np.zeros_like(v)
    future = np.triu(np.ones((seq, seq), dtype=bool), 1)
    for b in range(batch):
        sl = slice(b * seq, (b + 1) * seq)
        for h in range(nq):
            hk = h // g
            S = (q[sl, h, :] @ k[sl, hk, :].T) * scale
            S[future] = -np.inf
            E = np.exp(S - np.max(S, axis=1, keepdims=True))
            P = E / np.sum(E, axis=1, keepdims=True)
            dO = do[sl, h, :]
            dv[sl, hk, :] += P.T @ dO
            dP = dO @ v[sl, hk, :].T
            dS = P * (dP - np.sum(dP * P, axis=1, keepdims=True))
            dq[sl, h, :] = (dS @ k[sl, hk, :]) * scale
            dk[sl, hk, :] += (dS.T @ q[sl, h, :]) * scale
    return dq, dk, dv


# --------------------------------------------------------------------------- activations
def sigmoid(x):
    return 1.0 / (1.0 + np.exp(-x))


def swiglu_fwd(g, u):
    """a = silu(g) * u, silu(g) = g * sigmoid(g)."""
    return g * sigmoid(g) * u


def swiglu_bwd(da, g, u):
    """dg = da*u*sig*(1 + g*(1-sig)), du = da*g*sig."""
    s = sigmoid(g)
    return da * u * s * (1.0 + g * (1.0 - s)), da * g * s


try:  # the error function as a library primitive
    from scipy.special import erf as _erf
except ImportError:  # pragma: no cover
    import math
    _erf = np.vectorize(math.erf, otypes=[np.float64])
_K0 = np.sqrt(2.0 / np.pi)
_K1 = 0.044715


def gelu_fwd(x, form=0):
    """GeLU.  form 0, tanh form: 0.5 x (1 + tanh(sqrt(2/pi) (x + 0.044715 x^3)));
    form 1, erf form: x Phi(x) = 0.5 x (1 + erf(x / sqrt 2))."""
    if form == 1:
        return 0.5 * x * (1.0 + _erf(x / np.sqrt(2.0)))
    return 0.5 * x * (1.0 + np.tanh(_K0 * (x + _K1 * x ** 3)))


def gelu_bwd(dy, x, form=0):
    if form == 1:  # d/dx [x Phi(x)] = Phi(x) + x phi(x)
        return dy * (0.5 * (1.0 + _erf(x / np.sqrt(2.0))) + x * np.exp(-0.5 * x * x) / np.sqrt(2.0 * np.pi))
    t = np.tanh(_K0 * (x + _K1 * x ** 3))
    return dy * (0.5 * (1.0 + t) + 0.5 * x * (1.0 - t * t) * _K0 * (1.0 + 3.0 * _K1 * x * x))


# --------------------------------------------------------------------------- stand-in
def standin_sum(own, peers):
    """One-GPU stand-in of a tensor-parallel all-reduce (Sec. 2.1, "Collective Communication"):
    own partial plus the frozen peer partials, added in index order."""
    acc = np.array(own, dtype=np.float64, copy=True)
    if peers is not None:
        for r in range(len(peers)):
            acc += peers[r].astype(np.float64)
    return acc


# --------------------------------------------------------------------------- Llama-style layer
def llama_fwd(cfg, W, x, peers=None):
    """Forward of one pre-norm Llama-style layer shard.  Returns (out, saved dict).

    W: g1[H], Wqkv[H,n_qkv], Wo[nq*d,H], g2[H], Wgu[H,2F], Wd[F,H].
    peers: optional dict 'ar1','ar2' -> [R-1,T,H] frozen partials of the two forward collectives.
    """
    peers = peers or {}
    T, nq, nkv, d, F = cfg.T, cfg.nq, cfg.nkv, cfg.d, cfg.F
    h1, r1 = rmsnorm_fwd(x, W["g1"], cfg.eps)
    qkv = h1 @ W["Wqkv"]
    q = qkv[:, : nq * d].reshape(T, nq, d)
    k = qkv[:, nq * d: (nq + nkv) * d].reshape(T, nkv, d)
    v = qkv[:, (nq + nkv) * d:].reshape(T, nkv, d)
    q = rope(q, cfg.seq, cfg.rope_base, pairing=cfg.rope_pairing)
    k = rope(k, cfg.seq, cfg.rope_base, pairing=cfg.rope_pairing)
    o, lse = attention_fwd(q, k, v, cfg.batch, cfg.seq)
    o2 = o.reshape(T, nq * d)
    y = standin_sum(o2 @ W["Wo"], peers.get("ar1"))
    x2 = x + y
    h2, r2 = rmsnorm_fwd(x2, W["g2"], cfg.eps)
    gu = h2 @ W["Wgu"]
    g, u = gu[:, :F], gu[:, F:]
    a = swiglu_fwd(g, u)
    z = standin_sum(a @ W["Wd"], peers.get("ar2"))
    out = x2 + z
    saved = dict(x=x, r1=r1, h1=h1, q=q, k=k, v=v, o=o2, lse=lse, x2=x2, r2=r2, h2=h2, g=g, u=u, a=a)
    return out, saved


def llama_bwd(cfg, W, saved, dout, peers=None):
    """Backward of llama_fwd.  Returns (dx, grads) where grads holds dWqkv, dWo, dWgu, dWd, dg1, dg2
    (the increments that are added to the shared gradient buffers).
    peers: optional 'ar3','ar4' -> frozen partials of the two backward collectives."""
    peers = peers or {}
    T, nq, nkv, d, F = cfg.T, cfg.nq, cfg.nkv, cfg.d, cfg.F
    s = saved
    da = dout @ W["Wd"].T
    dWd = s["a"].T @ dout
    dg, du = swiglu_bwd(da, s["g"], s["u"])
    dgu = np.concatenate([dg, du], axis=1)
    dWgu = s["h2"].T @ dgu
    dh2 = standin_sum(dgu @ W["Wgu"].T, peers.get("ar3"))
    dx2n, dg2 = rmsnorm_bwd(dh2, s["x2"], W["g2"], s["r2"])
    dx2 = dout + dx2n
    do = dx2 @ W["Wo"].T
    dWo = s["o"].T @ dx2
    dq, dk, dv = attention_bwd(do.reshape(T, nq, d), s["q"], s["k"], s["v"], cfg.batch, cfg.seq)
    dq = rope(dq, cfg.seq, cfg.rope_base, inverse=True, pairing=cfg.rope_pairing)
    dk = rope(dk, cfg.seq, cfg.rope_base, inverse=True, pairing=cfg.rope_pairing)
    dqkv = np.concatenate([dq.reshape(T, -1), dk.reshape(T, -1), dv.reshape(T, -1)], axis=1)
    dWqkv = s["h1"].T @ dqkv
    dh1 = standin_sum(dqkv @ W["Wqkv"].T, peers.get("ar4"))
    dxn, dg1 = rmsnorm_bwd(dh1, s["x"], W["g1"], s["r1"])
    dx = dx2 + dxn
    grads = dict(dWqkv=dWqkv, dWo=dWo, dWgu=dWgu, dWd=dWd, dg1=dg1, dg2=dg2)
    inter = dict(da=da, dgu=dgu, dh2=dh2, dx2=dx2, do=do, dqkv=dqkv, dh1=dh1)
    return dx, grads, inter


# --------------------------------------------------------------------------- MoE (top-2, Sec. 6.1 "LLM/MoE Models")
def router_top2(logits):
    """Top-2 gate: softmax over the experts, keep the two largest (ties: lower expert id first), renormalise
    the two kept probabilities to sum 1 (= softmax over the two kept logits).  logits[T,E] ->
    idx[T,2] (descending logit), prob[T,2]."""
    T, E = logits.shape
    idx = np.zeros((T, 2), dtype=np.int64)
    prob = np.zeros((T, 2))
    for t in range(T):
        order = sorted(range(E), key=lambda e: (-logits[t, e], e))
        i, j = order[0], order[1]
        ei, ej = np.exp(logits[t, i] - logits[t, i]), np.exp(logits[t, j] - logits[t, i])
        idx[t] = (i, j)
        prob[t] = (ei / (ei + ej), ej / (ei + ej))
    return idx, prob


def router_top2_bwd(dprob, idx, prob, E):
    """Gradient w.r.t. the logits; only the two selected logits receive any."""
    T = idx.shape[0]
    dl = np.zeros((T, E))
    s = np.sum(dprob * prob, axis=1)
    for k in range(2):
        dl[np.arange(T), idx[:, k]] = prob[:, k] * (dprob[:, k] - s)
    return dl


def permute_rows(idx, E):
    """Stable grouping of the 2T (token, k) assignments by expert id: row order = expert ascending, then
    token ascending, then k.  Returns dest[T,2] (row of each assignment), src_tok[2T], counts[E]."""
    T = idx.shape[0]
    keys = [(int(idx[t, k]), t, k) for t in range(T) for k in range(2)]
    keys.sort()
    dest = np.zeros((T, 2), dtype=np.int64)
    src = np.zeros(2 * T, dtype=np.int64)
    counts = np.zeros(E, dtype=np.int64)
    for row, (e, t, k) in enumerate(keys):
        dest[t, k] = row
        src[row] = t
        counts[e] += 1
    return dest, src, counts


def a2a_dispatch_order(counts, n_local):
    """One-GPU stand-in of the expert-parallel all-to-all: the send buffer is ordered by logical expert
    e = src_rank*n_local + local_expert; the receive buffer is ordered [local_expert][src_rank].  Returns for
    every receive row the send row it copies (a permutation), and the rows per local expert."""
    E = len(counts)
    start = np.concatenate([[0], np.cumsum(counts)])
    rows = []
    group_rows = []
    for le in range(n_local):
        n = 0
        for src in range(E // n_local):
            e = src * n_local + le
            rows.extend(range(start[e], start[e + 1]))
            n += counts[e]
        group_rows.append(n)
    return np.array(rows, dtype=np.int64), group_rows


def moe_ffn_fwd(h2, logits, Wgu, Wd, n_local):
    """Weight-tied MoE block: y_t = sum_k p_tk * FFN_{e_k % n_local}(h2_t), FFN = SwiGLU MLP.
    Wgu[n_local,H,2F], Wd[n_local,F,H].  Goes through the same data movement as the GPU path
    (permute, dispatch, per-expert FFN, combine, weighted un-permute) so intermediates can be compared."""
    T, H = h2.shape
    E = logits.shape[1]
    F = Wd.shape[1]
    idx, prob = router_top2(logits)
    dest, src, counts = permute_rows(idx, E)
    xp = h2[src]                              # permute
    order, group_rows = a2a_dispatch_order(counts, n_local)
    xg = xp[order]                            # all-to-all dispatch
    yg = np.zeros_like(xg)
    gu = np.zeros((2 * T, 2 * F))
    r0 = 0
    for le in range(n_local):
        r1 = r0 + group_rows[le]
        gu[r0:r1] = xg[r0:r1] @ Wgu[le]
        yg[r0:r1] = swiglu_fwd(gu[r0:r1, :F], gu[r0:r1, F:]) @ Wd[le]
        r0 = r1
    yp = np.zeros_like(yg)
    yp[order] = yg                            # all-to-all combine
    y = prob[:, 0:1] * yp[dest[:, 0]] + prob[:, 1:2] * yp[dest[:, 1]]
    saved = dict(idx=idx, prob=prob, dest=dest, src=src, counts=counts, order=order, group_rows=group_rows,
                 xg=xg, gu=gu, yp=yp)
    return y, saved


def moe_ffn_bwd(dy, h2, Wgu, Wd, saved, n_local):
    """Backward of moe_ffn_fwd: returns dh2, dlogits, dWgu, dWd."""
    T, H = h2.shape
    F = Wd.shape[1]
    s = saved
    E = len(s["counts"])
    dprob = np.stack([np.sum(dy * s["yp"][s["dest"][:, k]], axis=1) for k in range(2)], axis=1)
    dyp = np.zeros_like(s["yp"])
    for k in range(2):
        dyp[s["dest"][:, k]] = s["prob"][:, k:k + 1] * dy
    dyg = dyp[s["order"]]
    dxg = np.zeros_like(dyg)
    dWgu = np.zeros_like(Wgu)
    dWd = np.zeros_like(Wd)
    r0 = 0
    for le in range(n_local):
        r1 = r0 + s["group_rows"][le]
        g, u = s["gu"][r0:r1, :F], s["gu"][r0:r1, F:]
        a = swiglu_fwd(g, u)
        da = dyg[r0:r1] @ Wd[le].T
        dWd[le] = a.T @ dyg[r0:r1]
        dg, du = swiglu_bwd(da, g, u)
        dgu = np.concatenate([dg, du], axis=1)
        dWgu[le] = s["xg"][r0:r1].T @ dgu
        dxg[r0:r1] = dgu @ Wgu[le].T
        r0 = r1
    dxp = np.zeros_like(dxg)
    dxp[s["order"]] = dxg
    dh2 = dxp[s["dest"][:, 0]] + dxp[s["dest"][:, 1]]
    dlogits = router_top2_bwd(dprob, s["idx"], s["prob"], E)
    return dh2, dlogits, dWgu, dWd


# --------------------------------------------------------------------------- GPT-style layer with sequence parallelism
def allgather_standin(own, peers):
    """One-GPU stand-in of a sequence-parallel all-gather (Sec. 2.1): this rank's rows first, then the frozen
    peer shards in rank order.  own[Ts,H], peers[R-1,Ts,H] -> [R*Ts,H]."""
    parts = [np.asarray(own, dtype=np.float64)]
    if peers is not None:
        parts += [peers[r].astype(np.float64) for r in range(len(peers))]
    return np.concatenate(parts, axis=0)


def reducescatter_standin(part, peers):
    """Stand-in of the reduce-scatter: this rank's row slice (the first Ts rows) of the sum over ranks.  part[T,H] is
    this rank's full partial, peers[R-1,Ts,H] the other ranks' partials restricted to this rank's slice."""
    Ts = part.shape[0] if peers is None else peers.shape[1]
    return standin_sum(part[:Ts], peers)


def gpt_fwd(cfg, W, x_s, peers=None):
    """Forward of one pre-norm GPT-style layer shard under tensor + sequence parallelism (Sec. 2.1): LayerNorm on
    the sequence shard, all-gather, column-parallel GEMM (+bias), causal attention without rotary embedding,
    row-parallel GEMM, reduce-scatter, bias + residual; the same for the GeLU MLP.
    x_s[Ts,H] with Ts = T / R.  W: g1,b1[H], Wqkv[H,n_qkv], bqkv[n_qkv], Wo[nq*d,H], bo[H], g2,b2[H], W1[H,F],
    bf1[F], W2[F,H], bf2[H].  peers: 'ag1','ag2' [R-1,Ts,H] (peer LayerNorm outputs), 'rs1','rs2' [R-1,Ts,H]."""
    peers = peers or {}
    T, nq, nkv, d = cfg.T, cfg.nq, cfg.nkv, cfg.d
    h1_s, mu1, r1 = layernorm_fwd(x_s, W["g1"], W["b1"], cfg.eps)
    h1 = allgather_standin(h1_s, peers.get("ag1"))
    qkv = h1 @ W["Wqkv"] + W["bqkv"]
    q = qkv[:, : nq * d].reshape(T, nq, d)
    k = qkv[:, nq * d: (nq + nkv) * d].reshape(T, nkv, d)
    v = qkv[:, (nq + nkv) * d:].reshape(T, nkv, d)
    o, lse = attention_fwd(q, k, v, cfg.batch, cfg.seq)
    o2 = o.reshape(T, nq * d)
    y_s = reducescatter_standin(o2 @ W["Wo"], peers.get("rs1"))
    x2_s = x_s + y_s + W["bo"]
    h2_s, mu2, r2 = layernorm_fwd(x2_s, W["g2"], W["b2"], cfg.eps)
    h2 = allgather_standin(h2_s, peers.get("ag2"))
    f = h2 @ W["W1"] + W["bf1"]
    a = gelu_fwd(f, cfg.gelu_form)
    z_s = reducescatter_standin(a @ W["W2"], peers.get("rs2"))
    out_s = x2_s + z_s + W["bf2"]
    saved = dict(x=x_s, mu1=mu1, r1=r1, h1=h1, q=q, k=k, v=v, o=o2, lse=lse, x2=x2_s, mu2=mu2, r2=r2, h2=h2, f=f, a=a)
    return out_s, saved


def gpt_bwd(cfg, W, saved, dout_s, peers=None):
    """Backward of gpt_fwd: every all-gather turns into a reduce-scatter and vice versa (Sec. 2.1).
    peers: 'ag3','ag4' [R-1,Ts,H] = the peers' gradient shards entering the two backward all-gathers,
    'rs3','rs4' [R-1,Ts,H] = the peers' partial gradients for this rank's rows.  Weight and bias gradients of
    the sharded linears sum over all T rows; LayerNorm and row-parallel-bias gradients over this rank's rows."""
    peers = peers or {}
    T, nq, nkv, d = cfg.T, cfg.nq, cfg.nkv, cfg.d
    s = saved
    Ts = dout_s.shape[0]
    dbf2 = dout_s.sum(axis=0)
    dz = allgather_standin(dout_s, peers.get("ag3"))
    da = dz @ W["W2"].T
    dW2 = s["a"].T @ dz
    df = gelu_bwd(da, s["f"], cfg.gelu_form)
    dbf1 = df.sum(axis=0)
    dW1 = s["h2"].T @ df
    dh2_s = reducescatter_standin(df @ W["W1"].T, peers.get("rs3"))
    dx2n, dg2, db2 = layernorm_bwd(dh2_s, s["x2"], W["g2"], s["mu2"], s["r2"])
    dx2_s = dout_s + dx2n
    dbo = dx2_s.sum(axis=0)
    dy = allgather_standin(dx2_s, peers.get("ag4"))
    do = dy @ W["Wo"].T
    dWo = s["o"].T @ dy
    dq, dk, dv = attention_bwd(do.reshape(T, nq, d), s["q"], s["k"], s["v"], cfg.batch, cfg.seq)
    dqkv = np.concatenate([dq.reshape(T, -1), dk.reshape(T, -1), dv.reshape(T, -1)], axis=1)
    dbqkv = dqkv.sum(axis=0)
    dWqkv = s["h1"].T @ dqkv
    dh1_s = reducescatter_standin(dqkv @ W["Wqkv"].T, peers.get("rs4"))
    dxn, dg1, db1 = layernorm_bwd(dh1_s, s["x"], W["g1"], s["mu1"], s["r1"])
    dx_s = dx2_s + dxn
    grads = dict(dWqkv=dWqkv, dbqkv=dbqkv, dWo=dWo, dbo=dbo, dW1=dW1, dbf1=dbf1, dW2=dW2, dbf2=dbf2,
                 dg1=dg1, db1=db1, dg2=dg2, db2=db2)
    inter = dict(dz=dz, da=da, df=df, dh2=dh2_s, dx2=dx2_s, do=do, dqkv=dqkv, dh1=dh1_s)
    assert dx_s.shape[0] == Ts
    return dx_s, grads, inter


# --------------------------------------------------------------------------- MoE layer (attention + expert-parallel FFN)
def moe_layer_fwd(cfg, W, x, logits, n_local):
    """Forward of a pre-norm layer whose FFN is the top-2 MoE block above; attention is not sharded (expert
    parallelism lives inside data parallelism, Sec. 2.1), so the only communication is the two all-to-alls.
    W: g1, Wqkv, Wo, g2, Wgu[n_local,H,2F], Wd[n_local,F,H].  logits[T,E] are an input."""
    T, nq, nkv, d = cfg.T, cfg.nq, cfg.nkv, cfg.d
    h1, r1 = rmsnorm_fwd(x, W["g1"], cfg.eps)
    qkv = h1 @ W["Wqkv"]
    q = rope(qkv[:, : nq * d].reshape(T, nq, d), cfg.seq, cfg.rope_base, pairing=cfg.rope_pairing)
    k = rope(qkv[:, nq * d: (nq + nkv) * d].reshape(T, nkv, d), cfg.seq, cfg.rope_base, pairing=cfg.rope_pairing)
    v = qkv[:, (nq + nkv) * d:].reshape(T, nkv, d)
    o, lse = attention_fwd(q, k, v, cfg.batch, cfg.seq)
    o2 = o.reshape(T, nq * d)
    x2 = x + o2 @ W["Wo"]
    h2, r2 = rmsnorm_fwd(x2, W["g2"], cfg.eps)
    m, msaved = moe_ffn_fwd(h2, logits, W["Wgu"], W["Wd"], n_local)
    out = x2 + m
    saved = dict(x=x, r1=r1, h1=h1, q=q, k=k, v=v, o=o2, lse=lse, x2=x2, r2=r2, h2=h2, moe=msaved)
    return out, saved


def moe_layer_bwd(cfg, W, saved, dout, n_local):
    """Backward of moe_layer_fwd; dlogits is an output next to dx and the weight gradients."""
    T, nq, nkv, d = cfg.T, cfg.nq, cfg.nkv, cfg.d
    s = saved
    dh2, dlogits, dWgu, dWd = moe_ffn_bwd(dout, s["h2"], W["Wgu"], W["Wd"], s["moe"], n_local)
    dx2n, dg2 = rmsnorm_bwd(dh2, s["x2"], W["g2"], s["r2"])
    dx2 = dout + dx2n
    do = dx2 @ W["Wo"].T
    dWo = s["o"].T @ dx2
    dq, dk, dv = attention_bwd(do.reshape(T, nq, d), s["q"], s["k"], s["v"], cfg.batch, cfg.seq)
    dq = rope(dq, cfg.seq, cfg.rope_base, inverse=True, pairing=cfg.rope_pairing)
    dk = rope(dk, cfg.seq, cfg.rope_base, inverse=True, pairing=cfg.rope_pairing)
    dqkv = np.concatenate([dq.reshape(T, -1), dk.reshape(T, -1), dv.reshape(T, -1)], axis=1)
    dWqkv = s["h1"].T @ dqkv
    dh1 = dqkv @ W["Wqkv"].T
    dxn, dg1 = rmsnorm_bwd(dh1, s["x"], W["g1"], s["r1"])
    dx = dx2 + dxn
    grads = dict(dWqkv=dWqkv, dWo=dWo, dWgu=dWgu, dWd=dWd, dg1=dg1, dg2=dg2, dlogits=dlogits)
    return dx, grads


# --------------------------------------------------------------------------- context parallelism (Sec. 2.1 "Intra-layer
# parallelism", Sec. 2.1 and 2.3: key/value chunks of the other ranks arrive by Send/Recv, ring-attention style)
def attention_ctx_fwd(q, k, v, batch, s_l, q_off):
    """Attention of a context-parallel rank: its s_l queries per sequence sit at positions q_off..q_off+s_l-1 and
    read the keys/values of positions 0..q_off+s_l-1 (the earlier ranks' chunks followed by its own), causally.
    q[batch*s_l,nq,d], k,v[batch*S,nkv,d] with S = q_off+s_l -> o[batch*s_l,nq,d], lse[nq,batch*s_l]."""
    Tq, nq, d = q.shape
    nkv = k.shape[1]
    g = nq // nkv
    S_all = q_off + s_l
    scale = 1.0 / np.sqrt(d)
    o = np.zeros_like(q)
    lse = np.zeros((nq, Tq))
    future = np.arange(S_all)[None, :] > (q_off + np.arange(s_l))[:, None]
    for b in range(batch):
        ql = slice(b * s_l, (b + 1) * s_l)
        kl = slice(b * S_all, (b + 1) * S_all)
        for h in range(nq):
            S = (q[ql, h, :] @ k[kl, h // g, :].T) * scale
            S[future] = -np.inf
            m = np.max(S, axis=1, keepdims=True)
            E = np.exp(S - m)
            Z = np.sum(E, axis=1, keepdims=True)
            o[ql, h, :] = (E / Z) @ v[kl, h // g, :]
            lse[h, ql] = (m + np.log(Z))[:, 0]
    return o, lse


def attention_ctx_bwd(do, q, k, v, batch, s_l, q_off):
    """Chain rule of attention_ctx_fwd: dq for the rank's own queries, dk/dv for every key row it read
    (rows of earlier chunks are what the rank sends back to their owners)."""
    Tq, nq, d = q.shape
    nkv = k.shape[1]
    g = nq // nkv
    S_all = q_off + s_l
    scale = 1.0 / np.sqrt(d)
    dq = np.zeros_like(q)
    dk = np.zeros_like(k)
    dv = np.zeros_like(v)
    future = np.arange(S_all)[None, :] > (q_off + np.arange(s_l))[:, None]
    for b in range(batch):
        ql = slice(b * s_l, (b + 1) * s_l)
        kl = slice(b * S_all, (b + 1) * S_all)
        for h in range(nq):
            hk = h // g
            S = (q[ql, h, :] @ k[kl, hk, :].T) * scale
            S[future] = -np.inf
            E = np.exp(S - np.max(S, axis=1, keepdims=True))
            P = E / np.sum(E, axis=1, keepdims=True)
            dO = do[ql, h, :]
            dv[kl, hk, :] += P.T @ dO
            dP = dO @ v[kl, hk, :].T
            dS = P * (dP - np.sum(dP * P, axis=1, keepdims=True))
            dq[ql, h, :] = (dS @ k[kl, hk, :]) * scale
            dk[kl, hk, :] += (dS.T @ q[ql, h, :]) * scale
    return dq, dk, dv


def cp_gather_kv(k, v, peer_kv, batch, s_l, cp_rank):
    """Key/value rows a rank attends to, per sequence: chunks 0..cp_rank-1 from the peers, then its own.
    k,v[batch*s_l,nkv,d]; peer_kv[CP-1, batch*s_l, 2*nkv*d] holds the other ranks' chunks ([k heads | v heads], keys
    already rotated), ordered by source rank with this rank left out.  Chunks of later ranks arrive too (the ring
    passes every chunk through every rank) but no causal query reads them."""
    nkv, d = k.shape[1], k.shape[2]
    S_all = (cp_rank + 1) * s_l
    K = np.zeros((batch * S_all, nkv, d))
    V = np.zeros((batch * S_all, nkv, d))
    for b in range(batch):
        for c in range(cp_rank):
            rows = slice(b * S_all + c * s_l, b * S_all + (c + 1) * s_l)
            chunk = peer_kv[c][b * s_l:(b + 1) * s_l].astype(np.float64)
            K[rows] = chunk[:, : nkv * d].reshape(s_l, nkv, d)
            V[rows] = chunk[:, nkv * d:].reshape(s_l, nkv, d)
        own = slice(b * S_all + cp_rank * s_l, (b + 1) * S_all)
        K[own] = k[b * s_l:(b + 1) * s_l]
        V[own] = v[b * s_l:(b + 1) * s_l]
    return K, V


def llama_cp_fwd(cfg, W, x, cp_rank, peers=None):
    """llama_fwd for context-parallel rank cp_rank: cfg.seq is the rank's chunk length, its rows sit at positions
    cp_rank*seq.. of each sequence.  peers: 'ar1','ar2' as llama_fwd, 'kv' -> [CP-1, T, 2*nkv*d] (see cp_gather_kv)."""
    peers = peers or {}
    T, nq, nkv, d, F = cfg.T, cfg.nq, cfg.nkv, cfg.d, cfg.F
    q_off = cp_rank * cfg.seq
    h1, r1 = rmsnorm_fwd(x, W["g1"], cfg.eps)
    qkv = h1 @ W["Wqkv"]
    q = rope(qkv[:, : nq * d].reshape(T, nq, d), cfg.seq, cfg.rope_base, pos0=q_off, pairing=cfg.rope_pairing)
    k = rope(qkv[:, nq * d: (nq + nkv) * d].reshape(T, nkv, d), cfg.seq, cfg.rope_base, pos0=q_off, pairing=cfg.rope_pairing)
    v = qkv[:, (nq + nkv) * d:].reshape(T, nkv, d)
    K, V = cp_gather_kv(k, v, peers.get("kv"), cfg.batch, cfg.seq, cp_rank)
    o, lse = attention_ctx_fwd(q, K, V, cfg.batch, cfg.seq, q_off)
    o2 = o.reshape(T, nq * d)
    y = standin_sum(o2 @ W["Wo"], peers.get("ar1"))
    x2 = x + y
    h2, r2 = rmsnorm_fwd(x2, W["g2"], cfg.eps)
    gu = h2 @ W["Wgu"]
    g, u = gu[:, :F], gu[:, F:]
    a = swiglu_fwd(g, u)
    z = standin_sum(a @ W["Wd"], peers.get("ar2"))
    out = x2 + z
    saved = dict(x=x, r1=r1, h1=h1, q=q, k=k, v=v, K=K, V=V, o=o2, lse=lse, x2=x2, r2=r2, h2=h2, g=g, u=u, a=a)
    return out, saved


def llama_cp_bwd(cfg, W, saved, dout, cp_rank, peers=None):
    """Backward of llama_cp_fwd.  peers: 'ar3','ar4' as llama_bwd; 'dkv' -> [CP-1, T, 2*nkv*d], the other ranks'
    gradient contributions to this rank's own keys/values (same order as 'kv'); only later ranks read this rank's
    keys, so the chunks of ranks > cp_rank are added (index order, after the rank's own contribution).
    Returns (dx, grads, inter); inter['dkv_peers'][c] = [T, 2*nkv*d] is the gradient this rank sends to rank c < cp_rank."""
    peers = peers or {}
    T, nq, nkv, d, F = cfg.T, cfg.nq, cfg.nkv, cfg.d, cfg.F
    s_l, q_off = cfg.seq, cp_rank * cfg.seq
    S_all = q_off + s_l
    s = saved
    da = dout @ W["Wd"].T
    dWd = s["a"].T @ dout
    dg, du = swiglu_bwd(da, s["g"], s["u"])
    dgu = np.concatenate([dg, du], axis=1)
    dWgu = s["h2"].T @ dgu
    dh2 = standin_sum(dgu @ W["Wgu"].T, peers.get("ar3"))
    dx2n, dg2 = rmsnorm_bwd(dh2, s["x2"], W["g2"], s["r2"])
    dx2 = dout + dx2n
    do = dx2 @ W["Wo"].T
    dWo = s["o"].T @ dx2
    dq, dK, dV = attention_ctx_bwd(do.reshape(T, nq, d), s["q"], s["K"], s["V"], cfg.batch, s_l, q_off)
    dk = np.zeros((T, nkv, d))
    dv = np.zeros((T, nkv, d))
    dkv_peers = np.zeros((cp_rank, T, 2 * nkv * d))
    for b in range(cfg.batch):
        own = slice(b * S_all + q_off, (b + 1) * S_all)
        dk[b * s_l:(b + 1) * s_l] = dK[own]
        dv[b * s_l:(b + 1) * s_l] = dV[own]
        for c in range(cp_rank):
            rows = slice(b * S_all + c * s_l, b * S_all + (c + 1) * s_l)
            dkv_peers[c, b * s_l:(b + 1) * s_l, : nkv * d] = dK[rows].reshape(s_l, nkv * d)
            dkv_peers[c, b * s_l:(b + 1) * s_l, nkv * d:] = dV[rows].reshape(s_l, nkv * d)
    dkv_own = np.concatenate([dk.reshape(T, -1), dv.reshape(T, -1)], axis=1)
    if peers.get("dkv") is not None:
        for c in range(cp_rank, len(peers["dkv"])):  # entries cp_rank.. are the ranks after this one
            dkv_own = dkv_own + peers["dkv"][c].astype(np.float64)
    dk = dkv_own[:, : nkv * d].reshape(T, nkv, d)
    dv = dkv_own[:, nkv * d:]
    dq = rope(dq, s_l, cfg.rope_base, inverse=True, pos0=q_off, pairing=cfg.rope_pairing)
    dk = rope(dk, s_l, cfg.rope_base, inverse=True, pos0=q_off, pairing=cfg.rope_pairing)
    dqkv = np.concatenate([dq.reshape(T, -1), dk.reshape(T, -1), dv], axis=1)
    dWqkv = s["h1"].T @ dqkv
    dh1 = standin_sum(dqkv @ W["Wqkv"].T, peers.get("ar4"))
    dxn, dg1 = rmsnorm_bwd(dh1, s["x"], W["g1"], s["r1"])
    dx = dx2 + dxn
    grads = dict(dWqkv=dWqkv, dWo=dWo, dWgu=dWgu, dWd=dWd, dg1=dg1, dg2=dg2)
    inter = dict(da=da, dgu=dgu, dh2=dh2, dx2=dx2, do=do, dqkv=dqkv, dh1=dh1, dkv_peers=dkv_peers, dkv_own=dkv_own)
    return dx, grads, inter
