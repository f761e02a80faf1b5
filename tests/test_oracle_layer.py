"""Pins for oracle/layer_ref.py: finite differences, brute force, closed forms, invariants and an
independent autograd composition.  None of these re-use the oracle's own formulas."""
import math
import numpy as np
import pytest
import torch

from oracle import layer_ref as R

rng = np.random.default_rng(1234)


def fd_grad(f, x, h=1e-6):
    """Central finite differences of scalar f at array x."""
    g = np.zeros_like(x)
    it = np.nditer(x, flags=["multi_index"])
    for _ in it:
        i = it.multi_index
        old = x[i]
        x[i] = old + h
        fp = f()
        x[i] = old - h
        fm = f()
        x[i] = old
        g[i] = (fp - fm) / (2 * h)
    return g


def relerr(a, b):
    return np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300)


# ------------------------------------------------------------------ norms
def test_rmsnorm_forward_definition_by_loops():
    x = rng.standard_normal((3, 5)); g = rng.standard_normal(5)
    h, r = R.rmsnorm_fwd(x, g, 1e-5)
    for t in range(3):
        ms = sum(x[t, j] ** 2 for j in range(5)) / 5
        for j in range(5):
            assert abs(h[t, j] - g[j] * x[t, j] / math.sqrt(ms + 1e-5)) < 1e-13


def test_rmsnorm_bwd_fd_and_projection_identity():
    x = rng.standard_normal((4, 7)); g = rng.standard_normal(7); w = rng.standard_normal((4, 7))
    _, r = R.rmsnorm_fwd(x, g, 1e-5)
    dx, dg = R.rmsnorm_bwd(w, x, g, r)
    f = lambda: float(np.sum(R.rmsnorm_fwd(x, g, 1e-5)[0] * w))
    assert relerr(dx, fd_grad(f, x)) < 1e-7
    assert relerr(dg, fd_grad(f, g)) < 1e-7
    # with eps -> 0 the output is scale invariant in x, so dx is orthogonal to x row by row
    _, r0 = R.rmsnorm_fwd(x, g, 0.0)
    dx0, _ = R.rmsnorm_bwd(w, x, g, r0)
    assert np.max(np.abs(np.sum(dx0 * x, axis=1))) < 1e-12


def test_layernorm_bwd_fd_and_invariants():
    x = rng.standard_normal((4, 6)); g = rng.standard_normal(6); b = rng.standard_normal(6)
    w = rng.standard_normal((4, 6))
    h, mu, r = R.layernorm_fwd(x, g, b, 1e-5)
    # unit gain, zero shift -> zero mean and (almost) unit variance rows
    h1, _, _ = R.layernorm_fwd(x, np.ones(6), np.zeros(6), 0.0)
    assert np.max(np.abs(h1.mean(axis=1))) < 1e-14 and np.max(np.abs(h1.var(axis=1) - 1)) < 1e-12
    dx, dg, db = R.layernorm_bwd(w, x, g, mu, r)
    f = lambda: float(np.sum(R.layernorm_fwd(x, g, b, 1e-5)[0] * w))
    assert relerr(dx, fd_grad(f, x)) < 1e-7
    assert relerr(dg, fd_grad(f, g)) < 1e-7
    assert relerr(db, fd_grad(f, b)) < 1e-7
    assert np.max(np.abs(dx.sum(axis=1))) < 1e-12  # shift invariance


# ------------------------------------------------------------------ RoPE
def test_rope_properties():
    seq, d = 5, 8
    q = rng.standard_normal((2 * seq, 3, d))
    rq = R.rope(q, seq, 10000.0)
    assert np.allclose(np.linalg.norm(rq, axis=-1), np.linalg.norm(q, axis=-1), atol=1e-13)
    assert np.allclose(rq[0], q[0]) and np.allclose(rq[seq], q[seq])       # position 0 of each sequence
    assert np.allclose(R.rope(rq, seq, 10000.0, inverse=True), q, atol=1e-13)
    # relative-position property: <R_m a, R_n b> depends on m-n only
    a = rng.standard_normal(d); b = rng.standard_normal(d)
    A = R.rope(np.tile(a, (seq, 1, 1)), seq, 10000.0)[:, 0]
    B = R.rope(np.tile(b, (seq, 1, 1)), seq, 10000.0)[:, 0]
    assert abs(A[3] @ B[1] - A[4] @ B[2]) < 1e-12 and abs(A[2] @ B[2] - a @ b) < 1e-12


def test_rope_pairing_and_angle_by_hand():
    d, base = 4, 10000.0
    q = np.zeros((3, 1, d)); q[2, 0] = [1.0, 2.0, 3.0, 4.0]
    out = R.rope(q, 3, base)[2, 0]
    th = [1.0, base ** (-2.0 / d)]
    exp = [1 * math.cos(2 * th[0]) - 3 * math.sin(2 * th[0]), 2 * math.cos(2 * th[1]) - 4 * math.sin(2 * th[1]),
           1 * math.sin(2 * th[0]) + 3 * math.cos(2 * th[0]), 2 * math.sin(2 * th[1]) + 4 * math.cos(2 * th[1])]
    assert np.allclose(out, exp, atol=1e-14)


def test_rope_adjacent_pairing():
    """Pairing (2i, 2i+1): by hand on one vector; the same rotation as the half-split pairing seen through the
    permutation that brings element 2i to i and 2i+1 to i + d/2; norm, position 0, inverse and relative position."""
    d, base = 4, 10000.0
    q = np.zeros((3, 1, d)); q[2, 0] = [1.0, 2.0, 3.0, 4.0]
    out = R.rope(q, 3, base, pairing=1)[2, 0]
    th = [1.0, base ** (-2.0 / d)]
    exp = [1 * math.cos(2 * th[0]) - 2 * math.sin(2 * th[0]), 1 * math.sin(2 * th[0]) + 2 * math.cos(2 * th[0]),
           3 * math.cos(2 * th[1]) - 4 * math.sin(2 * th[1]), 3 * math.sin(2 * th[1]) + 4 * math.cos(2 * th[1])]
    assert np.allclose(out, exp, atol=1e-14)
    seq, d = 6, 16
    x = rng.standard_normal((2 * seq, 3, d))
    perm = np.concatenate([np.arange(0, d, 2), np.arange(1, d, 2)])   # halves layout <- adjacent layout
    via_halves = np.empty_like(x)
    via_halves[..., perm] = R.rope(x[..., perm], seq, 500.0, pos0=3)
    got = R.rope(x, seq, 500.0, pos0=3, pairing=1)
    assert np.allclose(got, via_halves, atol=1e-14)
    assert not np.allclose(got, R.rope(x, seq, 500.0, pos0=3))        # and it is a different map on the same layout
    assert np.allclose(np.linalg.norm(got, axis=-1), np.linalg.norm(x, axis=-1), atol=1e-13)
    assert np.allclose(R.rope(x, seq, 500.0, pairing=1)[0], x[0])
    assert np.allclose(R.rope(got, seq, 500.0, inverse=True, pos0=3, pairing=1), x, atol=1e-13)
    a = rng.standard_normal(d); b2 = rng.standard_normal(d)
    A = R.rope(np.tile(a, (seq, 1, 1)), seq, 500.0, pairing=1)[:, 0]
    B = R.rope(np.tile(b2, (seq, 1, 1)), seq, 500.0, pairing=1)[:, 0]
    assert abs(A[3] @ B[1] - A[5] @ B[3]) < 1e-12


# ------------------------------------------------------------------ attention
def brute_attention(q, k, v, batch, seq):
    T, nq, d = q.shape
    g = nq // k.shape[1]
    o = np.zeros_like(q)
    for b in range(batch):
        for h in range(nq):
            for i in range(seq):
                sc = [sum(q[b * seq + i, h, c] * k[b * seq + j, h // g, c] for c in range(d)) / math.sqrt(d)
                      for j in range(i + 1)]
                m = max(sc)
                e = [math.exp(s - m) for s in sc]
                z = sum(e)
                for c in range(d):
                    o[b * seq + i, h, c] = sum(e[j] / z * v[b * seq + j, h // g, c] for j in range(i + 1))
    return o


def test_attention_vs_brute_force_and_invariants():
    batch, seq, nq, nkv, d = 2, 5, 4, 2, 4
    T = batch * seq
    q = rng.standard_normal((T, nq, d)); k = rng.standard_normal((T, nkv, d)); v = rng.standard_normal((T, nkv, d))
    o, lse = R.attention_fwd(q, k, v, batch, seq)
    assert np.max(np.abs(o - brute_attention(q, k, v, batch, seq))) < 1e-13
    # lse normalises the probabilities
    for h in range(nq):
        for i in range(seq):
            s = q[i, h] @ k[: i + 1, h // 2].T / math.sqrt(d)
            assert abs(np.sum(np.exp(s - lse[h, i])) - 1) < 1e-12
    # causality: changing a later token does not change earlier outputs; sequences are independent
    k2 = k.copy(); v2 = v.copy(); k2[3] += 1.0; v2[3] -= 2.0
    o2, _ = R.attention_fwd(q, k2, v2, batch, seq)
    assert np.array_equal(o2[:3], o[:3]) and np.array_equal(o2[seq:], o[seq:])
    assert not np.allclose(o2[3:seq], o[3:seq])
    # first token of a sequence attends to itself only
    assert np.allclose(o[0], np.repeat(v[0], 2, axis=0)) and np.allclose(o[seq], np.repeat(v[seq], 2, axis=0))
    # grouped heads == multi-head attention with repeated kv heads
    om, _ = R.attention_fwd(q, np.repeat(k, 2, axis=1), np.repeat(v, 2, axis=1), batch, seq)
    assert np.allclose(om, o, atol=1e-14)


def test_attention_bwd_fd_and_softmax_rowsum():
    batch, seq, nq, nkv, d = 1, 4, 2, 1, 4
    T = batch * seq
    q = rng.standard_normal((T, nq, d)); k = rng.standard_normal((T, nkv, d)); v = rng.standard_normal((T, nkv, d))
    w = rng.standard_normal((T, nq, d))
    dq, dk, dv = R.attention_bwd(w, q, k, v, batch, seq)
    f = lambda: float(np.sum(R.attention_fwd(q, k, v, batch, seq)[0] * w))
    assert relerr(dq, fd_grad(f, q)) < 1e-7
    assert relerr(dk, fd_grad(f, k)) < 1e-7
    assert relerr(dv, fd_grad(f, v)) < 1e-7
    # adding a constant to all scores of a row leaves softmax unchanged: shifting every key by a
    # vector c adds q.c to each score of a row, so sum_j dk_j must be orthogonal to nothing
    # in particular but the directional derivative along the shift is zero:
    c = rng.standard_normal(d)
    f2 = lambda e: float(np.sum(R.attention_fwd(q, k + e * c, v, batch, seq)[0] * w))
    assert abs(np.sum(dk * c)) < 1e-12 and abs(f2(1e-3) - f2(0.0)) < 1e-12


# ------------------------------------------------------------------ activations
def test_swiglu_and_gelu_scalar_forms():
    g = rng.standard_normal((3, 4)); u = rng.standard_normal((3, 4)); w = rng.standard_normal((3, 4))
    a = R.swiglu_fwd(g, u)
    assert abs(a[1, 2] - g[1, 2] / (1 + math.exp(-g[1, 2])) * u[1, 2]) < 1e-15
    dg, du = R.swiglu_bwd(w, g, u)
    f = lambda: float(np.sum(R.swiglu_fwd(g, u) * w))
    assert relerr(dg, fd_grad(f, g)) < 1e-8 and relerr(du, fd_grad(f, u)) < 1e-8
    x = rng.standard_normal((3, 4))
    assert R.gelu_fwd(np.zeros(1))[0] == 0.0 and abs(R.gelu_bwd(np.ones(1), np.zeros(1))[0] - 0.5) < 1e-15
    assert abs(R.gelu_fwd(np.array([10.0]))[0] - 10.0) < 1e-9 and abs(R.gelu_fwd(np.array([-10.0]))[0]) < 1e-9
    fg = lambda: float(np.sum(R.gelu_fwd(x) * w))
    assert relerr(R.gelu_bwd(w, x), fd_grad(fg, x)) < 1e-8
    # tanh form stays within 1e-3 of the erf definition x*Phi(x)
    xs = np.linspace(-4, 4, 33)
    erf_form = np.array([0.5 * t * (1 + math.erf(t / math.sqrt(2))) for t in xs])
    assert np.max(np.abs(R.gelu_fwd(xs) - erf_form)) < 1e-3


def test_gelu_erf_form():
    """x Phi(x): Phi from the printed normal table (4 digits) and from Simpson integration of the density (no error
    function involved), the odd-part identity gelu(x) - gelu(-x) = x, the derivative Phi(x) + x phi(x) by hand at one
    point and by finite differences."""
    def phi_cdf(t, n=20000):   # 0.5 + integral of the density from 0 to t, Simpson's rule
        h = t / n
        f = lambda u: math.exp(-0.5 * u * u) / math.sqrt(2 * math.pi)
        acc = f(0.0) + f(t) + sum((4 if i % 2 else 2) * f(i * h) for i in range(1, n))
        return 0.5 + acc * h / 3
    assert R.gelu_fwd(np.zeros(1), 1)[0] == 0.0 and abs(R.gelu_bwd(np.ones(1), np.zeros(1), 1)[0] - 0.5) < 1e-15
    assert abs(R.gelu_fwd(np.array([1.0]), 1)[0] - 0.8413) < 5e-5             # table: Phi(1.00) = 0.8413
    assert abs(R.gelu_fwd(np.array([-1.96]), 1)[0] + 1.96 * 0.0250) < 1e-4    # table: Phi(-1.96) = 0.0250
    for t in (0.3, 1.0, 2.5, -1.7):
        assert abs(R.gelu_fwd(np.array([t]), 1)[0] - t * phi_cdf(t)) < 1e-12
    x = rng.standard_normal((3, 4)); w = rng.standard_normal((3, 4))
    assert np.allclose(R.gelu_fwd(x, 1) - R.gelu_fwd(-x, 1), x, atol=1e-15)
    d1 = phi_cdf(1.0) + 1.0 * math.exp(-0.5) / math.sqrt(2 * math.pi)
    assert abs(R.gelu_bwd(np.ones(1), np.ones(1), 1)[0] - d1) < 1e-12
    fg = lambda: float(np.sum(R.gelu_fwd(x, 1) * w))
    assert relerr(R.gelu_bwd(w, x, 1), fd_grad(fg, x)) < 1e-8
    assert np.max(np.abs(R.gelu_fwd(x, 1) - R.gelu_fwd(x, 0))) > 1e-5      # the two forms do differ


def test_standin_sum_is_exact_ordered_sum():
    own = rng.standard_normal((3, 4)); peers = rng.standard_normal((7, 3, 4)).astype(np.float32)
    s = R.standin_sum(own, peers)
    exp = own.copy()
    for r in range(7):
        exp = exp + peers[r].astype(np.float64)
    assert np.array_equal(s, exp)
    assert np.array_equal(R.standin_sum(own, None), own)
    ints = np.arange(12.0).reshape(3, 4)
    assert np.array_equal(R.standin_sum(ints, np.stack([ints, 2 * ints]).astype(np.float32)), 4 * ints)


# ------------------------------------------------------------------ whole layer
def tiny_layer(batch=2, seq=3, H=8, nq=2, nkv=1, d=4, F=6):
    cfg = R.LayerCfg(batch=batch, seq=seq, H=H, nq=nq, nkv=nkv, d=d, F=F)
    W = dict(g1=1 + 0.1 * rng.standard_normal(H), Wqkv=0.3 * rng.standard_normal((H, cfg.n_qkv)),
             Wo=0.3 * rng.standard_normal((nq * d, H)), g2=1 + 0.1 * rng.standard_normal(H),
             Wgu=0.3 * rng.standard_normal((H, 2 * F)), Wd=0.3 * rng.standard_normal((F, H)))
    x = rng.standard_normal((cfg.T, H))
    return cfg, W, x


def test_layer_bwd_fd_all_inputs_and_weights():
    cfg, W, x = tiny_layer()
    Rm = rng.standard_normal((cfg.T, cfg.H))
    pf = dict(ar1=rng.standard_normal((2, cfg.T, cfg.H)), ar2=rng.standard_normal((2, cfg.T, cfg.H)))
    out, saved = R.llama_fwd(cfg, W, x, pf)
    dx, grads, _ = R.llama_bwd(cfg, W, saved, Rm)
    f = lambda: float(np.sum(R.llama_fwd(cfg, W, x, pf)[0] * Rm))
    assert relerr(dx, fd_grad(f, x)) < 1e-6
    for name, gname in [("Wqkv", "dWqkv"), ("Wo", "dWo"), ("Wgu", "dWgu"), ("Wd", "dWd"), ("g1", "dg1"), ("g2", "dg2")]:
        assert relerr(grads[gname], fd_grad(f, W[name])) < 1e-6, name


def test_layer_bwd_peer_grads_enter_linearly():
    cfg, W, x = tiny_layer()
    Rm = rng.standard_normal((cfg.T, cfg.H))
    _, saved = R.llama_fwd(cfg, W, x)
    dx0, g0, _ = R.llama_bwd(cfg, W, saved, Rm)
    p4 = rng.standard_normal((3, cfg.T, cfg.H))
    dx1, g1, _ = R.llama_bwd(cfg, W, saved, Rm, dict(ar4=p4))
    # a frozen partial added to dh1 passes through norm-1 backward only: weight grads are unchanged
    extra, dg1x = R.rmsnorm_bwd(p4.sum(axis=0), saved["x"], W["g1"], saved["r1"])
    assert np.allclose(dx1 - dx0, extra, atol=1e-12)
    for kname in ("dWqkv", "dWo", "dWgu", "dWd", "dg2"):
        assert np.array_equal(g0[kname], g1[kname])
    assert np.allclose(g1["dg1"] - g0["dg1"], dg1x, atol=1e-12)


def test_layer_zero_weights_gives_input_plus_peer_sums():
    cfg, W, x = tiny_layer()
    for kname in ("Wqkv", "Wo", "Wgu", "Wd"):
        W[kname] = np.zeros_like(W[kname])
    pf = dict(ar1=rng.standard_normal((3, cfg.T, cfg.H)), ar2=rng.standard_normal((3, cfg.T, cfg.H)))
    out, _ = R.llama_fwd(cfg, W, x, pf)
    assert np.allclose(out, x + pf["ar1"].sum(axis=0) + pf["ar2"].sum(axis=0), atol=1e-13)


def torch_llama(cfg, W, x):
    """The same layer composed from torch library ops in float64; gradients by autograd."""
    t = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in W.items()}
    xt = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    T, nq, nkv, d, F = cfg.T, cfg.nq, cfg.nkv, cfg.d, cfg.F

    def norm(z, g):
        return torch.nn.functional.rms_norm(z, (cfg.H,), g, cfg.eps)

    def rot(z):
        half = d // 2
        pos = (torch.arange(T) % cfg.seq).double()
        inv = cfg.rope_base ** (-torch.arange(0, d, 2).double() / d)
        ang = torch.outer(pos, inv)
        z_c = torch.complex(z[..., :half], z[..., half:]) * torch.polar(torch.ones_like(ang), ang)[:, None, :]
        return torch.cat([z_c.real, z_c.imag], dim=-1)

    qkv = norm(xt, t["g1"]) @ t["Wqkv"]
    q, k, v = torch.split(qkv, [nq * d, nkv * d, nkv * d], dim=1)
    q = rot(q.reshape(T, nq, d)); k = rot(k.reshape(T, nkv, d)); v = v.reshape(T, nkv, d)

    def bh(z):  # [T, nh, d] -> [batch, nh, seq, d]
        return z.reshape(cfg.batch, cfg.seq, -1, d).transpose(1, 2)

    o = torch.nn.functional.scaled_dot_product_attention(
        bh(q), bh(k).repeat_interleave(nq // nkv, dim=1), bh(v).repeat_interleave(nq // nkv, dim=1), is_causal=True)
    o = o.transpose(1, 2).reshape(T, nq * d)
    x2 = xt + o @ t["Wo"]
    gu = norm(x2, t["g2"]) @ t["Wgu"]
    out = x2 + (torch.nn.functional.silu(gu[:, :F]) * gu[:, F:]) @ t["Wd"]
    return out, xt, t


def test_layer_matches_torch_autograd_composition():
    cfg, W, x = tiny_layer(batch=2, seq=7, H=16, nq=4, nkv=2, d=8, F=12)
    Rm = rng.standard_normal((cfg.T, cfg.H))
    out, saved = R.llama_fwd(cfg, W, x)
    dx, grads, _ = R.llama_bwd(cfg, W, saved, Rm)
    tout, xt, t = torch_llama(cfg, W, x)
    tout.backward(torch.tensor(Rm))
    assert relerr(out, tout.detach().numpy()) < 1e-13
    assert relerr(dx, xt.grad.numpy()) < 1e-12
    for name, gname in [("Wqkv", "dWqkv"), ("Wo", "dWo"), ("Wgu", "dWgu"), ("Wd", "dWd"), ("g1", "dg1"), ("g2", "dg2")]:
        assert relerr(grads[gname], t[name].grad.numpy()) < 1e-12, name
