"""Pins of the context-parallel oracle (Sec. 2.1/2.2: a rank holds one chunk of each sequence and receives the other
ranks' keys/values): a group of CP ranks, each run through the per-rank oracle with the *actual* keys/values and
key/value gradients of the others, must reproduce the plain full-sequence layer, which other tests pin to autograd."""
import numpy as np
import pytest

from oracle import layer_ref as R
from paper_2411_15871_amd import inputs as gen


def chunk_rows(a, batch, S, s_l, c):
    """Rows of chunk c of every sequence from a [batch*S, ...] array -> [batch*s_l, ...]."""
    return np.concatenate([a[b * S + c * s_l: b * S + (c + 1) * s_l] for b in range(batch)])


@pytest.mark.parametrize("batch,s_l,cp,nq,nkv,d", [(1, 5, 3, 2, 1, 4), (2, 3, 4, 4, 2, 8), (1, 7, 1, 2, 2, 4)])
def test_ctx_attention_is_a_row_slice_of_causal_attention(batch, s_l, cp, nq, nkv, d):
    S = cp * s_l
    q = gen.normal(1, (batch * S, nq, d)).astype(np.float64)
    k = gen.normal(2, (batch * S, nkv, d)).astype(np.float64)
    v = gen.normal(3, (batch * S, nkv, d)).astype(np.float64)
    do = gen.normal(4, (batch * S, nq, d)).astype(np.float64)
    o_full, lse_full = R.attention_fwd(q, k, v, batch, S)
    dq_full, dk_full, dv_full = R.attention_bwd(do, q, k, v, batch, S)
    dk_sum, dv_sum = np.zeros_like(k), np.zeros_like(v)
    for r in range(cp):
        S_r = (r + 1) * s_l
        qr, dor = chunk_rows(q, batch, S, s_l, r), chunk_rows(do, batch, S, s_l, r)
        kr = np.concatenate([k[b * S: b * S + S_r] for b in range(batch)])
        vr = np.concatenate([v[b * S: b * S + S_r] for b in range(batch)])
        o, lse = R.attention_ctx_fwd(qr, kr, vr, batch, s_l, r * s_l)
        assert np.allclose(o, chunk_rows(o_full, batch, S, s_l, r), rtol=1e-12, atol=1e-13)
        assert np.allclose(lse, np.concatenate([lse_full[:, b * S + r * s_l: b * S + (r + 1) * s_l] for b in range(batch)], axis=1),
                           rtol=1e-12, atol=1e-13)
        dq, dk, dv = R.attention_ctx_bwd(dor, qr, kr, vr, batch, s_l, r * s_l)
        assert np.allclose(dq, chunk_rows(dq_full, batch, S, s_l, r), rtol=1e-11, atol=1e-13)
        for b in range(batch):  # every rank's contribution lands on the rows it read
            dk_sum[b * S: b * S + S_r] += dk[b * S_r:(b + 1) * S_r]
            dv_sum[b * S: b * S + S_r] += dv[b * S_r:(b + 1) * S_r]
    assert np.allclose(dk_sum, dk_full, rtol=1e-11, atol=1e-13)
    assert np.allclose(dv_sum, dv_full, rtol=1e-11, atol=1e-13)


@pytest.mark.parametrize("batch,s_l,cp", [(1, 6, 3), (2, 4, 2)])
def test_cp_group_reproduces_the_full_sequence_layer(batch, s_l, cp):
    H, nq, nkv, d, F = 16, 4, 2, 4, 12
    S = cp * s_l
    full = R.LayerCfg(batch, S, H, nq, nkv, d, F)
    part = R.LayerCfg(batch, s_l, H, nq, nkv, d, F)
    W = {k: v.astype(np.float64) for k, v in gen.llama_weights(H, (nq + 2 * nkv) * d, nq * d, F, False).items()}
    x = gen.strand_input(0, batch * S, H, False).astype(np.float64)
    dout = gen.strand_upstream_grad(0, batch * S, H, False).astype(np.float64)
    out_full, saved_full = R.llama_fwd(full, W, x)
    dx_full, g_full, _ = R.llama_bwd(full, W, saved_full, dout)

    # forward: a rank's peers are the other ranks' actual (rotated) keys and values
    xs = [chunk_rows(x, batch, S, s_l, r) for r in range(cp)]
    own_kv = []
    for r in range(cp):
        _, sv = R.llama_cp_fwd(part, W, xs[r], r, {"kv": np.zeros((cp - 1, batch * s_l, 2 * nkv * d))})
        own_kv.append(np.concatenate([sv["k"].reshape(batch * s_l, -1), sv["v"].reshape(batch * s_l, -1)], axis=1))
    saved = []
    for r in range(cp):
        peer_kv = np.stack([own_kv[c] for c in range(cp) if c != r]) if cp > 1 else np.zeros((0, batch * s_l, 2 * nkv * d))
        out, sv = R.llama_cp_fwd(part, W, xs[r], r, {"kv": peer_kv})
        assert np.allclose(out, chunk_rows(out_full, batch, S, s_l, r), rtol=1e-11, atol=1e-12)
        saved.append(sv)

    # backward, last rank first: rank r adds what the later ranks send back for its keys/values
    sent = {}  # (from rank c, to rank r) -> [T_l, 2*nkv*d]
    grads_sum = None
    for r in reversed(range(cp)):
        peer_dkv = np.zeros((max(cp - 1, 0), batch * s_l, 2 * nkv * d))
        for c in range(r + 1, cp):
            peer_dkv[c - 1] = sent[(c, r)]  # slot of rank c in the "all ranks but r" order
        dx, g, inter = R.llama_cp_bwd(part, W, saved[r], chunk_rows(dout, batch, S, s_l, r), r, {"dkv": peer_dkv})
        for c in range(r):
            sent[(r, c)] = inter["dkv_peers"][c]
        assert np.allclose(dx, chunk_rows(dx_full, batch, S, s_l, r), rtol=1e-10, atol=1e-12)
        grads_sum = g if grads_sum is None else {k: grads_sum[k] + g[k] for k in g}
    for k in g_full:
        assert np.allclose(grads_sum[k], g_full[k], rtol=1e-10, atol=1e-12), k


def test_unused_later_chunks_and_earlier_dkv_do_not_matter():
    """Causality: the chunks of later ranks never change a rank's output, and gradient contributions listed for
    earlier ranks (which never read this rank's keys) are not added."""
    batch, s_l, cp, r = 1, 4, 4, 1
    H, nq, nkv, d, F = 16, 2, 1, 8, 8
    cfg = R.LayerCfg(batch, s_l, H, nq, nkv, d, F)
    W = {k: v.astype(np.float64) for k, v in gen.llama_weights(H, (nq + 2 * nkv) * d, nq * d, F, False).items()}
    x = gen.strand_input(0, s_l, H, False).astype(np.float64)
    dout = gen.strand_upstream_grad(0, s_l, H, False).astype(np.float64)
    kv = gen.normal(5, (cp - 1, s_l, 2 * nkv * d)).astype(np.float64)
    kv2 = kv.copy(); kv2[r:] += 1.0  # later ranks' chunks
    out1, sv1 = R.llama_cp_fwd(cfg, W, x, r, {"kv": kv})
    out2, _ = R.llama_cp_fwd(cfg, W, x, r, {"kv": kv2})
    assert np.array_equal(out1, out2)
    dkv = gen.normal(6, (cp - 1, s_l, 2 * nkv * d), 1e-2).astype(np.float64)
    dkv2 = dkv.copy(); dkv2[:r] += 1.0  # earlier ranks
    dx1, g1, _ = R.llama_cp_bwd(cfg, W, sv1, dout, r, {"dkv": dkv})
    dx2, g2, _ = R.llama_cp_bwd(cfg, W, sv1, dout, r, {"dkv": dkv2})
    assert np.array_equal(dx1, dx2) and all(np.array_equal(g1[k], g2[k]) for k in g1)
    dkv3 = dkv.copy(); dkv3[r:] += 1.0
    dx3, _, _ = R.llama_cp_bwd(cfg, W, sv1, dout, r, {"dkv": dkv3})
    assert not np.allclose(dx1, dx3)
