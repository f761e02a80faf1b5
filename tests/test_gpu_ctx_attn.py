"""GPU parity of the context-parallel attention operators (offset causal attention over a gathered key/value buffer,
rotary embedding at a position offset) through the C ABI against the fp64 oracle.
Tolerances: relative L2 <= 1e-5 (fp32), <= 2e-2 (bf16, 1e-2 for the forward output)."""
import numpy as np
import pytest
import torch

from oracle import layer_ref as R
from paper_2411_15871_amd import inputs as gen

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dh():
    from paper_2411_15871_amd import dhelix
    assert torch.cuda.is_available()
    return dhelix


def dev(a, bf16):
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    return t.to(torch.bfloat16) if bf16 else t


def host(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def rel(a, b, floor=0.0):
    return np.linalg.norm(a - b) / max(np.linalg.norm(b), floor, 1e-30)


CASES = [  # bf16, batch, seq (queries per sequence), q_off, nq, nkv, d
    (False, 1, 5, 0, 2, 1, 8), (False, 2, 7, 14, 4, 2, 16), (False, 1, 70, 130, 2, 2, 64), (False, 1, 33, 99, 4, 1, 128),
    (True, 1, 128, 0, 2, 1, 128), (True, 1, 128, 128, 2, 1, 128), (True, 2, 200, 256, 4, 2, 64), (True, 1, 300, 384, 2, 2, 128),
    (True, 1, 1100, 1152, 4, 1, 128),   # rows long enough to be cut into chunks, ragged tail
    (True, 1, 1024, 3072, 4, 1, 128),   # the last rank of four
    (True, 2, 64, 128, 2, 2, 64),
]


@pytest.mark.parametrize("bf16,batch,seq,q_off,nq,nkv,d", CASES)
def test_ctx_attention_fwd_bwd(dh, bf16, batch, seq, q_off, nq, nkv, d):
    print("case", bf16, batch, seq, q_off, nq, nkv, d, flush=True)
    dtp = dh.DH_BF16 if bf16 else dh.DH_F32
    tdt = torch.bfloat16 if bf16 else torch.float32
    T, S = batch * seq, q_off + seq
    nqkv = (nq + 2 * nkv) * d
    qkv = gen.normal(50, (T, nqkv), 1.0, 0.0, bf16)   # only the q columns are read
    kv = gen.normal(52, (batch * S, 2 * nkv * d), 1.0, 0.0, bf16)
    do = gen.normal(51, (T, nq * d), 1.0, 0.0, bf16)
    qd, kvd, dod = dev(qkv, bf16), dev(kv, bf16), dev(do, bf16)
    o = torch.empty(T, nq * d, dtype=tdt, device="cuda")
    lse = torch.empty(nq, T, dtype=torch.float32, device="cuda")
    fwsb = dh.dh_attn_ctx_fwd_workspace_bytes(dtp, batch, seq, q_off, nq, nkv, d)
    fws = torch.empty(max(fwsb, 16), dtype=torch.uint8, device="cuda")
    dh.dh_attn_ctx_fwd(dtp, batch, seq, q_off, nq, nkv, d, qd, kvd, o, lse, fws, fwsb)
    o_ns = torch.empty_like(o); lse_ns = torch.empty_like(lse)
    dh.dh_attn_ctx_fwd(dtp, batch, seq, q_off, nq, nkv, d, qd, kvd, o_ns, lse_ns)  # no workspace: rows not split
    torch.cuda.synchronize()
    q64 = qkv[:, : nq * d].astype(np.float64).reshape(T, nq, d)
    k64 = kv[:, : nkv * d].astype(np.float64).reshape(batch * S, nkv, d)
    v64 = kv[:, nkv * d:].astype(np.float64).reshape(batch * S, nkv, d)
    o_ref, lse_ref = R.attention_ctx_fwd(q64, k64, v64, batch, seq, q_off)
    tol = 1e-2 if bf16 else 1e-5
    for got_o, got_l in ((o, lse), (o_ns, lse_ns)):
        assert rel(host(got_o), o_ref.reshape(T, nq * d)) <= tol
        assert np.max(np.abs(host(got_l) - lse_ref)) <= (2e-2 if bf16 else 1e-5)
    qcols = torch.full((T, nqkv), 7.0, dtype=tdt, device="cuda")
    dkv = torch.zeros(batch * S, 2 * nkv * d, dtype=tdt, device="cuda")
    delta = torch.empty(nq, T, dtype=torch.float32, device="cuda")
    wsb = dh.dh_attn_ctx_bwd_workspace_bytes(dtp, batch, seq, q_off, nq, nkv, d)
    ws = torch.empty(max(wsb, 16), dtype=torch.uint8, device="cuda")
    dh.dh_attn_ctx_bwd(dtp, batch, seq, q_off, nq, nkv, d, qd, kvd, o, dod, lse, qcols, dkv, delta, ws, wsb)
    torch.cuda.synchronize()
    dq, dk, dv = R.attention_ctx_bwd(do.astype(np.float64).reshape(T, nq, d), q64, k64, v64, batch, seq, q_off)
    tol = 2e-2 if bf16 else 1e-5
    got_q, got_kv = host(qcols), host(dkv)
    assert rel(got_q[:, : nq * d], dq.reshape(T, nq * d)) <= tol
    assert np.all(got_q[:, nq * d:] == 7.0)  # the k, v columns of dqkv are not this call's to write
    assert rel(got_kv[:, : nkv * d], dk.reshape(batch * S, nkv * d)) <= tol
    assert rel(got_kv[:, nkv * d:], dv.reshape(batch * S, nkv * d)) <= tol


def test_ctx_attention_rejects_bad_geometry(dh):
    q = torch.zeros(128, 4 * 128, dtype=torch.bfloat16, device="cuda"); kv = torch.zeros(192, 2 * 128, dtype=torch.bfloat16, device="cuda")
    o = torch.zeros(128, 2 * 128, dtype=torch.bfloat16, device="cuda"); lse = torch.zeros(2, 128, device="cuda")
    with pytest.raises(dh.DhelixError):
        dh.dh_attn_ctx_fwd(dh.DH_BF16, 1, 128, 64, 2, 1, 128, q, kv, o, lse)  # bf16 offsets come in multiples of 128
    with pytest.raises(dh.DhelixError):
        dh.dh_attn_ctx_fwd(dh.DH_BF16, 1, 128, -128, 2, 1, 128, q, kv, o, lse)
    with pytest.raises(dh.DhelixError):
        dh.dh_attn_ctx_fwd(dh.DH_BF16, 1, 128, 0, 2, 1, 128, q, None, o, lse)


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("batch,seq,pos0,nh,d", [(1, 9, 27, 3, 16), (2, 130, 4096, 5, 128)])
def test_rope_at(dh, bf16, batch, seq, pos0, nh, d):
    T = batch * seq
    t = gen.normal(9, (T, nh * d), 1.0, 0.0, bf16)
    td = dev(t, bf16)
    dh.dh_rope_at(dh.DH_BF16 if bf16 else dh.DH_F32, T, seq, pos0, nh, d, nh * d, 10000.0, False, td)
    torch.cuda.synchronize()
    ref = R.rope(t.astype(np.float64).reshape(T, nh, d), seq, 10000.0, pos0=pos0).reshape(T, nh * d)
    assert rel(host(td), ref) <= (4e-3 if bf16 else 2e-6)


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("n_blocks", [0, 1, 3])
def test_cp_exchange_and_grad_reduce(dh, bf16, n_blocks):
    """The Send/Recv stand-ins: chunk copies between buffers of different pitch (bit-exact) and the ordered sum that
    forms the key/value gradient a rank keeps."""
    dtp = dh.DH_BF16 if bf16 else dh.DH_F32
    batch, rows, W, cp, r = 2, 45, 48, 4, 2
    S, ld_own = (r + 1) * rows, 80
    own = gen.normal(1, (batch * rows, ld_own), 1.0, 0.0, bf16)          # packed rows, key/value columns start at 24
    peers = gen.normal(2, (cp - 1, batch * rows, W), 1.0, 0.0, bf16)
    ownd, peersd = dev(own, bf16), dev(peers, bf16)
    kv = torch.zeros(batch * S, W, dtype=ownd.dtype, device="cuda")
    recv = torch.zeros(cp - 1 - r, batch * rows, W, dtype=ownd.dtype, device="cuda")
    es = ownd.element_size()
    moves = []
    for k in range(cp):
        src = ownd.data_ptr() + 24 * es if k == r else peersd.data_ptr() + (k if k < r else k - 1) * batch * rows * W * es
        if k <= r:
            moves.append(dh.cp_move(src, kv, ld_own if k == r else W, rows, 0, W, S, k * rows))
        else:
            moves.append(dh.cp_move(src, recv.data_ptr() + (k - r - 1) * batch * rows * W * es, W, rows, 0, W, rows, 0))
    dh.dh_cp_exchange(dtp, moves, batch, rows, W, n_blocks)
    torch.cuda.synchronize()
    k64 = own[:, 24:24 + W // 2].reshape(batch * rows, 1, W // 2); v64 = own[:, 24 + W // 2:24 + W].reshape(batch * rows, 1, W // 2)
    K, V = R.cp_gather_kv(k64.astype(np.float64), v64.astype(np.float64), peers, batch, rows, r)
    assert np.array_equal(host(kv), np.concatenate([K.reshape(batch * S, -1), V.reshape(batch * S, -1)], axis=1))
    assert np.array_equal(host(recv), peers[r:].astype(np.float64))
    # gradient kept by the rank: its own rows of a [batch*S, W] buffer plus the later ranks' contributions, into packed rows
    dkv = gen.normal(3, (batch * S, W), 1.0, 0.0, bf16)
    later = gen.normal(4, (cp - 1 - r, batch * rows, W), 1.0, 0.0, bf16)
    dkvd, laterd = dev(dkv, bf16), dev(later, bf16)
    dq = torch.full((batch * rows, ld_own), 3.0, dtype=ownd.dtype, device="cuda")
    mv = dh.cp_move(dkvd, dq.data_ptr() + 24 * es, W, S, r * rows, ld_own, rows, 0)
    dh.dh_cp_grad_reduce(dtp, mv, [laterd.data_ptr() + i * batch * rows * W * es for i in range(cp - 1 - r)], batch, rows, W, n_blocks)
    torch.cuda.synchronize()
    ref = np.concatenate([dkv[b * S + r * rows:(b + 1) * S] for b in range(batch)]).astype(np.float64) + later.astype(np.float64).sum(axis=0)
    got = host(dq)
    assert np.linalg.norm(got[:, 24:24 + W] - ref) <= (1e-2 if bf16 else 1e-6) * np.linalg.norm(ref)
    assert np.all(got[:, :24] == 3.0) and np.all(got[:, 24 + W:] == 3.0)
    with pytest.raises(dh.DhelixError):
        dh.dh_cp_exchange(dtp, [dh.cp_move(ownd, kv, ld_own, rows, 0, W, S, S - rows + 1)], batch, rows, W)  # runs past its sequence
