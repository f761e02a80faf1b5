"""GPU parity on seeded random shapes (through the C ABI, against the fp64 oracle): the hand-picked cases of
the other files sit on tile boundaries somebody thought of; these sit wherever the generator puts them, so
that tile choosers, tail splits, chunked attention launches and ragged last tiles are crossed in
combinations nobody listed.  Shapes stay inside each entry point's documented limits."""
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


def dev(a, bf16=True):
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    return t.to(torch.bfloat16) if bf16 else t


def host(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def rel(a, b):
    return np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-30)


def gemm_shapes():
    rng = np.random.default_rng(20241115)
    out = []
    for i in range(36):
        # a third small, a third around one to a few tiles, a third many tiles with a sparse last round
        hi = (300, 1200, 4600)[i % 3]
        M = int(rng.integers(1, hi)); N = int(rng.integers(1, hi // 8 + 1)) * 8
        K = int(rng.integers(1, (hi if i % 3 < 2 else 1600) // 8 + 1)) * 8
        ta, tb = [(0, 0), (0, 1), (1, 0)][int(rng.integers(0, 3))]
        if ta:
            M = (M + 7) // 8 * 8
        out.append((ta, tb, M, N, K))
    return out


@pytest.mark.parametrize("ta,tb,M,N,K", gemm_shapes())
def test_gemm_bf16_random(dh, ta, tb, M, N, K):
    A = gen.normal(60, (K, M) if ta else (M, K), 1.0, 0.0, True)
    B = gen.normal(61, (N, K) if tb else (K, N), 0.05, 0.0, True)
    Ad, Bd = dev(A), dev(B)
    wsb = dh.dh_gemm_workspace_bytes(dh.DH_BF16, ta, tb, M, N, K)
    ws = torch.empty(max(wsb, 16), dtype=torch.uint8, device="cuda")
    ref = (A.T if ta else A).astype(np.float64) @ (B.T if tb else B).astype(np.float64)
    guard = 64  # elements after C: nothing may be written past the matrix
    Cd = torch.full((M * N + guard,), 7.0, dtype=torch.bfloat16, device="cuda")
    dh.dh_gemm(dh.DH_BF16, ta, tb, M, N, K, Ad, Bd, Cd, False, ws, wsb)
    assert rel(host(Cd[: M * N]).reshape(M, N), ref) <= 4e-3
    assert torch.all(Cd[M * N:] == 7.0)
    Cf = torch.full((M * N + guard,), 1.0, dtype=torch.float32, device="cuda")
    dh.dh_gemm(dh.DH_BF16, ta, tb, M, N, K, Ad, Bd, Cf, True, ws, wsb)
    assert rel(host(Cf[: M * N]).reshape(M, N) - 1.0, ref) <= 2e-5
    assert torch.all(Cf[M * N:] == 1.0)
    # the result does not depend on whether a workspace was given beyond rounding order, and is the same
    # bits on a second call with the same arguments (ordered reductions, no atomics)
    Cf2 = torch.full((M * N,), 1.0, dtype=torch.float32, device="cuda")
    dh.dh_gemm(dh.DH_BF16, ta, tb, M, N, K, Ad, Bd, Cf2, True, ws, wsb)
    assert torch.equal(Cf2, Cf[: M * N])


def attn_shapes():
    rng = np.random.default_rng(2411)
    out = []
    for i in range(14):
        d = (64, 128)[i % 2]
        nkv = int(rng.integers(1, 4)); nq = nkv * int(rng.integers(1, 5))
        batch = int(rng.integers(1, 4))
        seq = int(rng.integers(1, (700, 2600)[i % 4 == 3]))
        out.append((batch, seq, nq, nkv, d))
    return out


@pytest.mark.parametrize("batch,seq,nq,nkv,d", attn_shapes())
def test_attention_bf16_random(dh, batch, seq, nq, nkv, d):
    T = batch * seq
    nqkv = (nq + 2 * nkv) * d
    qkv = gen.normal(70, (T, nqkv), 1.0, 0.0, True); do = gen.normal(71, (T, nq * d), 1.0, 0.0, True)
    qd, dod = dev(qkv), dev(do)
    o = torch.empty(T, nq * d, dtype=torch.bfloat16, device="cuda")
    lse = torch.empty(nq, T, dtype=torch.float32, device="cuda")
    fwsb = dh.dh_attn_fwd_workspace_bytes(dh.DH_BF16, batch, seq, nq, nkv, d)
    fws = torch.empty(max(fwsb, 16), dtype=torch.uint8, device="cuda")
    dh.dh_attn_fwd(dh.DH_BF16, batch, seq, nq, nkv, d, qd, o, lse, fws, fwsb)
    q64 = qkv[:, : nq * d].astype(np.float64).reshape(T, nq, d)
    k64 = qkv[:, nq * d: (nq + nkv) * d].astype(np.float64).reshape(T, nkv, d)
    v64 = qkv[:, (nq + nkv) * d:].astype(np.float64).reshape(T, nkv, d)
    o_ref, lse_ref = R.attention_fwd(q64, k64, v64, batch, seq)
    assert rel(host(o), o_ref.reshape(T, nq * d)) <= 1e-2
    assert np.max(np.abs(host(lse) - lse_ref)) <= 2e-2
    dqkv = torch.full((T, nqkv), 3.0, dtype=torch.bfloat16, device="cuda")
    delta = torch.empty(nq, T, dtype=torch.float32, device="cuda")
    wsb = dh.dh_attn_bwd_workspace_bytes(dh.DH_BF16, batch, seq, nq, nkv, d)
    ws = torch.empty(max(wsb, 16), dtype=torch.uint8, device="cuda")
    dh.dh_attn_bwd(dh.DH_BF16, batch, seq, nq, nkv, d, qd, o, dod, lse, dqkv, delta, ws, wsb)
    dq, dk, dv = R.attention_bwd(do.astype(np.float64).reshape(T, nq, d), q64, k64, v64, batch, seq)
    got = host(dqkv)
    floor = np.linalg.norm(dv) if seq == 1 else 0.0   # dq = dk = 0 exactly when a row sees one key

    def relf(a, b):
        return np.linalg.norm(a - b) / max(np.linalg.norm(b), floor)
    assert relf(got[:, : nq * d], dq.reshape(T, -1)) <= 2e-2
    assert relf(got[:, nq * d: (nq + nkv) * d], dk.reshape(T, -1)) <= 2e-2
    assert relf(got[:, (nq + nkv) * d:], dv.reshape(T, -1)) <= 2e-2


def row_shapes():
    rng = np.random.default_rng(158)
    return [(int(rng.integers(1, 3000)), int(rng.integers(1, 1100)) * 8) for _ in range(10)]


@pytest.mark.parametrize("T,H", row_shapes())
def test_norms_random(dh, T, H):
    x = gen.normal(1, (T, H), 1.0, 0.0, True); res = gen.normal(2, (T, H), 0.5, 0.0, True)
    g = gen.normal(3, (H,), 0.02, 1.0, True); dy = gen.normal(4, (T, H), 1e-2, 0.0, True)
    xd, rd, gd, dyd = (dev(a) for a in (x, res, g, dy))
    x2 = torch.empty_like(xd); h = torch.empty_like(xd); rstd = torch.empty(T, dtype=torch.float32, device="cuda")
    dh.dh_rmsnorm_fwd(dh.DH_BF16, T, H, xd, rd, gd, 1e-5, x2, h, rstd)
    h_ref, r_ref = R.rmsnorm_fwd(host(x2), g.astype(np.float64), 1e-5)
    assert rel(host(x2), x.astype(np.float64) + res) <= 4e-3
    assert rel(host(h), h_ref) <= 6e-3
    assert rel(host(rstd), r_ref[:, 0]) <= 1e-5
    dx = torch.empty_like(xd); dg = torch.zeros((H,), dtype=torch.float32, device="cuda")
    wsb = dh.dh_rmsnorm_bwd_ws_bytes(T, H)
    ws = torch.empty(max(wsb, 16), dtype=torch.uint8, device="cuda")
    dh.dh_rmsnorm_bwd(dh.DH_BF16, T, H, dyd, x2, gd, rstd, None, dx, dg, ws, wsb)
    dx_ref, dg_ref = R.rmsnorm_bwd(dy.astype(np.float64), host(x2), g.astype(np.float64), host(rstd)[:, None])
    assert rel(host(dx), dx_ref) <= 6e-3
    assert rel(host(dg), dg_ref) <= 1e-4


def grouped_cases():
    rng = np.random.default_rng(777)
    out = []
    for i in range(10):
        G = int(rng.integers(1, 6))
        hi = (400, 1500, 2600)[i % 3]
        rows = [int(rng.integers(0, hi)) if rng.random() > 0.15 else 0 for _ in range(G)]
        K = int(rng.integers(1, 130)) * 8; N = int(rng.integers(1, (130, 520)[i % 2])) * 8
        out.append((tuple(rows), K, N))
    return out


@pytest.mark.parametrize("rows,K,N", grouped_cases())
def test_gemm_grouped_random(dh, rows, K, N):
    """Row counts are device data: groups of any size, empty ones included, in all three grouped forms."""
    G, Tt = len(rows), sum(rows)
    A = gen.normal(31, (max(Tt, 1), K), 1.0, 0.0, True); W = gen.normal(32, (G, K, N), 0.05, 0.0, True)
    dC = gen.normal(33, (max(Tt, 1), N), 1.0, 0.0, True)
    Ad, Wd, dCd = dev(A), dev(W), dev(dC)
    Cd = torch.full((max(Tt, 1) + 1, N), 5.0, dtype=torch.bfloat16, device="cuda")   # one guard row behind the groups
    dAd = torch.full((max(Tt, 1) + 1, K), 5.0, dtype=torch.bfloat16, device="cuda")
    dW = torch.full((G, K, N), 0.5, dtype=torch.float32, device="cuda")
    rd = torch.tensor(rows, dtype=torch.int32, device="cuda")
    dh.dh_gemm_grouped(dh.DH_BF16, 0, G, rd, Tt, K, N, Ad, Wd, Cd)
    dh.dh_gemm_grouped(dh.DH_BF16, 1, G, rd, Tt, N, K, dCd, Wd, dAd)
    dh.dh_gemm_grouped(dh.DH_BF16, 2, G, rd, Tt, K, N, Ad, dCd, dW)
    torch.cuda.synchronize()
    A64, W64, dC64 = A.astype(np.float64), W.astype(np.float64), dC.astype(np.float64)
    r0 = 0
    for g in range(G):
        r1 = r0 + rows[g]
        if r1 > r0:
            assert rel(host(Cd)[r0:r1], A64[r0:r1] @ W64[g]) <= 4e-3
            assert rel(host(dAd)[r0:r1], dC64[r0:r1] @ W64[g].T) <= 4e-3
        ref = A64[r0:r1].T @ dC64[r0:r1]
        assert np.linalg.norm(host(dW)[g] - 0.5 - ref) <= 2e-5 * max(np.linalg.norm(ref), 1e-30) + 1e-12
        r0 = r1
    assert torch.all(Cd[Tt:] == 5.0) and torch.all(dAd[Tt:] == 5.0)


def ctx_cases():
    rng = np.random.default_rng(4096)
    out = []
    for i in range(8):
        d = (128, 64)[i % 2]
        nkv = int(rng.integers(1, 3)); nq = nkv * int(rng.integers(1, 5))
        batch = int(rng.integers(1, 3))
        seq = int(rng.integers(1, (500, 1500)[i % 4 == 1]))
        q_off = 128 * int(rng.integers(0, (8, 20)[i % 4 == 2]))   # the matrix-core kernels take offsets in whole key blocks
        out.append((batch, seq, q_off, nq, nkv, d))
    return out


@pytest.mark.parametrize("batch,seq,q_off,nq,nkv,d", ctx_cases())
def test_ctx_attention_bf16_random(dh, batch, seq, q_off, nq, nkv, d):
    T, S = batch * seq, q_off + seq
    nqkv = (nq + 2 * nkv) * d
    qkv = gen.normal(50, (T, nqkv), 1.0, 0.0, True)
    kv = gen.normal(52, (batch * S, 2 * nkv * d), 1.0, 0.0, True)
    do = gen.normal(51, (T, nq * d), 1.0, 0.0, True)
    qd, kvd, dod = dev(qkv), dev(kv), dev(do)
    o = torch.empty(T, nq * d, dtype=torch.bfloat16, device="cuda")
    lse = torch.empty(nq, T, dtype=torch.float32, device="cuda")
    fwsb = dh.dh_attn_ctx_fwd_workspace_bytes(dh.DH_BF16, batch, seq, q_off, nq, nkv, d)
    fws = torch.empty(max(fwsb, 16), dtype=torch.uint8, device="cuda")
    dh.dh_attn_ctx_fwd(dh.DH_BF16, batch, seq, q_off, nq, nkv, d, qd, kvd, o, lse, fws, fwsb)
    q64 = qkv[:, : nq * d].astype(np.float64).reshape(T, nq, d)
    k64 = kv[:, : nkv * d].astype(np.float64).reshape(batch * S, nkv, d)
    v64 = kv[:, nkv * d:].astype(np.float64).reshape(batch * S, nkv, d)
    o_ref, lse_ref = R.attention_ctx_fwd(q64, k64, v64, batch, seq, q_off)
    assert rel(host(o), o_ref.reshape(T, nq * d)) <= 1e-2
    assert np.max(np.abs(host(lse) - lse_ref)) <= 2e-2
    qcols = torch.full((T, nqkv), 7.0, dtype=torch.bfloat16, device="cuda")
    dkv = torch.zeros(batch * S, 2 * nkv * d, dtype=torch.bfloat16, device="cuda")
    delta = torch.empty(nq, T, dtype=torch.float32, device="cuda")
    wsb = dh.dh_attn_ctx_bwd_workspace_bytes(dh.DH_BF16, batch, seq, q_off, nq, nkv, d)
    ws = torch.empty(max(wsb, 16), dtype=torch.uint8, device="cuda")
    dh.dh_attn_ctx_bwd(dh.DH_BF16, batch, seq, q_off, nq, nkv, d, qd, kvd, o, dod, lse, qcols, dkv, delta, ws, wsb)
    torch.cuda.synchronize()
    dq, dk, dv = R.attention_ctx_bwd(do.astype(np.float64).reshape(T, nq, d), q64, k64, v64, batch, seq, q_off)
    got_q, got_kv = host(qcols), host(dkv)
    floor = np.linalg.norm(dv) if S == 1 else 0.0

    def relf(a, b):
        return np.linalg.norm(a - b) / max(np.linalg.norm(b), floor, 1e-30)
    assert relf(got_q[:, : nq * d], dq.reshape(T, nq * d)) <= 2e-2
    assert np.all(got_q[:, nq * d:] == 7.0)   # only the query columns of the gradient rows are written
    assert relf(got_kv[:, : nkv * d], dk.reshape(batch * S, nkv * d)) <= 2e-2
    assert relf(got_kv[:, nkv * d:], dv.reshape(batch * S, nkv * d)) <= 2e-2
