"""GPU parity of the mixture-of-experts operators (through the C ABI) against the fp64 oracle.
Routing indices, permutation tables and row counts are compared bit-exact; floating-point results to
relative L2 <= 1e-5 (fp32 storage) and <= 2e-2 (bf16)."""
import numpy as np
import pytest
import torch

from oracle import layer_ref as R
from paper_2411_15871_amd import inputs as gen

pytestmark = pytest.mark.gpu

TOL = {False: 1e-5, True: 2e-2}


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


def rel(a, b):
    return np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-30)


def dt(dh, bf16):
    return dh.DH_BF16 if bf16 else dh.DH_F32


def i32(n):
    return torch.full((max(n, 1),), -7, dtype=torch.int32, device="cuda")


def make_tables(dh, T, E, n_local):
    t = dict(rank=i32(2 * T), dest=i32(2 * T), src_tok=i32(2 * T), send_of_recv=i32(2 * T), recv_of_send=i32(2 * T),
             counts=i32(E), offsets=i32(E + 1), recv_start=i32(E), group_rows=i32(n_local))
    return t, dh.moe_tables(**t)


def logits_case(T, E, ties):
    l = gen.router_logits(T, E)
    if ties:  # few distinct values: many exact ties, decided by the lower expert id
        l = np.round(l * 2.0) / 2.0
    return l.astype(np.float32)


@pytest.mark.parametrize("ties", [False, True])
@pytest.mark.parametrize("T,E", [(0, 16), (1, 2), (777, 8), (4096, 16), (513, 64)])
def test_route_exact_indices(dh, T, E, ties):
    l = logits_case(T, E, ties)
    ld = torch.from_numpy(l).cuda()
    idx = i32(2 * T); prob = torch.zeros(max(2 * T, 1), dtype=torch.float32, device="cuda")
    dh.dh_moe_route(T, E, ld, idx, prob)
    torch.cuda.synchronize()
    if T == 0:
        return
    ridx, rprob = R.router_top2(l.astype(np.float64))
    assert np.array_equal(idx.cpu().numpy()[:2 * T].reshape(T, 2), ridx)
    assert rel(host(prob)[:2 * T].reshape(T, 2), rprob) <= 1e-6
    dprob = gen.normal(11, (T, 2), 1.0, 0.0, False).astype(np.float32)
    dl = torch.full((T, E), 3.0, dtype=torch.float32, device="cuda")
    dh.dh_moe_route_bwd(T, E, torch.from_numpy(dprob).cuda(), idx, prob, dl)
    torch.cuda.synchronize()
    dl_ref = R.router_top2_bwd(dprob.astype(np.float64), ridx, host(prob)[:2 * T].reshape(T, 2), E)
    assert rel(host(dl), dl_ref) <= 1e-5


@pytest.mark.parametrize("ties", [False, True])
@pytest.mark.parametrize("T,E,n_local", [(0, 8, 2), (1, 2, 1), (777, 8, 2), (4096, 16, 2), (513, 64, 8), (300, 16, 16)])
def test_plan_tables_exact(dh, T, E, n_local, ties):
    l = logits_case(T, E, ties)
    ridx, _ = R.router_top2(l.astype(np.float64)) if T else (np.zeros((0, 2), dtype=np.int64), None)
    idx = torch.from_numpy(ridx.astype(np.int32).reshape(-1)).cuda() if T else i32(0)
    tb, tbs = make_tables(dh, T, E, n_local)
    dh.dh_moe_plan(T, E, n_local, idx, tbs)
    torch.cuda.synchronize()
    dest, src, counts = R.permute_rows(ridx, E)
    order, group_rows = R.a2a_dispatch_order(counts, n_local)
    g = {k: v.cpu().numpy() for k, v in tb.items()}
    assert np.array_equal(g["counts"][:E], counts)
    assert np.array_equal(g["offsets"][:E + 1], np.concatenate([[0], np.cumsum(counts)]))
    assert np.array_equal(g["group_rows"][:n_local], np.array(group_rows))
    assert np.array_equal(g["dest"][:2 * T].reshape(T, 2), dest)
    assert np.array_equal(g["src_tok"][:2 * T], src)
    assert np.array_equal(g["send_of_recv"][:2 * T], order)
    inv = np.zeros(2 * T, dtype=np.int64); inv[order] = np.arange(2 * T)
    assert np.array_equal(g["recv_of_send"][:2 * T], inv)


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("T,H,n_blocks", [(0, 64, 0), (5, 8, 0), (333, 4096, 0), (1000, 520, 16)])
def test_gather_combine(dh, bf16, T, H, n_blocks):
    E, n_local = 8, 2
    l = logits_case(T, E, False)
    x = gen.normal(21, (T, H), 1.0, 0.0, bf16)
    if T == 0:
        dh.dh_moe_gather_rows(dt(dh, bf16), 0, H, None, None, None, n_blocks)
        dh.dh_moe_combine(dt(dh, bf16), 0, H, None, None, None, None, None)
        dh.dh_moe_combine_bwd(dt(dh, bf16), 0, H, None, None, None, None, None, None)
        return
    ridx, rprob = R.router_top2(l.astype(np.float64))
    dest, src, counts = R.permute_rows(ridx, E)
    srcd = torch.from_numpy(src.astype(np.int32)).cuda()
    destd = torch.from_numpy(dest.astype(np.int32).reshape(-1)).cuda()
    probd = torch.from_numpy(rprob.astype(np.float32).reshape(-1)).cuda()
    xd = dev(x, bf16)
    xp = torch.empty(2 * T, H, dtype=xd.dtype, device="cuda")
    dh.dh_moe_gather_rows(dt(dh, bf16), 2 * T, H, xd, srcd, xp, n_blocks)
    torch.cuda.synchronize()
    assert np.array_equal(host(xp), x.astype(np.float64)[src])  # a copy: exact
    yp = gen.normal(22, (2 * T, H), 1.0, 0.0, bf16)
    ypd = dev(yp, bf16)
    y = torch.empty_like(xd)
    dh.dh_moe_combine(dt(dh, bf16), T, H, ypd, destd, probd, None, y)
    y1 = torch.empty_like(xd)
    dh.dh_moe_combine(dt(dh, bf16), T, H, ypd, destd, None, xd, y1)
    torch.cuda.synchronize()
    p32 = rprob.astype(np.float32).astype(np.float64)
    y_ref = p32[:, 0:1] * yp[dest[:, 0]] + p32[:, 1:2] * yp[dest[:, 1]]
    assert rel(host(y), y_ref) <= TOL[bf16]
    assert rel(host(y1), yp[dest[:, 0]].astype(np.float64) + yp[dest[:, 1]] + x) <= TOL[bf16]
    dy = gen.normal(23, (T, H), 1e-2, 0.0, bf16)
    dyp = torch.zeros_like(ypd); dprob = torch.zeros(2 * T, dtype=torch.float32, device="cuda")
    dh.dh_moe_combine_bwd(dt(dh, bf16), T, H, dev(dy, bf16), ypd, destd, probd, dyp, dprob)
    torch.cuda.synchronize()
    dyp_ref = np.zeros((2 * T, H))
    for k in range(2):
        dyp_ref[dest[:, k]] = p32[:, k:k + 1] * dy
    dprob_ref = np.stack([np.sum(dy.astype(np.float64) * yp[dest[:, k]], axis=1) for k in range(2)], axis=1)
    assert rel(host(dyp), dyp_ref) <= TOL[bf16]
    assert rel(host(dprob).reshape(T, 2), dprob_ref) <= 1e-5 * (1 if not bf16 else 10)


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("rows,K,N", [([5, 0, 130], 64, 96), ([300, 212], 256, 264), ([0, 0], 64, 64)])
def test_gemm_grouped(dh, bf16, rows, K, N):
    G, Tt = len(rows), sum(rows)
    A = gen.normal(31, (Tt, K), 1.0, 0.0, bf16); W = gen.normal(32, (G, K, N), 0.05, 0.0, bf16)
    dC = gen.normal(33, (Tt, N), 1.0, 0.0, bf16)
    Ad, Wd, dCd = dev(A, bf16), dev(W, bf16), dev(dC, bf16)
    Cd = torch.zeros(max(Tt, 1), N, dtype=Ad.dtype, device="cuda")
    dAd = torch.zeros(max(Tt, 1), K, dtype=Ad.dtype, device="cuda")
    dW = torch.full((G, K, N), 0.5, dtype=torch.float32, device="cuda")
    rd = torch.tensor(rows, dtype=torch.int32, device="cuda")
    dh.dh_gemm_grouped(dt(dh, bf16), 0, G, rd, Tt, K, N, Ad, Wd, Cd)
    dh.dh_gemm_grouped(dt(dh, bf16), 1, G, rd, Tt, N, K, dCd, Wd, dAd)
    dh.dh_gemm_grouped(dt(dh, bf16), 2, G, rd, Tt, K, N, Ad, dCd, dW)
    torch.cuda.synchronize()
    r0 = 0
    A64, W64, dC64 = A.astype(np.float64), W.astype(np.float64), dC.astype(np.float64)
    for g in range(G):
        r1 = r0 + rows[g]
        if r1 > r0:
            assert rel(host(Cd)[r0:r1], A64[r0:r1] @ W64[g]) <= TOL[bf16]
            assert rel(host(dAd)[r0:r1], dC64[r0:r1] @ W64[g].T) <= TOL[bf16]
        ref = A64[r0:r1].T @ dC64[r0:r1]
        assert np.linalg.norm(host(dW)[g] - 0.5 - ref) <= TOL[bf16] * max(np.linalg.norm(ref), 1e-30) + 1e-12
        r0 = r1


@pytest.mark.parametrize("rows", [[2100, 2000], [2304, 1792], [2660, 1000], [4100, 0]])
def test_gemm_grouped_large_tiles_and_remainders(dh, rows):
    """Shapes that take the 256x256 tile: with 2100 + 2000 rows the large tiles would need a nearly empty second round,
    so the groups' remainder rows go to the second (small-tile) launch; the other row counts keep everything in the first."""
    K = N = 4096
    G, Tt = len(rows), sum(rows)
    A = gen.normal(31, (Tt, K), 1.0, 0.0, True); W = gen.normal(32, (G, K, N), 0.02, 0.0, True)
    Ad, Wd = dev(A, True), dev(W, True)
    Cd = torch.zeros(Tt, N, dtype=Ad.dtype, device="cuda"); dAd = torch.zeros(Tt, K, dtype=Ad.dtype, device="cuda")
    rd = torch.tensor(rows, dtype=torch.int32, device="cuda")
    dh.dh_gemm_grouped(dh.DH_BF16, 0, G, rd, Tt, K, N, Ad, Wd, Cd)
    dh.dh_gemm_grouped(dh.DH_BF16, 1, G, rd, Tt, N, K, Ad, Wd, dAd)   # A stands in for an upstream gradient [Tt, N]
    torch.cuda.synchronize()
    r0 = 0
    A64, W64 = A.astype(np.float64), W.astype(np.float64)
    for g in range(G):
        r1 = r0 + rows[g]
        if r1 > r0:
            assert rel(host(Cd)[r0:r1], A64[r0:r1] @ W64[g]) <= TOL[True]
            assert rel(host(dAd)[r0:r1], A64[r0:r1] @ W64[g].T) <= TOL[True]
            # the seam between the two launches: last whole large-tile row and first remainder row
            seam = r0 + rows[g] // 256 * 256
            for r in (seam - 1, seam, r1 - 1):
                if r0 <= r < r1:
                    assert rel(host(Cd)[r], A64[r] @ W64[g]) <= TOL[True]
        r0 = r1


@pytest.mark.parametrize("bf16,T,H,F,E,n_local", [(False, 300, 64, 96, 8, 2), (True, 1000, 256, 384, 16, 2),
                                                  (True, 257, 128, 64, 4, 4)])
def test_moe_block_fwd_bwd(dh, bf16, T, H, F, E, n_local):
    """Whole MoE FFN block composed from the C-ABI operators in the order of the layer, against
    oracle moe_ffn_fwd / moe_ffn_bwd on the same inputs."""
    d = dt(dh, bf16)
    l = logits_case(T, E, False)
    h2 = gen.normal(41, (T, H), 1.0, 0.0, bf16)
    Wgu = gen.normal(42, (n_local, H, 2 * F), 0.05, 0.0, bf16); Wd = gen.normal(43, (n_local, F, H), 0.05, 0.0, bf16)
    dy = gen.normal(44, (T, H), 1e-2, 0.0, bf16)
    y_ref, sv = R.moe_ffn_fwd(h2.astype(np.float64), l.astype(np.float64), Wgu.astype(np.float64), Wd.astype(np.float64), n_local)
    dh2_ref, dl_ref, dWgu_ref, dWd_ref = R.moe_ffn_bwd(dy.astype(np.float64), h2.astype(np.float64), Wgu.astype(np.float64),
                                                       Wd.astype(np.float64), sv, n_local)
    ld = torch.from_numpy(l).cuda(); h2d, Wgud, Wdd, dyd = dev(h2, bf16), dev(Wgu, bf16), dev(Wd, bf16), dev(dy, bf16)
    idx = i32(2 * T); prob = torch.zeros(2 * T, dtype=torch.float32, device="cuda")
    tb, tbs = make_tables(dh, T, E, n_local)

    def buf(r, c):
        return torch.empty(r, c, dtype=h2d.dtype, device="cuda")

    # forward
    dh.dh_moe_route(T, E, ld, idx, prob)
    dh.dh_moe_plan(T, E, n_local, idx, tbs)
    rows = tb["group_rows"].cpu().numpy()[:n_local].tolist()
    assert rows == [int(r) for r in sv["group_rows"]]
    assert np.array_equal(idx.cpu().numpy().reshape(T, 2), sv["idx"])
    xp, xg, gu, a, yg, yp, y = buf(2 * T, H), buf(2 * T, H), buf(2 * T, 2 * F), buf(2 * T, F), buf(2 * T, H), buf(2 * T, H), buf(T, H)
    dh.dh_moe_gather_rows(d, 2 * T, H, h2d, tb["src_tok"], xp)
    dh.dh_moe_gather_rows(d, 2 * T, H, xp, tb["send_of_recv"], xg)
    dh.dh_gemm_grouped(d, 0, n_local, tb["group_rows"], 2 * T, H, 2 * F, xg, Wgud, gu)
    dh.dh_swiglu_fwd(d, 2 * T, F, gu, a)
    dh.dh_gemm_grouped(d, 0, n_local, tb["group_rows"], 2 * T, F, H, a, Wdd, yg)
    dh.dh_moe_gather_rows(d, 2 * T, H, yg, tb["recv_of_send"], yp)
    dh.dh_moe_combine(d, T, H, yp, tb["dest"], prob, None, y)
    torch.cuda.synchronize()
    assert rel(host(y), y_ref) <= TOL[bf16]
    # backward
    dyp, dyg, da, dgu, dxg, dxp, dh2 = buf(2 * T, H), buf(2 * T, H), buf(2 * T, F), buf(2 * T, 2 * F), buf(2 * T, H), buf(2 * T, H), buf(T, H)
    dprob = torch.zeros(2 * T, dtype=torch.float32, device="cuda"); dl = torch.zeros(T, E, dtype=torch.float32, device="cuda")
    dWgu = torch.zeros(n_local, H, 2 * F, dtype=torch.float32, device="cuda"); dWd = torch.zeros(n_local, F, H, dtype=torch.float32, device="cuda")
    dh.dh_moe_combine_bwd(d, T, H, dyd, yp, tb["dest"], prob, dyp, dprob)
    dh.dh_moe_route_bwd(T, E, dprob, idx, prob, dl)
    dh.dh_moe_gather_rows(d, 2 * T, H, dyp, tb["send_of_recv"], dyg)
    dh.dh_gemm_grouped(d, 1, n_local, tb["group_rows"], 2 * T, H, F, dyg, Wdd, da)
    dh.dh_gemm_grouped(d, 2, n_local, tb["group_rows"], 2 * T, F, H, a, dyg, dWd)
    dh.dh_swiglu_bwd(d, 2 * T, F, gu, da, dgu)
    dh.dh_gemm_grouped(d, 2, n_local, tb["group_rows"], 2 * T, H, 2 * F, xg, dgu, dWgu)
    dh.dh_gemm_grouped(d, 1, n_local, tb["group_rows"], 2 * T, 2 * F, H, dgu, Wgud, dxg)
    dh.dh_moe_gather_rows(d, 2 * T, H, dxg, tb["recv_of_send"], dxp)
    dh.dh_moe_combine(d, T, H, dxp, tb["dest"], None, None, dh2)
    torch.cuda.synchronize()
    assert rel(host(dh2), dh2_ref) <= TOL[bf16]
    assert rel(host(dl), dl_ref) <= TOL[bf16]
    assert rel(host(dWgu), dWgu_ref) <= TOL[bf16]
    assert rel(host(dWd), dWd_ref) <= TOL[bf16]


def test_moe_errors(dh):
    with pytest.raises(dh.DhelixError):
        dh.dh_moe_route(4, 1, 1, 1, 1)
    with pytest.raises(dh.DhelixError):
        dh.dh_moe_gather_rows(dh.DH_F32, 4, 12, 1, 1, 1)
    tb, tbs = make_tables(dh, 4, 6, 2)
    with pytest.raises(dh.DhelixError):
        dh.dh_moe_plan(4, 6, 4, i32(8), tbs)
