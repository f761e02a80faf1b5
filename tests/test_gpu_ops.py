"""GPU parity of the single operators (through the C ABI) against the fp64 oracle, element by element
on the same seeded inputs.  Tolerances: relative L2 <= 1e-5 (fp32 storage) and <= 2e-2 (bf16)."""
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


def row_err(got, ref, width=None):
    """Largest error norm of a row against the row's own oracle norm, floored at the tensor's root-mean-square row
    norm (a whole-tensor norm hides one wrong row); width cuts the rows into pieces (one head of a token)."""
    if width is not None:
        got, ref = got.reshape(-1, width), ref.reshape(-1, width)
    d, n = np.linalg.norm(got - ref, axis=1), np.linalg.norm(ref, axis=1)
    floor = max(float(np.sqrt(np.mean(n * n))), 1e-30)
    return float((d / np.maximum(n, floor)).max())


ROW_TOL = {False: 2e-5, True: 3e-2}  # per row: fp32 storage, bf16 storage


def dt(dh, bf16):
    return dh.DH_BF16 if bf16 else dh.DH_F32


def tdtype(bf16):
    return torch.bfloat16 if bf16 else torch.float32


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("T,H", [(1, 8), (37, 256), (130, 4096), (19, 8192), (0, 64), (7, 16384)])  # 16384: the widest row
def test_rmsnorm_fwd_bwd(dh, bf16, T, H):
    x = gen.normal(1, (T, H), 1.0, 0.0, bf16); res = gen.normal(2, (T, H), 0.5, 0.0, bf16)
    g = gen.normal(3, (H,), 0.02, 1.0, bf16); dy = gen.normal(4, (T, H), 1e-2, 0.0, bf16)
    dres = gen.normal(5, (T, H), 1e-2, 0.0, bf16)
    xd, rd, gd, dyd, dresd = (dev(a, bf16) for a in (x, res, g, dy, dres))
    x2 = torch.empty_like(xd); h = torch.empty_like(xd); rstd = torch.empty(T, dtype=torch.float32, device="cuda")
    dh.dh_rmsnorm_fwd(dt(dh, bf16), T, H, xd, rd, gd, 1e-5, x2, h, rstd)
    dx = torch.empty_like(xd); dg = torch.full((H,), 0.25, dtype=torch.float32, device="cuda")
    wsb = dh.dh_rmsnorm_bwd_ws_bytes(T, H)
    ws = torch.empty(max(wsb, 16), dtype=torch.uint8, device="cuda")
    dh.dh_rmsnorm_bwd(dt(dh, bf16), T, H, dyd, x2, gd, rstd, dresd, dx, dg, ws, wsb)
    torch.cuda.synchronize()
    if T == 0:
        assert torch.all(dg == 0.25)
        return
    x2_ref = x.astype(np.float64) + res
    h_ref, r_ref = R.rmsnorm_fwd(x2_ref, g.astype(np.float64), 1e-5)
    assert rel(host(x2), x2_ref) <= TOL[bf16]
    assert rel(host(h), h_ref) <= TOL[bf16]
    assert rel(host(rstd), r_ref[:, 0]) <= TOL[bf16]
    # backward is checked at the stored (rounded) x2 and rstd the kernel itself read
    dx_ref, dg_ref = R.rmsnorm_bwd(dy.astype(np.float64), host(x2), g.astype(np.float64), host(rstd)[:, None])
    assert rel(host(dx), dx_ref + dres) <= TOL[bf16]
    assert rel(host(dg) - 0.25, dg_ref) <= TOL[bf16]
    rows = {"x2": row_err(host(x2), x2_ref), "h": row_err(host(h), h_ref), "dx": row_err(host(dx), dx_ref + dres)}
    print("rmsnorm T=%d H=%d bf16=%d worst per-row errors %r" % (T, H, bf16, rows), flush=True)
    assert max(rows.values()) <= ROW_TOL[bf16], rows
    # no residual: x_out untouched path
    h2 = torch.empty_like(xd)
    dh.dh_rmsnorm_fwd(dt(dh, bf16), T, H, xd, None, gd, 1e-5, None, h2, rstd)
    assert rel(host(h2), R.rmsnorm_fwd(x.astype(np.float64), g.astype(np.float64), 1e-5)[0]) <= TOL[bf16]


def test_rmsnorm_errors(dh):
    wide = torch.zeros(2, 16392, device="cuda"); r2 = torch.zeros(2, device="cuda")
    with pytest.raises(dh.DhelixError) as e:   # one chunk past the widest supported row
        dh.dh_rmsnorm_fwd(dh.DH_F32, 2, 16392, wide, None, wide, 1e-5, None, wide, r2)
    assert e.value.code == dh.DH_ERR_SHAPE
    x = torch.zeros(4, 12, device="cuda")
    with pytest.raises(dh.DhelixError) as e:
        dh.dh_rmsnorm_fwd(dh.DH_F32, 4, 12, x, None, x, 1e-5, None, x, x)
    assert e.value.code == dh.DH_ERR_SHAPE
    x = torch.zeros(16, 64, device="cuda"); r = torch.zeros(16, device="cuda")
    with pytest.raises(dh.DhelixError) as e:
        dh.dh_rmsnorm_bwd(dh.DH_F32, 16, 64, x, x, x, r, None, x, r, x, 16)
    assert e.value.code == dh.DH_ERR_WORKSPACE_TOO_SMALL


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("batch,seq,nh,d,extra", [(1, 128, 4, 64, 0), (2, 333, 5, 128, 256), (1, 4096, 2, 128, 128)])
def test_rope(dh, bf16, batch, seq, nh, d, extra):
    T = batch * seq
    stride = nh * d + extra
    t = gen.normal(9, (T, stride), 1.0, 0.0, bf16)
    td = dev(t, bf16)
    dh.dh_rope(dt(dh, bf16), T, seq, nh, d, stride, 10000.0, False, td)
    got = host(td)
    ref = R.rope(t[:, : nh * d].astype(np.float64).reshape(T, nh, d), seq, 10000.0).reshape(T, nh * d)
    assert rel(got[:, : nh * d], ref) <= (4e-3 if bf16 else 2e-6)
    assert np.array_equal(got[:, nh * d:], t[:, nh * d:].astype(np.float64))  # columns after the heads untouched
    if not bf16:
        dh.dh_rope(dt(dh, bf16), T, seq, nh, d, stride, 10000.0, True, td)
        assert rel(host(td)[:, : nh * d], t[:, : nh * d]) <= 2e-6


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("batch,seq,pos0,nh,d,extra", [(1, 9, 0, 3, 16, 0), (2, 130, 4096, 5, 128, 64), (1, 700, 37, 2, 64, 8)])
def test_rope_adjacent_pairs(dh, bf16, batch, seq, pos0, nh, d, extra):
    """Pairing (2i, 2i+1), at a position offset, forward and back."""
    T = batch * seq
    stride = nh * d + extra
    t = gen.normal(9, (T, stride), 1.0, 0.0, bf16)
    td = dev(t, bf16)
    dh.dh_rope_pairs(dt(dh, bf16), dh.DH_ROPE_ADJACENT, T, seq, pos0, nh, d, stride, 10000.0, False, td)
    got = host(td)
    ref = R.rope(t[:, : nh * d].astype(np.float64).reshape(T, nh, d), seq, 10000.0, pos0=pos0, pairing=1).reshape(T, nh * d)
    assert rel(got[:, : nh * d], ref) <= (4e-3 if bf16 else 2e-6)
    assert np.array_equal(got[:, nh * d:], t[:, nh * d:].astype(np.float64))
    if not bf16:
        dh.dh_rope_pairs(dt(dh, bf16), dh.DH_ROPE_ADJACENT, T, seq, pos0, nh, d, stride, 10000.0, True, td)
        assert rel(host(td)[:, : nh * d], t[:, : nh * d]) <= 2e-6
    with pytest.raises(dh.DhelixError):
        dh.dh_rope_pairs(dt(dh, bf16), 2, T, seq, pos0, nh, d, stride, 10000.0, False, td)


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("T,F", [(5, 8), (77, 688), (256, 1792)])
def test_swiglu_and_add(dh, bf16, T, F):
    gu = gen.normal(11, (T, 2 * F), 2.0, 0.0, bf16); da = gen.normal(12, (T, F), 1.0, 0.0, bf16)
    gud, dad = dev(gu, bf16), dev(da, bf16)
    a = torch.empty(T, F, dtype=tdtype(bf16), device="cuda"); dgu = torch.empty_like(gud)
    dh.dh_swiglu_fwd(dt(dh, bf16), T, F, gud, a)
    dh.dh_swiglu_bwd(dt(dh, bf16), T, F, gud, dad, dgu)
    g64, u64 = gu[:, :F].astype(np.float64), gu[:, F:].astype(np.float64)
    assert rel(host(a), R.swiglu_fwd(g64, u64)) <= (4e-3 if bf16 else 1e-6)
    dg, du = R.swiglu_bwd(da.astype(np.float64), g64, u64)
    assert rel(host(dgu), np.concatenate([dg, du], axis=1)) <= (4e-3 if bf16 else 1e-6)
    out = torch.empty_like(gud)
    dh.dh_add(dt(dh, bf16), T * 2 * F, gud, dgu, out)
    assert rel(host(out), gu.astype(np.float64) + host(dgu)) <= (4e-3 if bf16 else 1e-7)


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("n,R_", [(8, 1), (128 * 256, 2), (1000 * 8, 8), (3 * 1024 * 1024 + 8, 8)])
def test_comm_standin_allreduce(dh, bf16, n, R_):
    parts = [gen.normal(20 + r, (n,), 1.0, 0.0, bf16) for r in range(R_)]
    pd = [dev(p, bf16) for p in parts]
    out = torch.empty(n, dtype=tdtype(bf16), device="cuda")
    dh.dh_comm_standin(dh.DH_COMM_ALLREDUCE, pd, out, n, dt(dh, bf16), n_blocks=(0 if R_ % 2 else 3))
    ref = R.standin_sum(parts[0].astype(np.float64), np.stack(parts[1:]) if R_ > 1 else None)
    if bf16:
        assert np.array_equal(host(out), gen.round_bf16(ref.astype(np.float32)).astype(np.float64)) or rel(host(out), ref) <= 4e-3
    else:
        # fp32 sum in index order: identical to the same sum done in float32 on the host
        acc = parts[0].copy()
        for r in range(1, R_):
            acc = acc + parts[r]
        assert np.array_equal(host(out), acc.astype(np.float64))
        assert rel(host(out), ref) <= 1e-6


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("kind", ["DH_COMM_A2A_DISPATCH", "DH_COMM_A2A_COMBINE"])
def test_comm_standin_a2a_equal_split(dh, bf16, kind):
    n, R_ = 5000 * 8, 8
    parts = [gen.normal(60 + r, (n,), 1.0, 0.0, bf16) for r in range(R_)]
    pd = [dev(p, bf16) for p in parts]
    out = torch.empty(n * R_, dtype=tdtype(bf16), device="cuda")
    dh.dh_comm_standin(getattr(dh, kind), pd, out, n, dt(dh, bf16), n_blocks=5)
    assert np.array_equal(host(out), np.concatenate(parts).astype(np.float64))  # a copy: exact


def test_comm_standin_errors_and_masked_stream(dh):
    a = torch.zeros(64, device="cuda")
    with pytest.raises(dh.DhelixError):
        dh.dh_comm_standin(dh.DH_COMM_ALLREDUCE, [a], a, 12, dh.DH_F32)
    with pytest.raises(dh.DhelixError):
        dh.dh_comm_standin(5, [a], a, 64, dh.DH_F32)
    with pytest.raises(dh.DhelixError) as e:  # a dtype outside {DH_F32, DH_BF16} is refused, not run as float32
        dh.dh_comm_standin(dh.DH_COMM_ALLREDUCE, [a], a, 64, 2)
    assert e.value.code == dh.DH_ERR_INVALID_ARG
    with pytest.raises(dh.DhelixError) as e:  # the kernels use 16-byte accesses
        dh.dh_comm_standin(dh.DH_COMM_ALLREDUCE, [a[1:33]], a, 32, dh.DH_F32)
    assert e.value.code == dh.DH_ERR_INVALID_ARG
    with pytest.raises(dh.DhelixError) as e:
        dh.dh_comm_standin(dh.DH_COMM_ALLREDUCE, [a], a[1:33], 32, dh.DH_F32)
    assert e.value.code == dh.DH_ERR_INVALID_ARG
    with pytest.raises(dh.DhelixError):
        dh.dh_stream_create_masked(0)
    try:
        s = dh.dh_stream_create_masked(16)
    except dh.DhelixError as e:   # systems that forbid compute-unit masks report it cleanly
        assert e.code == dh.DH_ERR_UNSUPPORTED
        assert float(torch.zeros(4, device="cuda").sum()) == 0.0   # and leave no HIP error behind
        return
    try:
        parts = [torch.full((4096,), float(r + 1), device="cuda") for r in range(4)]
        out = torch.empty(4096, device="cuda")
        torch.cuda.synchronize()
        dh.dh_comm_standin(dh.DH_COMM_ALLREDUCE, parts, out, 4096, dh.DH_F32, 0, s)
        torch.cuda.synchronize()
        assert torch.all(out == 10.0)
    finally:
        dh.dh_stream_destroy(s)


def gemm_ref(A, B, ta, tb):
    A = A.astype(np.float64); B = B.astype(np.float64)
    return (A.T if ta else A) @ (B.T if tb else B)


@pytest.mark.parametrize("ta,tb", [(0, 0), (0, 1), (1, 0), (1, 1)])
@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (64, 64, 16), (130, 75, 53), (257, 688, 256), (0, 8, 8), (8, 8, 0)])
def test_gemm_f32(dh, ta, tb, M, N, K):
    A = gen.normal(30, (K, M) if ta else (M, K)); B = gen.normal(31, (N, K) if tb else (K, N))
    Ad, Bd = dev(A, False), dev(B, False)
    Cd = torch.full((M, N), 0.5, dtype=torch.float32, device="cuda")
    dh.dh_gemm(dh.DH_F32, ta, tb, M, N, K, Ad, Bd, Cd)
    ref = gemm_ref(A, B, ta, tb) if K > 0 else np.zeros((M, N))
    if M * N:
        assert rel(host(Cd), ref) <= 1e-5 or (K == 0 and np.all(host(Cd) == 0))
    dh.dh_gemm(dh.DH_F32, ta, tb, M, N, K, Ad, Bd, Cd, out_f32_accumulate=True)
    if M * N and K:
        assert rel(host(Cd), 2 * ref) <= 1e-5


BF16_SHAPES = [(8, 8, 8), (128, 128, 64), (256, 256, 128), (300, 264, 200), (1000, 768, 520), (2048, 1024, 512),
               (77, 4096, 1024), (512, 512, 4096), (0, 64, 64),
               (4096, 1792, 136), (3900, 1704, 200),  # these two take the 256x128 tile when A is row-major
               (4104, 4104, 2056)]  # 17 x 17 large tiles: the 33 of the last round are issued apart with K split


@pytest.mark.parametrize("ta,tb", [(0, 0), (0, 1), (1, 0)])
@pytest.mark.parametrize("M,N,K", BF16_SHAPES)
def test_gemm_bf16(dh, ta, tb, M, N, K):
    if ta and M % 8:
        M = (M + 7) // 8 * 8
    A = gen.normal(40, (K, M) if ta else (M, K), 1.0, 0.0, True); B = gen.normal(41, (N, K) if tb else (K, N), 0.05, 0.0, True)
    Ad, Bd = dev(A, True), dev(B, True)
    wsb = dh.dh_gemm_workspace_bytes(dh.DH_BF16, ta, tb, M, N, K)
    ws = torch.empty(max(wsb, 16), dtype=torch.uint8, device="cuda")
    Cd = torch.zeros((M, N), dtype=torch.bfloat16, device="cuda")
    dh.dh_gemm(dh.DH_BF16, ta, tb, M, N, K, Ad, Bd, Cd, False, ws, wsb)
    if M * N == 0:
        torch.cuda.synchronize()
        return
    ref = gemm_ref(A, B, ta, tb)
    assert rel(host(Cd), ref) <= 4e-3          # one bf16 rounding of an fp32-accumulated sum
    # float32 accumulate epilogue (weight-gradient form): C += A*B, twice
    Cf = torch.full((M, N), 1.0, dtype=torch.float32, device="cuda")
    dh.dh_gemm(dh.DH_BF16, ta, tb, M, N, K, Ad, Bd, Cf, True, ws, wsb)
    dh.dh_gemm(dh.DH_BF16, ta, tb, M, N, K, Ad, Bd, Cf, True, ws, wsb)
    assert rel(host(Cf) - 1.0, 2 * ref) <= 2e-5
    # without workspace (no split-K) the result agrees to rounding
    Cn = torch.zeros((M, N), dtype=torch.float32, device="cuda")
    dh.dh_gemm(dh.DH_BF16, ta, tb, M, N, K, Ad, Bd, Cn, True, None, 0)
    assert rel(host(Cn), ref) <= 2e-5


# T, F, H.  The forward fusion needs at least 128 tiles of 256x256 (the first shape has too few: the error path), the
# backward one runs with each of the three tile shapes; K of 2, 3 and 5 ring steps and a long one; the Llama-8B
# shard's width (14 column tiles).
GLU_SHAPES = [(512, 256, 64), (4096, 1024, 96), (2048, 2048, 160), (4096, 2048, 64), (4096, 1792, 1024)]


@pytest.mark.parametrize("T,F,H", GLU_SHAPES)
def test_gemm_swiglu_fused(dh, T, F, H):
    """SwiGLU inside the GEMM epilogues (operator ACT of the layer merged into FC1 / FC2's data gradient): bit-identical to the
    GEMM followed by the row-wise kernel, and both within tolerance of the fp64 definition."""
    x = gen.normal(60, (T, H), 1.0, 0.0, True); w1 = gen.normal(61, (H, 2 * F), 0.05, 0.0, True)
    wd = gen.normal(62, (F, H), 0.05, 0.0, True); dy = gen.normal(63, (T, H), 1.0, 0.0, True)
    xd, w1d, wdd, dyd = dev(x, True), dev(w1, True), dev(wd, True), dev(dy, True)
    mk = lambda *shape: torch.zeros(shape, dtype=torch.bfloat16, device="cuda")
    wsb = max(dh.dh_gemm_workspace_bytes(dh.DH_BF16, 0, 0, T, 2 * F, H), dh.dh_gemm_workspace_bytes(dh.DH_BF16, 0, 1, T, F, H))
    ws = torch.empty(max(wsb, 16), dtype=torch.uint8, device="cuda")
    # forward: separate operators, then fused
    gu0, a0 = mk(T, 2 * F), mk(T, F)
    dh.dh_gemm(dh.DH_BF16, 0, 0, T, 2 * F, H, xd, w1d, gu0, False, ws, wsb)
    dh.dh_swiglu_fwd(dh.DH_BF16, T, F, gu0, a0)
    ref_gu = x.astype(np.float64) @ w1.astype(np.float64)
    g, u = ref_gu[:, :F], ref_gu[:, F:]
    ref_a = g / (1 + np.exp(-g)) * u
    assert rel(host(gu0), ref_gu) <= 4e-3 and rel(host(a0), ref_a) <= 2e-2
    print("fwd fits:", dh.dh_gemm_swiglu_fwd_fits(T, F, H), " bwd fits:", dh.dh_gemm_swiglu_bwd_fits(T, F, H), flush=True)
    if dh.dh_gemm_swiglu_fwd_fits(T, F, H):
        gu1, a1 = mk(T, 2 * F), mk(T, F)
        dh.dh_gemm_swiglu_fwd(T, F, H, xd, w1d, gu1, a1)
        assert torch.equal(gu0, gu1) and torch.equal(a0, a1)
    else:
        with pytest.raises(dh.DhelixError) as e:
            dh.dh_gemm_swiglu_fwd(T, F, H, xd, w1d, mk(T, 2 * F), mk(T, F))
        assert e.value.code == dh.DH_ERR_UNSUPPORTED
    # backward
    da0, dgu0 = mk(T, F), mk(T, 2 * F)
    dh.dh_gemm(dh.DH_BF16, 0, 1, T, F, H, dyd, wdd, da0, False, ws, wsb)
    dh.dh_swiglu_bwd(dh.DH_BF16, T, F, gu0, da0, dgu0)
    gq = host(gu0).astype(np.float64)   # the gradient at the stored gate/up values
    g, u = gq[:, :F], gq[:, F:]
    sg = 1 / (1 + np.exp(-g))
    ref_da = dy.astype(np.float64) @ wd.astype(np.float64).T
    ref_dgu = np.concatenate([ref_da * u * sg * (1 + g * (1 - sg)), ref_da * g * sg], axis=1)
    assert rel(host(dgu0), ref_dgu) <= 2e-2
    if dh.dh_gemm_swiglu_bwd_fits(T, F, H):
        dgu1 = mk(T, 2 * F)
        dh.dh_gemm_swiglu_bwd(T, F, H, dyd, wdd, gu0, dgu1)
        assert torch.equal(dgu0, dgu1)
    else:
        with pytest.raises(dh.DhelixError) as e:
            dh.dh_gemm_swiglu_bwd(T, F, H, dyd, wdd, gu0, mk(T, 2 * F))
        assert e.value.code == dh.DH_ERR_UNSUPPORTED


# trans_a, trans_b, M, N, K, accumulate: the weight-gradient form with each tile shape, the plain form, a ragged one
GEMM_AR_CASES = [(1, 0, 4096, 3584, 1024, True), (1, 0, 4096, 768, 1024, True), (0, 0, 4096, 1792, 512, False),
                 (0, 1, 2048, 4096, 256, False), (1, 0, 1000, 520, 264, True)]


@pytest.mark.parametrize("ta,tb,M,N,K,acc", GEMM_AR_CASES)
@pytest.mark.parametrize("n_ranks,n_blocks,elems", [(8, 64, 1 << 20), (1, 1, 8), (3, 7, 40 * 1024 + 8), (4, 65536, 1 << 16)])
def test_gemm_allreduce_one_launch(dh, ta, tb, M, N, K, acc, n_ranks, n_blocks, elems):
    """A GEMM that carries an all-reduce stand-in in its launch (Sec. 6.3, closing remark of the Table 7 analysis): both
    results bit-identical to dh_gemm and dh_comm_standin run apart."""
    if not dh.dh_gemm_allreduce_fits(ta, tb, M, N, K):
        pytest.skip("this GEMM is not a single launch")
    A = gen.normal(80, (K, M) if ta else (M, K), 1.0, 0.0, True); B = gen.normal(81, (N, K) if tb else (K, N), 0.05, 0.0, True)
    Ad, Bd = dev(A, True), dev(B, True)
    parts = [dev(gen.normal(90 + r, (elems,), 1.0, 0.0, True), True) for r in range(n_ranks)]
    cdt = torch.float32 if acc else torch.bfloat16
    C0 = torch.full((M, N), 0.25, dtype=cdt, device="cuda"); C1 = C0.clone()
    out0 = torch.zeros(elems, dtype=torch.bfloat16, device="cuda"); out1 = torch.zeros_like(out0)
    dh.dh_gemm(dh.DH_BF16, ta, tb, M, N, K, Ad, Bd, C0, acc, None, 0)
    dh.dh_comm_standin(dh.DH_COMM_ALLREDUCE, parts, out0, elems, dh.DH_BF16, n_blocks)
    dh.dh_gemm_allreduce(ta, tb, M, N, K, Ad, Bd, C1, acc, parts, out1, elems, n_blocks)
    torch.cuda.synchronize()
    assert torch.equal(C0, C1) and torch.equal(out0, out1)
    ref = gemm_ref(A, B, ta, tb)
    assert rel(host(C1) - (0.25 if acc else 0.0), ref) <= (2e-5 if acc else 4e-3)
    ref_sum = np.zeros(elems, np.float32)
    for q in parts:
        ref_sum = ref_sum + host(q).astype(np.float32)    # rank order, float32, one rounding at the end
    assert np.array_equal(host(out1).astype(np.float32), gen.round_bf16(ref_sum))


def test_gemm_allreduce_rejects(dh):
    a = torch.zeros(64 * 64, dtype=torch.bfloat16, device="cuda")
    big = dh.dh_gemm_allreduce_fits(0, 0, 4104, 4104, 2056)   # needs a tail launch
    assert not big
    with pytest.raises(dh.DhelixError) as e:
        dh.dh_gemm_allreduce(0, 0, 4104, 4104, 2056, a, a, a, False, [a], a, 64, 4)
    assert e.value.code == dh.DH_ERR_UNSUPPORTED
    for kw in (dict(elems=12), dict(n_blocks=0), dict(parts=[])):
        with pytest.raises(dh.DhelixError):
            dh.dh_gemm_allreduce(0, 0, 64, 64, 64, a, a, a, False, kw.get("parts", [a]), a, kw.get("elems", 64), kw.get("n_blocks", 4))


def test_gemm_bf16_shape_errors(dh):
    a = torch.zeros(64 * 64, dtype=torch.bfloat16, device="cuda")
    for args in [(0, 0, 16, 12, 16), (0, 0, 16, 16, 12), (1, 0, 12, 16, 16), (1, 1, 16, 16, 16)]:
        with pytest.raises(dh.DhelixError) as e:
            dh.dh_gemm(dh.DH_BF16, args[0], args[1], args[2], args[3], args[4], a, a, a)
        assert e.value.code in (dh.DH_ERR_SHAPE, dh.DH_ERR_UNSUPPORTED)


@pytest.mark.parametrize("batch,seq,nq,nkv,d", [(1, 700, 4, 1, 128), (2, 300, 2, 2, 64), (1, 2100, 2, 1, 128)])
def test_attention_scores_rising_along_the_keys(dh, batch, seq, nq, nkv, d):
    """The matrix-core forward keeps a row's reference maximum until a tile outgrows it by 2^8 and only then rescales
    its accumulators.  Scores that climb by ~90 (base 2) along the keys make that happen about ten times per row, with
    probabilities above 1 in between; half of the heads keep ordinary scores.  Forward and backward against the fp64
    definition, row by row."""
    T = batch * seq
    nqkv = (nq + 2 * nkv) * d
    qkv = gen.normal(70, (T, nqkv), 1.0, 0.0, False)
    u = gen.normal(71, (d,), 1.0, 0.0, False)
    u /= np.linalg.norm(u)
    pos = np.tile(np.arange(seq), batch)[:, None]
    for h in range(0, nq, 2):      # every other query head looks along u with weight 8 sqrt(d)
        qkv[:, h * d:(h + 1) * d] = 0.1 * qkv[:, h * d:(h + 1) * d] + 8.0 * np.sqrt(d) * u
    for h in range(nkv):           # keys grow along u: score of key j ~ 8 * 8 j / seq = up to 64 (92 in base 2)
        c0 = (nq + h) * d
        qkv[:, c0:c0 + d] = qkv[:, c0:c0 + d] + (8.0 * pos / seq) * u
    qkv = gen.round_bf16(qkv)
    do = gen.normal(72, (T, nq * d), 1.0, 0.0, True)
    qd, dod = dev(qkv, True), dev(do, True)
    o = torch.empty(T, nq * d, dtype=torch.bfloat16, device="cuda")
    lse = torch.empty(nq, T, dtype=torch.float32, device="cuda")
    fwsb = dh.dh_attn_fwd_workspace_bytes(dh.DH_BF16, batch, seq, nq, nkv, d)
    fws = torch.empty(max(fwsb, 16), dtype=torch.uint8, device="cuda")
    dh.dh_attn_fwd(dh.DH_BF16, batch, seq, nq, nkv, d, qd, o, lse, fws, fwsb)
    o_ns = torch.empty_like(o); lse_ns = torch.empty_like(lse)
    dh.dh_attn_fwd(dh.DH_BF16, batch, seq, nq, nkv, d, qd, o_ns, lse_ns)
    q64 = qkv[:, : nq * d].astype(np.float64).reshape(T, nq, d)
    k64 = qkv[:, nq * d: (nq + nkv) * d].astype(np.float64).reshape(T, nkv, d)
    v64 = qkv[:, (nq + nkv) * d:].astype(np.float64).reshape(T, nkv, d)
    o_ref, lse_ref = R.attention_fwd(q64, k64, v64, batch, seq)
    assert lse_ref.max() > 40.0     # the scores did climb
    assert rel(host(o), o_ref.reshape(T, nq * d)) <= 1e-2 and rel(host(o_ns), o_ref.reshape(T, nq * d)) <= 1e-2
    # lse is tens here: bf16 operands put ~2^-9 relative error into a score, the statistic inherits it
    assert np.max(np.abs(host(lse) - lse_ref) / np.maximum(1.0, np.abs(lse_ref))) <= 2e-2
    assert np.max(np.abs(host(lse_ns) - lse_ref) / np.maximum(1.0, np.abs(lse_ref))) <= 2e-2
    dqkv = torch.zeros(T, nqkv, dtype=torch.bfloat16, device="cuda")
    delta = torch.empty(nq, T, dtype=torch.float32, device="cuda")
    wsb = dh.dh_attn_bwd_workspace_bytes(dh.DH_BF16, batch, seq, nq, nkv, d)
    ws = torch.empty(max(wsb, 16), dtype=torch.uint8, device="cuda")
    dh.dh_attn_bwd(dh.DH_BF16, batch, seq, nq, nkv, d, qd, o, dod, lse, dqkv, delta, ws, wsb)
    dq, dk, dv = R.attention_bwd(do.astype(np.float64).reshape(T, nq, d), q64, k64, v64, batch, seq)
    got = host(dqkv)
    rows = {"o": row_err(host(o), o_ref.reshape(T, nq * d), d), "o_unsplit": row_err(host(o_ns), o_ref.reshape(T, nq * d), d),
            "dv": row_err(got[:, (nq + nkv) * d:], dv.reshape(T, -1), d)}
    print("rising scores %r worst per-row errors %r; dq %.2e dk %.2e" % ((batch, seq, nq, nkv, d), rows,
          rel(got[:, : nq * d], dq.reshape(T, -1)), rel(got[:, nq * d: (nq + nkv) * d], dk.reshape(T, -1))), flush=True)
    assert max(rows.values()) <= ROW_TOL[True], rows
    assert rel(got[:, (nq + nkv) * d:], dv.reshape(T, -1)) <= 2e-2
    assert rel(got[:, : nq * d], dq.reshape(T, -1)) <= 2e-2
    assert rel(got[:, nq * d: (nq + nkv) * d], dk.reshape(T, -1)) <= 2e-2


ATTN_CASES = [  # batch, seq, nq, nkv, d
    (1, 1, 2, 1, 64), (1, 128, 4, 4, 64), (2, 200, 4, 2, 64), (1, 333, 4, 1, 128), (2, 512, 2, 1, 128), (1, 1100, 8, 2, 128),
    (1, 2100, 2, 1, 64)]


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("batch,seq,nq,nkv,d", ATTN_CASES)
def test_attention_fwd_bwd(dh, bf16, batch, seq, nq, nkv, d):
    T = batch * seq
    nqkv = (nq + 2 * nkv) * d
    qkv = gen.normal(50, (T, nqkv), 1.0, 0.0, bf16); do = gen.normal(51, (T, nq * d), 1.0, 0.0, bf16)
    qd, dod = dev(qkv, bf16), dev(do, bf16)
    o = torch.empty(T, nq * d, dtype=tdtype(bf16), device="cuda")
    lse = torch.empty(nq, T, dtype=torch.float32, device="cuda")
    fwsb = dh.dh_attn_fwd_workspace_bytes(dt(dh, bf16), batch, seq, nq, nkv, d)
    fws = torch.empty(max(fwsb, 16), dtype=torch.uint8, device="cuda")
    dh.dh_attn_fwd(dt(dh, bf16), batch, seq, nq, nkv, d, qd, o, lse, fws, fwsb)  # long rows split over several blocks
    o_ns = torch.empty_like(o); lse_ns = torch.empty_like(lse)
    dh.dh_attn_fwd(dt(dh, bf16), batch, seq, nq, nkv, d, qd, o_ns, lse_ns)       # no workspace: rows not split
    q64 = qkv[:, : nq * d].astype(np.float64).reshape(T, nq, d)
    k64 = qkv[:, nq * d: (nq + nkv) * d].astype(np.float64).reshape(T, nkv, d)
    v64 = qkv[:, (nq + nkv) * d:].astype(np.float64).reshape(T, nkv, d)
    o_ref, lse_ref = R.attention_fwd(q64, k64, v64, batch, seq)
    tol = 1e-2 if bf16 else 1e-5
    assert rel(host(o), o_ref.reshape(T, nq * d)) <= tol
    assert np.max(np.abs(host(lse) - lse_ref)) <= (2e-2 if bf16 else 1e-5)
    assert rel(host(o_ns), o_ref.reshape(T, nq * d)) <= tol
    assert np.max(np.abs(host(lse_ns) - lse_ref)) <= (2e-2 if bf16 else 1e-5)
    assert bf16 or fwsb == 0  # only the matrix-core kernel splits rows (when that shortens the launch)
    dqkv = torch.zeros(T, nqkv, dtype=tdtype(bf16), device="cuda")
    delta = torch.empty(nq, T, dtype=torch.float32, device="cuda")
    wsb = dh.dh_attn_bwd_workspace_bytes(dt(dh, bf16), batch, seq, nq, nkv, d)
    ws = torch.empty(max(wsb, 16), dtype=torch.uint8, device="cuda")
    dh.dh_attn_bwd(dt(dh, bf16), batch, seq, nq, nkv, d, qd, o, dod, lse, dqkv, delta, ws, wsb)
    dq, dk, dv = R.attention_bwd(do.astype(np.float64).reshape(T, nq, d), q64, k64, v64, batch, seq)
    got = host(dqkv)
    tol = 2e-2 if bf16 else 1e-5
    # dq, dk vanish identically when every row sees a single key (seq = 1): what is left is the rounding
    # of dP - delta, two equal sums taken in different orders, so measure against dv's scale then
    floor = np.linalg.norm(dv) if seq == 1 else 0.0

    def relf(a, b):
        return np.linalg.norm(a - b) / max(np.linalg.norm(b), floor)
    assert relf(got[:, : nq * d], dq.reshape(T, -1)) <= tol
    assert relf(got[:, nq * d: (nq + nkv) * d], dk.reshape(T, -1)) <= tol
    assert relf(got[:, (nq + nkv) * d:], dv.reshape(T, -1)) <= tol
    # row by row: one head of one token at a time
    rows = {"o": row_err(host(o), o_ref.reshape(T, nq * d), d), "o_unsplit": row_err(host(o_ns), o_ref.reshape(T, nq * d), d),
            "dv": row_err(got[:, (nq + nkv) * d:], dv.reshape(T, -1), d)}
    if seq > 1:
        rows["dq"] = row_err(got[:, : nq * d], dq.reshape(T, -1), d)
        rows["dk"] = row_err(got[:, nq * d: (nq + nkv) * d], dk.reshape(T, -1), d)
    print("attention %r bf16=%d worst per-row errors %r" % ((batch, seq, nq, nkv, d), bf16, rows), flush=True)
    assert max(rows.values()) <= ROW_TOL[bf16], rows
