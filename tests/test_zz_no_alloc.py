"""dh_rmsnorm_bwd_noalloc (the entry point for callers that cannot allocate: its scratch is a static device array)
against dh_rmsnorm_bwd with a caller workspace, through the C ABI: bitwise, on two calls in a row, the second smaller
than the first, so that the array still holds the first call's partial rows when the second runs."""
import numpy as np
import pytest
import torch

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


def run_both(dh, bf16, T, H, seed):
    dt = dh.DH_BF16 if bf16 else dh.DH_F32
    x = dev(gen.normal(seed, (T, H), 1.0, 0.0, bf16), bf16)
    g = dev(gen.normal(seed + 1, (H,), 0.02, 1.0, bf16), bf16)
    dy = dev(gen.normal(seed + 2, (T, H), 1e-2, 0.0, bf16), bf16)
    dres = dev(gen.normal(seed + 3, (T, H), 1e-2, 0.0, bf16), bf16)
    h = torch.empty_like(x)
    rstd = torch.empty(T, dtype=torch.float32, device="cuda")
    dh.dh_rmsnorm_fwd(dt, T, H, x, None, g, 1e-5, None, h, rstd)
    wsb = dh.dh_rmsnorm_bwd_ws_bytes(T, H)
    ws = torch.empty(max(wsb, 16), dtype=torch.uint8, device="cuda")
    dx_a = torch.empty_like(x); dg_a = torch.full((H,), 0.5, dtype=torch.float32, device="cuda")
    dx_b = torch.empty_like(x); dg_b = torch.full((H,), 0.5, dtype=torch.float32, device="cuda")
    dh.dh_rmsnorm_bwd(dt, T, H, dy, x, g, rstd, dres, dx_a, dg_a, ws, wsb)
    dh.dh_rmsnorm_bwd_noalloc(dt, T, H, dy, x, g, rstd, dres, dx_b, dg_b)
    torch.cuda.synchronize()
    assert torch.equal(dx_a, dx_b)
    assert torch.equal(dg_a, dg_b)
    assert bool(torch.any(dg_b != 0.5))


@pytest.mark.parametrize("bf16", [True, False])
def test_noalloc_two_calls_second_smaller(dh, bf16):
    run_both(dh, bf16, 4096 if bf16 else 2048, 512, 11)  # 512 (fp32: 512) partial rows
    run_both(dh, bf16, 333, 256, 21)                     # fewer, narrower rows: stale partial rows lie behind them


def test_noalloc_limit(dh):
    assert dh.dh_rmsnorm_bwd_noalloc_max_bytes() == 8 << 20
    T, H = 8192, 4096  # 1024 partial rows of 16 KiB = 16 MiB
    assert dh.dh_rmsnorm_bwd_ws_bytes(T, H) > dh.dh_rmsnorm_bwd_noalloc_max_bytes()
    x = torch.zeros(8, device="cuda")
    with pytest.raises(dh.DhelixError) as e:  # refused before any pointer is touched
        dh.dh_rmsnorm_bwd_noalloc(dh.DH_F32, T, H, x, x, x, x, None, x, x)
    assert e.value.code == dh.DH_ERR_WORKSPACE_TOO_SMALL
