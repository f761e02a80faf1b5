"""Pins for the MoE part of oracle/layer_ref.py."""
import numpy as np

from oracle import layer_ref as R

rng = np.random.default_rng(77)


def fd_grad(f, x, h=1e-6):
    g = np.zeros_like(x)
    it = np.nditer(x, flags=["multi_index"])
    for _ in it:
        i = it.multi_index
        old = x[i]
        x[i] = old + h; fp = f()
        x[i] = old - h; fm = f()
        x[i] = old
        g[i] = (fp - fm) / (2 * h)
    return g


def relerr(a, b):
    return np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300)


def test_router_top2_against_argsort_and_special_cases():
    logits = rng.standard_normal((50, 16))
    idx, prob = R.router_top2(logits)
    top = np.argsort(-logits, axis=1, kind="stable")[:, :2]
    assert np.array_equal(idx, top)
    assert np.allclose(prob.sum(axis=1), 1.0, atol=1e-15)
    # renormalised softmax over all experts == softmax over the two kept logits
    sm = np.exp(logits) / np.exp(logits).sum(axis=1, keepdims=True)
    kept = np.take_along_axis(sm, idx, axis=1)
    assert np.allclose(prob, kept / kept.sum(axis=1, keepdims=True), atol=1e-14)
    # all logits equal: experts (0, 1) with weights (1/2, 1/2); ties go to the lower id
    i2, p2 = R.router_top2(np.zeros((3, 8)))
    assert np.array_equal(i2, np.tile([0, 1], (3, 1))) and np.allclose(p2, 0.5)
    i3, _ = R.router_top2(np.array([[1.0, 3.0, 3.0, 0.0]]))
    assert i3.tolist() == [[1, 2]]


def test_router_bwd_finite_differences():
    logits = rng.standard_normal((6, 5))
    w = rng.standard_normal((6, 2))
    idx, prob = R.router_top2(logits)
    dl = R.router_top2_bwd(w, idx, prob, 5)
    f = lambda: float(np.sum(R.router_top2(logits)[1] * w))
    assert relerr(dl, fd_grad(f, logits)) < 1e-7
    assert np.allclose(dl.sum(axis=1), 0.0, atol=1e-14)      # shifting all logits changes nothing


def test_permute_and_dispatch_are_permutations():
    logits = rng.standard_normal((40, 16))
    idx, _ = R.router_top2(logits)
    dest, src, counts = R.permute_rows(idx, 16)
    assert sorted(dest.reshape(-1).tolist()) == list(range(80)) and counts.sum() == 80
    for t in range(40):
        for k in range(2):
            assert src[dest[t, k]] == t
    experts_in_row_order = [int(idx[src[r], list(dest[src[r]]).index(r)]) for r in range(80)]
    assert experts_in_row_order == sorted(experts_in_row_order)
    order, group_rows = R.a2a_dispatch_order(counts, 2)
    assert sorted(order.tolist()) == list(range(80)) and sum(group_rows) == 80
    # receive rows of local expert 0 hold exactly the assignments to the even logical experts
    got = sorted(experts_in_row_order[r] for r in order[: group_rows[0]])
    assert all(e % 2 == 0 for e in got) and len(got) == counts[0::2].sum()
    x = rng.standard_normal((80, 3))
    back = np.zeros_like(x); back[order] = x[order]
    assert np.array_equal(back, x)


def test_moe_equals_dense_mlp_when_experts_share_weights():
    T, H, F = 12, 8, 6
    h2 = rng.standard_normal((T, H)); logits = rng.standard_normal((T, 16))
    W1 = 0.3 * rng.standard_normal((H, 2 * F)); W2 = 0.3 * rng.standard_normal((F, H))
    y, _ = R.moe_ffn_fwd(h2, logits, np.stack([W1, W1]), np.stack([W2, W2]), 2)
    gu = h2 @ W1
    dense = R.swiglu_fwd(gu[:, :F], gu[:, F:]) @ W2
    assert np.allclose(y, dense, atol=1e-13)                 # gate weights sum to one


def test_moe_bwd_finite_differences():
    T, H, F, E = 7, 6, 4, 8
    h2 = rng.standard_normal((T, H)); logits = rng.standard_normal((T, E))
    Wgu = 0.4 * rng.standard_normal((2, H, 2 * F)); Wd = 0.4 * rng.standard_normal((2, F, H))
    w = rng.standard_normal((T, H))
    y, saved = R.moe_ffn_fwd(h2, logits, Wgu, Wd, 2)
    dh2, dlogits, dWgu, dWd = R.moe_ffn_bwd(w, h2, Wgu, Wd, saved, 2)
    f = lambda: float(np.sum(R.moe_ffn_fwd(h2, logits, Wgu, Wd, 2)[0] * w))
    assert relerr(dh2, fd_grad(f, h2)) < 1e-6
    assert relerr(dlogits, fd_grad(f, logits)) < 1e-6
    assert relerr(dWgu, fd_grad(f, Wgu)) < 1e-6
    assert relerr(dWd, fd_grad(f, Wd)) < 1e-6
