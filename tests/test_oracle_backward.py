"""Pins of the backward oracle (oracle/backward.py): torch's reverse-mode differentiation of a
forward written independently with torch operations in float64 (unfold-free: index gathers,
scaled_dot_product_attention-style softmax, conv2d for LCE), central finite differences of the
forward oracle (the C one), and closed forms."""
import numpy as np
import torch

import oracle
from oracle import backward as obw
from synthetic_inputs import make_inputs


def torch_forward(X, Wqkv, Wo, Wlce, Ir, S, heads):
    B, H, W, C = X.shape
    d = C // heads
    rh, rw = H // S, W // S
    qkv = X.reshape(B, H * W, C) @ Wqkv
    Q, K, V = qkv[..., :C], qkv[..., C:2 * C], qkv[..., 2 * C:]
    ids = torch.arange(H * W).reshape(S, rh, S, rw).permute(0, 2, 1, 3).reshape(S * S, rh * rw)   # region -> tokens
    out = torch.zeros(B, H * W, C, dtype=X.dtype)
    for b in range(B):
        for i in range(S * S):
            keys = ids[torch.as_tensor(Ir[b, i], dtype=torch.long)].reshape(-1)
            q = Q[b, ids[i]].reshape(-1, heads, d).transpose(0, 1)
            k = K[b, keys].reshape(-1, heads, d).transpose(0, 1)
            v = V[b, keys].reshape(-1, heads, d).transpose(0, 1)
            att = torch.softmax(q @ k.transpose(1, 2) / d ** 0.5, dim=-1) @ v
            out[b, ids[i]] = att.transpose(0, 1).reshape(-1, C)
    lce = torch.nn.functional.conv2d(V.reshape(B, H, W, C).permute(0, 3, 1, 2), Wlce[:, None], padding=2, groups=C)
    O = out + lce.permute(0, 2, 3, 1).reshape(B, H * W, C)
    return (O @ Wo).reshape(B, H, W, C)


def case(seed, B=2, H=6, W=8, C=8, heads=2, S=2, k=2):
    X, Wqkv, Wo, Wlce = make_inputs(B, H, W, C, seed=seed)
    r = np.random.Generator(np.random.PCG64(seed + 1))
    dY = r.standard_normal(X.shape)
    Ir = np.stack([np.stack([r.permutation(S * S)[:k] for _ in range(S * S)]) for _ in range(B)]).astype(np.int32)
    return X, Wqkv, Wo, Wlce, dY, Ir, dict(S=S, heads=heads)


def test_backward_matches_reverse_mode_differentiation():
    for seed, kw in [(1, {}), (2, dict(H=9, W=6, S=3, k=4, C=12, heads=3)), (3, dict(B=1, H=4, W=4, S=2, k=4, heads=1))]:
        X, Wqkv, Wo, Wlce, dY, Ir, skw = case(seed, **kw)
        got = obw.bra_backward(X, Wqkv, Wo, Wlce, dY, Ir, **skw)
        t = [torch.tensor(np.asarray(a, dtype=np.float64), requires_grad=True) for a in (X, Wqkv, Wo, Wlce)]
        Y = torch_forward(*t, Ir, skw["S"], skw["heads"])
        assert np.abs(Y.detach().numpy() - got["Y"]).max() < 1e-12
        (Y * torch.tensor(dY)).sum().backward()
        for name, ten in zip(("dX", "dWqkv", "dWo", "dWlce"), t):
            ref = ten.grad.numpy()
            assert np.abs(got[name] - ref).max() <= 1e-11 * max(1.0, np.abs(ref).max()), name


def test_backward_matches_finite_differences_of_the_forward_oracle():
    X, Wqkv, Wo, Wlce, dY, Ir, skw = case(5, B=1, H=4, W=6, C=8, heads=2, S=2, k=2)
    got = obw.bra_backward(X, Wqkv, Wo, Wlce, dY, Ir, **skw)
    k = Ir.shape[-1]

    def loss(Xa, Wa, Woa, Wl):
        return float((oracle.bra_forward(Xa, Wa, Woa, Wl, S=skw["S"], k=k, heads=skw["heads"], Ir_in=Ir,
                                         precision="f64")["Y"] * dY).sum())

    r = np.random.Generator(np.random.PCG64(6))
    args = [np.asarray(a, dtype=np.float64) for a in (X, Wqkv, Wo, Wlce)]
    for which, name in enumerate(("dX", "dWqkv", "dWo", "dWlce")):
        for _ in range(6):
            idx = tuple(int(r.integers(0, n)) for n in args[which].shape)
            eps = 1e-5
            plus = [a.copy() for a in args]; minus = [a.copy() for a in args]
            plus[which][idx] += eps; minus[which][idx] -= eps
            fd = (loss(*plus) - loss(*minus)) / (2 * eps)
            assert abs(fd - got[name][idx]) < 1e-6 * max(1.0, abs(fd)), (name, idx, fd, got[name][idx])


def test_backward_closed_forms():
    X, Wqkv, Wo, Wlce, dY, Ir, skw = case(7)
    C = X.shape[-1]
    # dWo = O^T dY and dX is linear in dY: doubling dY doubles every gradient
    a = obw.bra_backward(X, Wqkv, Wo, Wlce, dY, Ir, **skw)
    b = obw.bra_backward(X, Wqkv, Wo, Wlce, 2 * dY, Ir, **skw)
    for name in ("dX", "dWqkv", "dWo", "dWlce"):
        assert np.abs(b[name] - 2 * a[name]).max() < 1e-10
    # with Wv = 0 the value path is dead: nothing flows to Wq, Wk, Wlce, and dX = 0
    Wz = Wqkv.copy(); Wz[:, 2 * C:] = 0
    z = obw.bra_backward(X, Wz, Wo, Wlce, dY, Ir, **skw)
    assert np.abs(z["dWqkv"][:, :2 * C]).max() < 1e-12 and np.abs(z["dWlce"]).max() < 1e-12
    assert np.abs(z["dX"]).max() < 1e-12
    # one region attending to itself only (k = 1, one key per query region when n = 1): softmax over a
    # single key is constant, so Q and K get no gradient
    X1, W1, Wo1, Wl1, dY1, _, _ = case(8, B=1, H=2, W=2, C=4, heads=1, S=2, k=1)
    Iself = np.arange(4, dtype=np.int32).reshape(1, 4, 1)
    s = obw.bra_backward(X1, W1, Wo1, Wl1, dY1, Iself, S=2, heads=1)
    assert np.abs(s["dWqkv"][:, :8]).max() < 1e-12
