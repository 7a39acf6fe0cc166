"""Pins of the whole-block oracle (oracle/block.py) against things other than itself:
library routines in float64 (torch's convolution, layer norm, GELU, linear), brute-force
loops on tiny inputs, closed-form values and structural special cases (Sec. 3.4)."""
import math

import numpy as np
import torch

import oracle
from oracle import block as ob
from synthetic_inputs import make_block_params, make_inputs


def _rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def test_pos_encoding_matches_library_depthwise_convolution():
    r = _rng(1)
    X = r.standard_normal((2, 6, 9, 5))
    Wp = r.standard_normal((5, 3, 3))
    bp = r.standard_normal(5)
    got = ob.pos_encoding(X, Wp, bp)
    xt = torch.from_numpy(X).permute(0, 3, 1, 2)
    conv = torch.nn.functional.conv2d(xt, torch.from_numpy(Wp)[:, None], torch.from_numpy(bp), padding=1, groups=5)
    ref = (xt + conv).permute(0, 2, 3, 1).numpy()
    assert np.abs(got - ref).max() < 1e-12


def test_pos_encoding_brute_force_and_orientation():
    # an asymmetric kernel tells cross-correlation from convolution and ky from kx
    r = _rng(2)
    X = r.standard_normal((1, 4, 5, 2))
    Wp = r.standard_normal((2, 3, 3))
    bp = r.standard_normal(2)
    got = ob.pos_encoding(X, Wp, bp)
    for y in range(4):
        for x in range(5):
            for c in range(2):
                acc = X[0, y, x, c] + bp[c]
                for ky in range(3):
                    for kx in range(3):
                        yy, xx = y + ky - 1, x + kx - 1
                        if 0 <= yy < 4 and 0 <= xx < 5:
                            acc += Wp[c, ky, kx] * X[0, yy, xx, c]
                assert abs(got[0, y, x, c] - acc) < 1e-12
    # a kernel that is 1 at (ky, kx) = (0, 1) copies the token above
    Wd = np.zeros((2, 3, 3)); Wd[:, 0, 1] = 1.0
    sh = ob.pos_encoding(X, Wd, np.zeros(2)) - X
    assert np.allclose(sh[0, 1:], X[0, :-1]) and np.all(sh[0, 0] == 0)


def test_layer_norm_library_and_invariants():
    r = _rng(3)
    X = 3.0 * r.standard_normal((2, 3, 4, 16)) + 1.5
    g = r.standard_normal(16); b = r.standard_normal(16)
    got = ob.layer_norm(X, g, b, 1e-6)
    ref = torch.nn.functional.layer_norm(torch.from_numpy(X), (16,), torch.from_numpy(g), torch.from_numpy(b), 1e-6).numpy()
    assert np.abs(got - ref).max() < 1e-12
    plain = ob.layer_norm(X, np.ones(16), np.zeros(16), 0.0)
    assert np.abs(plain.mean(-1)).max() < 1e-12 and np.abs((plain ** 2).mean(-1) - 1).max() < 1e-12
    # shifting and scaling a token does not change its normalised form (eps = 0)
    assert np.abs(ob.layer_norm(7.0 * X - 2.0, np.ones(16), np.zeros(16), 0.0) - plain).max() < 1e-11
    # closed form: the token (0, 2) has mean 1, variance 1
    two = ob.layer_norm(np.array([[0.0, 2.0]]), np.array([2.0, 3.0]), np.array([0.5, -0.5]), 0.0)
    assert np.allclose(two, [[-1.5, 2.5]])
    # eps sits inside the root: a constant token maps to beta, and (0, 2) with eps = 3 halves
    assert np.allclose(ob.layer_norm(np.full((1, 4), 5.0), np.ones(4), np.full(4, 0.25), 1e-6), 0.25)
    assert np.allclose(ob.layer_norm(np.array([[0.0, 2.0]]), np.ones(2), np.zeros(2), 3.0), [[-0.5, 0.5]])


def test_gelu_closed_forms_and_library():
    t = np.linspace(-6, 6, 241)
    g = ob.gelu(t)
    assert g[120] == 0.0
    assert np.abs(g - ob.gelu(-t) - t).max() < 1e-12          # x Phi(x) + x Phi(-x) = x
    assert abs(ob.gelu(1.0) - 0.8413447460685429) < 1e-12    # Phi(1)
    assert abs(ob.gelu(-1.0) + 0.15865525393145707) < 1e-12
    ref = torch.nn.functional.gelu(torch.from_numpy(t)).numpy()
    assert np.abs(g - ref).max() < 1e-12
    phi = np.array([0.5 * math.erfc(-x / math.sqrt(2.0)) for x in t])
    assert np.abs(g - t * phi).max() < 1e-12


def test_mlp_matches_library_linear_layers():
    r = _rng(4)
    T = r.standard_normal((3, 5, 8))
    W1 = r.standard_normal((8, 24)); b1 = r.standard_normal(24)
    W2 = r.standard_normal((24, 8)); b2 = r.standard_normal(8)
    got = ob.mlp(T, W1, b1, W2, b2)
    tt = torch.from_numpy(T)
    h = torch.nn.functional.gelu(torch.nn.functional.linear(tt, torch.from_numpy(W1).T, torch.from_numpy(b1)))
    ref = torch.nn.functional.linear(h, torch.from_numpy(W2).T, torch.from_numpy(b2)).numpy()
    assert np.abs(got - ref).max() < 1e-12


def _small_block(seed=5, C=16, heads=2, S=2, H=4, W=6, B=2):
    X, Wqkv, Wo, Wlce = make_inputs(B, H, W, C, seed=seed)
    P = make_block_params(C, 3 * C, seed=seed + 1)
    P.update(Wqkv=Wqkv, Wo=Wo, Wlce=Wlce)
    return X, P, dict(S=S, k=2, heads=heads)


def test_block_composition_against_library_modules():
    """The block's wiring: every stage but BRA redone with torch's float64 modules."""
    X, P, kw = _small_block()
    out = ob.block_forward(X, P, eps=1e-5, **kw)
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    C = X.shape[-1]
    xt = t(X).permute(0, 3, 1, 2)
    x1 = (xt + torch.nn.functional.conv2d(xt, t(P["Wpos"])[:, None], t(P["bpos"]), padding=1, groups=C)).permute(0, 2, 3, 1)
    xn = torch.nn.functional.layer_norm(x1, (C,), t(P["ln1_g"]), t(P["ln1_b"]), 1e-5)
    y = oracle.bra_forward(xn.numpy(), P["Wqkv"], P["Wo"], P["Wlce"], precision="f64", **kw)["Y"]
    x2 = x1 + t(y)
    h = torch.nn.functional.layer_norm(x2, (C,), t(P["ln2_g"]), t(P["ln2_b"]), 1e-5)
    h = torch.nn.functional.gelu(h @ t(P["W1"]) + t(P["b1"]))
    x3 = x2 + h @ t(P["W2"]) + t(P["b2"])
    assert np.abs(out["X1"] - x1.numpy()).max() < 1e-12
    assert np.abs(out["Xn"] - xn.numpy()).max() < 1e-12
    assert np.abs(out["X2"] - x2.numpy()).max() < 1e-11
    assert np.abs(out["Xout"] - x3.numpy()).max() < 1e-11


def test_block_structural_special_cases():
    X, P, kw = _small_block(seed=9)
    Xd = X.astype(np.float64)
    # every branch switched off: the three residual links leave X unchanged
    Z = dict(P)
    Z.update(Wpos=np.zeros_like(P["Wpos"]), bpos=np.zeros_like(P["bpos"]), Wo=np.zeros_like(P["Wo"]),
             W2=np.zeros_like(P["W2"]), b2=np.zeros_like(P["b2"]))
    assert np.array_equal(ob.block_forward(X, Z, **kw)["Xout"], Xd)
    # only b2 on: a constant per channel is added once
    Z["b2"] = P["b2"]
    assert np.abs(ob.block_forward(X, Z, **kw)["Xout"] - (Xd + P["b2"])).max() < 1e-12
    # only the position encoding on: the output is pos_encoding(X)
    Z["b2"] = np.zeros_like(P["b2"]); Z["Wpos"] = P["Wpos"]; Z["bpos"] = P["bpos"]
    assert np.abs(ob.block_forward(X, Z, **kw)["Xout"] - ob.pos_encoding(X, P["Wpos"], P["bpos"])).max() < 1e-12
    # BRA sees the normalised tensor, not X1: rescaling X1's tokens (eps = 0) leaves BRA's output alone
    Z = dict(P); Z.update(Wpos=np.zeros_like(P["Wpos"]), bpos=np.zeros_like(P["bpos"]))
    a = ob.block_forward(X, Z, eps=0.0, **kw)
    b = ob.block_forward(4.0 * X, Z, eps=0.0, **kw)
    assert np.abs(a["Y"] - b["Y"]).max() < 1e-9
    assert np.abs(b["X2"] - (4.0 * Xd + a["Y"])).max() < 1e-9
    # the MLP branch reads LayerNorm2(X2): with gamma2 = 0 its input is beta2 for every token
    Z = dict(P); Z["ln2_g"] = np.zeros_like(P["ln2_g"])
    o = ob.block_forward(X, Z, **kw)
    const = ob.mlp(P["ln2_b"].astype(np.float64), P["W1"], P["b1"], P["W2"], P["b2"])
    assert np.abs(o["Xout"] - (o["X2"] + const)).max() < 1e-12


def test_block_bf16_store_rounds_only_the_tensor_that_enters_bra():
    X, P, kw = _small_block(seed=11)
    a = ob.block_forward(X, P, store="bf16", **kw)
    bits = np.ascontiguousarray(a["Xn"], dtype=np.float32).view(np.uint32)
    assert a["Xn"].dtype == np.float64 and not np.any(bits & np.uint32(0xFFFF))
    b = ob.block_forward(X, P, **kw)
    assert np.array_equal(a["X1"], b["X1"])
    assert 0 < np.abs(a["Xn"] - b["Xn"]).max() <= 2.0 ** -8 * np.abs(b["Xn"]).max()
