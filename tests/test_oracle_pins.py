"""Pins for the CPU oracle: each test fixes the oracle to something other than itself.

The paper prints no worked numeric example of a BRA layer, so the pins are the
definition restated as brute force, library routines on the special cases that the
paper names (k = S^2 is full attention, Sec. 3.4 footnote; a region attending only
itself is window attention), closed forms (constant image, delta LCE kernels, the
complexity formula Eq. 8), the pooling identity of Appendix A, and the shape
bookkeeping of Table 7 / Appendix D stored in tests/golden/paper_values.txt.
"""
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
from synthetic_inputs import CONFIGS, make_config_inputs, make_inputs
from bra_bruteforce import brute_force_image, region_of

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_values.txt")


def golden():
    out = {}
    with open(GOLDEN) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if "=" in line:
                key, val = (s.strip() for s in line.split("="))
                out[key] = [int(v) for v in val.split(",")]
    return out


TINY = [  # (H, W, C, heads, S, k)
    (4, 4, 4, 1, 2, 1), (4, 4, 4, 2, 2, 2), (4, 4, 8, 2, 2, 4), (6, 6, 4, 1, 3, 2),
    (6, 6, 8, 2, 3, 5), (8, 8, 8, 2, 4, 3), (8, 8, 8, 1, 2, 2), (6, 4, 4, 2, 2, 3),
    (8, 12, 8, 4, 4, 7),
]


@pytest.mark.parametrize("H,W,C,heads,S,k", TINY)
@pytest.mark.parametrize("precision", ["f64", "f32"])
def test_p1_brute_force_dense_masked(H, W, C, heads, S, k, precision):
    X, Wqkv, Wo, Wlce = make_inputs(2, H, W, C, seed=100 + H * 7 + S * 3 + k)
    scale = 0.37
    o = oracle.bra_forward(X, Wqkv, Wo, Wlce, S=S, k=k, heads=heads, scale=scale,
                           precision=precision)
    tol = 1e-10 if precision == "f64" else 2e-5
    for b in range(2):
        Y, I, A = brute_force_image(X[b], Wqkv, Wo, Wlce, S, k, heads, scale)
        np.testing.assert_allclose(o["Ar"][b], A, atol=tol)
        if precision == "f64":
            np.testing.assert_array_equal(o["Ir"][b], I)
            np.testing.assert_allclose(o["Y"][b], Y, atol=tol)
        else:  # float rounding may swap a near-tie: compare on the oracle's routing
            Y2, _, _ = brute_force_image(X[b], Wqkv, Wo, Wlce, S, k, heads, scale,
                                         Ir_forced=o["Ir"][b])
            np.testing.assert_allclose(o["Y"][b], Y2, atol=tol)


def _torch_mhsa_lce(X, Wqkv, Wo, Wlce, heads, window=None):
    """Library routines: SDPA (default scale 1/sqrt(d)), conv2d, matmul."""
    B, H, W, C = X.shape
    d = C // heads
    x = torch.from_numpy(X).double()
    qkv = x.reshape(B, H * W, C) @ torch.from_numpy(Wqkv).double()
    q, k, v = qkv.split(C, dim=-1)

    def heads_first(t):
        return t.reshape(B, H * W, heads, d).transpose(1, 2)

    if window is None:
        o = F.scaled_dot_product_attention(heads_first(q), heads_first(k), heads_first(v))
        o = o.transpose(1, 2).reshape(B, H, W, C)
    else:
        rh, rw = window

        def win(t):  # [B,N,C] -> [B*nwin, heads, rh*rw, d]
            t = t.reshape(B, H // rh, rh, W // rw, rw, heads, d)
            return t.permute(0, 1, 3, 5, 2, 4, 6).reshape(-1, heads, rh * rw, d)

        o = F.scaled_dot_product_attention(win(q), win(k), win(v))
        o = o.reshape(B, H // rh, W // rw, heads, rh, rw, d).permute(0, 1, 4, 2, 5, 3, 6)
        o = o.reshape(B, H, W, C)
    vmap = v.reshape(B, H, W, C).permute(0, 3, 1, 2)
    lce = F.conv2d(vmap, torch.from_numpy(Wlce).double().unsqueeze(1), padding=2, groups=C)
    o = o + lce.permute(0, 2, 3, 1)
    return (o @ torch.from_numpy(Wo).double()).numpy()


@pytest.mark.parametrize("H,W,C,heads,S", [(14, 14, 64, 2, 7), (8, 8, 32, 1, 2), (12, 6, 64, 2, 3)])
def test_p2_k_equals_S2_is_full_attention(H, W, C, heads, S):
    X, Wqkv, Wo, Wlce = make_inputs(2, H, W, C, seed=7)
    o = oracle.bra_forward(X, Wqkv, Wo, Wlce, S=S, k=S * S, heads=heads)
    ref = _torch_mhsa_lce(X, Wqkv, Wo, Wlce, heads)
    np.testing.assert_allclose(o["Y"], ref, atol=1e-10)
    # every row of the routing index is a permutation of all regions
    assert np.all(np.sort(o["Ir"], axis=-1) == np.arange(S * S))


@pytest.mark.parametrize("H,W,C,heads,S", [(14, 14, 64, 2, 7), (8, 16, 32, 1, 4), (28, 28, 64, 2, 7)])
def test_p3_forced_self_routing_is_window_attention(H, W, C, heads, S):
    X, Wqkv, Wo, Wlce = make_inputs(2, H, W, C, seed=11)
    R = S * S
    Ir = np.broadcast_to(np.arange(R, dtype=np.int32)[None, :, None], (2, R, 1))
    o = oracle.bra_forward(X, Wqkv, Wo, Wlce, S=S, k=1, heads=heads, Ir_in=Ir)
    ref = _torch_mhsa_lce(X, Wqkv, Wo, Wlce, heads, window=(H // S, W // S))
    np.testing.assert_allclose(o["Y"], ref, atol=1e-10)


def test_p4_softmax_rows_and_convex_combination():
    H = W = 8; C = 8; heads = 2; S = 4; k = 3
    X, Wqkv, Wo, Wlce = make_inputs(2, H, W, C, seed=3)
    o = oracle.bra_forward(X, Wqkv, Wo, Wlce, S=S, k=k, heads=heads, want=("P", "Oatt"))
    P = o["P"]
    assert P.shape == (2, heads, S * S, 4, k * 4)
    assert np.all(P >= 0)
    np.testing.assert_allclose(P.sum(-1), 1.0, atol=1e-12)
    # the attention output of a token lies between the min and max of the V rows
    # of its routed regions, channel by channel
    V = X.astype(np.float64).reshape(2, H * W, C) @ Wqkv[:, 2 * C:].astype(np.float64)
    reg = region_of(H, W, S)
    Oatt = o["Oatt"].reshape(2, H * W, C)
    for b in range(2):
        for t in range(H * W):
            rows = np.isin(reg, o["Ir"][b, reg[t]])
            assert rows.sum() == k * 4
            assert np.all(Oatt[b, t] <= V[b, rows].max(0) + 1e-12)
            assert np.all(Oatt[b, t] >= V[b, rows].min(0) - 1e-12)


def test_p5_p6_pooling_identity_and_linearity():
    """Appendix A: mean pairwise affinity == affinity of the means; and pooling
    commutes with the projection (mean is linear)."""
    H, W, C, S = 6, 9, 8, 3
    X, Wqkv, Wo, Wlce = make_inputs(1, H, W, C, seed=5)
    o = oracle.bra_forward(X, Wqkv, Wo, Wlce, S=S, k=2, heads=2)
    x = X[0].astype(np.float64).reshape(-1, C)
    reg = region_of(H, W, S)
    Q, K = x @ Wqkv[:, :C].astype(np.float64), x @ Wqkv[:, C:2 * C].astype(np.float64)
    pair = Q @ K.T
    for i in range(S * S):
        for j in range(S * S):
            lhs = pair[np.ix_(reg == i, reg == j)].mean()
            assert abs(lhs - o["Ar"][0, i, j]) < 1e-12
    xr = np.stack([x[reg == r].mean(0) for r in range(S * S)])
    A_lin = (xr @ Wqkv[:, :C].astype(np.float64)) @ (xr @ Wqkv[:, C:2 * C].astype(np.float64)).T
    np.testing.assert_allclose(o["Ar"][0], A_lin, atol=1e-12)


def test_p7_constant_image_closed_form():
    H = W = 12; C = 8; heads = 2; S = 3; k = 4
    _, Wqkv, Wo, Wlce = make_inputs(1, H, W, C, seed=9)
    x0 = np.linspace(-1, 1, C).astype(np.float32)
    X = np.broadcast_to(x0, (1, H, W, C)).copy()
    o = oracle.bra_forward(X, Wqkv, Wo, Wlce, S=S, k=k, heads=heads, want=("Oatt", "Lce"))
    # all affinities equal -> ties resolve to the smallest indices, ascending
    assert np.ptp(o["Ar"]) < 1e-12
    assert np.all(o["Ir"] == np.arange(k))
    v = x0.astype(np.float64) @ Wqkv[:, 2 * C:].astype(np.float64)
    np.testing.assert_allclose(o["Oatt"], np.broadcast_to(v, (1, H, W, C)), atol=1e-12)
    # LCE = v_c * (sum of the taps whose input pixel lies inside the image)
    Wl = Wlce.astype(np.float64)
    for (y, x) in [(0, 0), (0, 5), (1, 1), (5, 5), (11, 11), (11, 0), (6, 10)]:
        kys = [ky for ky in range(5) if 0 <= y + ky - 2 < H]
        kxs = [kx for kx in range(5) if 0 <= x + kx - 2 < W]
        s = Wl[:, kys][:, :, kxs].sum((1, 2))
        np.testing.assert_allclose(o["Lce"][0, y, x], v * s, atol=1e-12)


def test_p8_lce_kernel_orientation_and_isolation():
    H = W = 8; C = 4; S = 2; k = 2
    X, Wqkv, _, _ = make_inputs(1, H, W, C, seed=13)
    Wo = np.eye(C, dtype=np.float32)
    V = (X[0].astype(np.float64).reshape(-1, C) @ Wqkv[:, 2 * C:].astype(np.float64)).reshape(H, W, C)
    base = oracle.bra_forward(X, Wqkv, Wo, np.zeros((C, 5, 5), np.float32), S=S, k=k, heads=1)
    # centre tap: LCE(V) = V
    Wl = np.zeros((C, 5, 5), np.float32); Wl[:, 2, 2] = 1
    o = oracle.bra_forward(X, Wqkv, Wo, Wl, S=S, k=k, heads=1)
    np.testing.assert_allclose(o["Y"][0] - base["Y"][0], V, atol=1e-12)
    # tap at (ky=0, kx=3): out[y, x] = V[y-2, x+1]  (cross-correlation, no flip)
    Wl = np.zeros((C, 5, 5), np.float32); Wl[:, 0, 3] = 1
    o = oracle.bra_forward(X, Wqkv, Wo, Wl, S=S, k=k, heads=1)
    exp = np.zeros_like(V)
    exp[2:, :-1] = V[:-2, 1:]
    np.testing.assert_allclose(o["Y"][0] - base["Y"][0], exp, atol=1e-12)
    # per-channel weights are not mixed across channels
    Wl = np.zeros((C, 5, 5), np.float32); Wl[1, 2, 2] = 2.5
    o = oracle.bra_forward(X, Wqkv, Wo, Wl, S=S, k=k, heads=1)
    exp = np.zeros_like(V); exp[:, :, 1] = 2.5 * V[:, :, 1]
    np.testing.assert_allclose(o["Y"][0] - base["Y"][0], exp, atol=1e-12)


def test_p9_permutation_equivariance():
    H = W = 8; C = 8; heads = 2; S = 4; k = 3
    rh = rw = 2
    X, Wqkv, Wo, _ = make_inputs(1, H, W, C, seed=17)
    Wl0 = np.zeros((C, 5, 5), np.float32)
    base = oracle.bra_forward(X, Wqkv, Wo, Wl0, S=S, k=k, heads=heads)
    rng = np.random.default_rng(0)
    # permute whole regions (blocks of the map)
    perm = rng.permutation(S * S)       # new region r holds old region perm[r]
    blocks = X[0].reshape(S, rh, S, rw, C).transpose(0, 2, 1, 3, 4).reshape(S * S, rh, rw, C)
    Xp = blocks[perm].reshape(S, S, rh, rw, C).transpose(0, 2, 1, 3, 4).reshape(1, H, W, C)
    o = oracle.bra_forward(np.ascontiguousarray(Xp), Wqkv, Wo, Wl0, S=S, k=k, heads=heads)
    Yb = base["Y"][0].reshape(S, rh, S, rw, C).transpose(0, 2, 1, 3, 4).reshape(S * S, rh, rw, C)
    Yp = o["Y"][0].reshape(S, rh, S, rw, C).transpose(0, 2, 1, 3, 4).reshape(S * S, rh, rw, C)
    np.testing.assert_allclose(Yp, Yb[perm], atol=1e-12)
    inv = np.argsort(perm)
    np.testing.assert_array_equal(o["Ir"][0], inv[base["Ir"][0][perm]])
    # permute the tokens inside one region: only that region's outputs move
    Xq = X.copy()
    Xq[0, 0:2, 0:2] = X[0, 0:2, 0:2][::-1, ::-1]
    o = oracle.bra_forward(Xq, Wqkv, Wo, Wl0, S=S, k=k, heads=heads)
    exp = base["Y"].copy()
    exp[0, 0:2, 0:2] = base["Y"][0, 0:2, 0:2][::-1, ::-1]
    np.testing.assert_allclose(o["Y"], exp, atol=1e-12)
    np.testing.assert_array_equal(o["Ir"], base["Ir"])


@pytest.mark.parametrize("idx", [1, 2, 3, 4, 5])
def test_p10_op_count_matches_complexity_formula(idx):
    """Eq. 8: FLOPs = 3HWC^2 + 2(S^2)^2 C + 2 HW k (HW/S^2) C, where the projection
    and attention terms count one per multiply-add and the routing term two."""
    cfg = CONFIGS[idx]
    if idx == 5:   # same formula, smaller map to keep the CPU suite short
        H = W = 32
    else:
        H, W = cfg.H, cfg.W
    X, Wqkv, Wo, Wlce = make_inputs(1, H, W, cfg.C, seed=1)
    o = oracle.bra_forward(X, Wqkv, Wo, Wlce, S=cfg.S, k=cfg.k, heads=cfg.heads, precision="f32")
    HW, C, S2 = H * W, cfg.C, cfg.S ** 2
    assert o["macs"][0] == 3 * HW * C * C
    assert 2 * o["macs"][1] == 2 * S2 * S2 * C
    assert o["macs"][2] == 2 * HW * cfg.k * (HW // S2) * C


def test_p10_tokens_to_attend_match_paper_tables():
    g = golden()
    maps = [56, 28, 14, 7]          # stage resolutions at 224^2 input
    for key, ks in [("tokens_to_attend_S7_k_1_4_16_49", (1, 4, 16, 49)),
                    ("tokens_to_attend_S7_k_1_2_8_32", (1, 2, 8, 32)),
                    ("tokens_to_attend_S7_k_2_8_32_49", (2, 8, 32, 49))]:
        assert [k * (m // 7) ** 2 for k, m in zip(ks, maps)] == g[key]
    assert 12 * (32 // 8) ** 2 == g["vit_adaptation_tokens"][0]
    for idx in (2, 3, 4):           # the benchmark's stage shapes attend 64 tokens
        assert CONFIGS[idx].kn == g["tokens_to_attend_S7_k_1_4_16_49"][idx - 2]
    assert all(c.d == g["head_channels"][0] for c in CONFIGS.values())
    # P has exactly k*n columns
    X, Wqkv, Wo, Wlce = make_inputs(1, 14, 14, 64, seed=2)
    o = oracle.bra_forward(X, Wqkv, Wo, Wlce, S=7, k=16, heads=2, want=("P",))
    assert o["P"].shape[-1] == 64


def test_p11_float_oracle_error_budget():
    cfg = CONFIGS[1]
    X, Wqkv, Wo, Wlce = make_config_inputs(cfg)
    o64 = oracle.bra_forward(X, Wqkv, Wo, Wlce, S=cfg.S, k=cfg.k, heads=cfg.heads)
    o32 = oracle.bra_forward(X, Wqkv, Wo, Wlce, S=cfg.S, k=cfg.k, heads=cfg.heads, precision="f32")
    assert np.abs(o32["Ar"] - o64["Ar"]).max() < 1e-5
    np.testing.assert_array_equal(o32["Ir"], o64["Ir"])
    assert np.abs(o32["Y"] - o64["Y"]).max() < 1e-5


def test_p12_topk_against_stable_argsort_with_ties():
    """Plant exact ties in the affinity by duplicating regions of the image."""
    H = W = 8; C = 8; S = 4
    X, Wqkv, Wo, Wlce = make_inputs(1, H, W, C, seed=23)
    # copy region (0,0) into regions (1,2) and (3,1): identical region keys -> equal columns
    X[0, 2:4, 4:6] = X[0, 0:2, 0:2]
    X[0, 6:8, 2:4] = X[0, 0:2, 0:2]
    for k in (1, 2, 5, 16):
        o = oracle.bra_forward(X, Wqkv, Wo, Wlce, S=S, k=k, heads=2)
        A = o["Ar"][0]
        assert np.all(A[:, 0] == A[:, 6]) and np.all(A[:, 0] == A[:, 13])
        ref = np.argsort(-A, axis=1, kind="stable")[:, :k]
        np.testing.assert_array_equal(o["Ir"][0], ref)


def test_scale_argument_and_default():
    X, Wqkv, Wo, Wlce = make_inputs(1, 8, 8, 64, seed=29)
    a = oracle.bra_forward(X, Wqkv, Wo, Wlce, S=2, k=2, heads=2)
    b = oracle.bra_forward(X, Wqkv, Wo, Wlce, S=2, k=2, heads=2, scale=1 / np.sqrt(32))
    np.testing.assert_array_equal(a["Y"], b["Y"])
    c = oracle.bra_forward(X, Wqkv, Wo, Wlce, S=2, k=2, heads=2, scale=1.0)
    assert np.abs(a["Y"] - c["Y"]).max() > 1e-3


def test_invalid_shapes_rejected():
    X, Wqkv, Wo, Wlce = make_inputs(1, 8, 8, 8, seed=1)
    for kw in (dict(S=3, k=1, heads=2), dict(S=2, k=5, heads=2), dict(S=2, k=1, heads=3),
               dict(S=2, k=0, heads=2)):
        with pytest.raises(ValueError):
            oracle.bra_forward(X, Wqkv, Wo, Wlce, **kw)
