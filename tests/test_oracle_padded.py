"""Pins of the oracle's padded variant (maps whose sides S does not divide) against a brute force
that never builds a padded tensor: it works on the real tokens only and accounts for the appended
zero tokens analytically (they add nothing to a region's sums but count in its size; as keys they
have logit 0 and value 0, so each adds exp(0) to a softmax denominator and nothing to its
numerator; for the 5x5 depth-wise term they are indistinguishable from its zero padding)."""
import numpy as np
from scipy.signal import correlate2d

import oracle
from synthetic_inputs import make_inputs


def phantom_brute_force(X, Wqkv, Wo, Wlce, S, k, heads):
    H, W, C = X.shape
    rh, rw = -(-H // S), -(-W // S)                 # region sides on the padded map
    n, R, d = rh * rw, S * S, C // heads
    X = X.astype(np.float64)
    Wq, Wk, Wv = (Wqkv[:, i * C:(i + 1) * C].astype(np.float64) for i in range(3))
    Q, K, V = X @ Wq, X @ Wk, X @ Wv                # [H, W, C], real tokens only
    reg = (np.arange(H)[:, None] // rh) * S + np.arange(W)[None, :] // rw
    real = np.array([(reg == r).sum() for r in range(R)])
    Qr = np.stack([Q[reg == r].sum(0) / n for r in range(R)])
    Kr = np.stack([K[reg == r].sum(0) / n for r in range(R)])
    A = Qr @ Kr.T
    I = np.argsort(-A, axis=1, kind="stable")[:, :k]
    O = np.zeros((H, W, C))
    for y in range(H):
        for x in range(W):
            routed = I[reg[y, x]]
            keys = np.isin(reg, routed)
            phantoms = int(sum(n - real[r] for r in routed))
            for h in range(heads):
                c = slice(h * d, (h + 1) * d)
                s = (K[keys][:, c] @ Q[y, x, c]) / np.sqrt(d)
                e = np.exp(s)
                O[y, x, c] = (e[:, None] * V[keys][:, c]).sum(0) / (e.sum() + phantoms)
    for ch in range(C):
        O[:, :, ch] += correlate2d(V[:, :, ch], Wlce[ch].astype(np.float64), mode="same")
    return O @ Wo.astype(np.float64), I, A


def test_padded_oracle_matches_phantom_key_brute_force():
    for (H, W, S, k, seed) in [(5, 7, 2, 2, 1), (7, 4, 3, 3, 2), (6, 9, 2, 1, 3)]:
        X, Wqkv, Wo, Wlce = make_inputs(2, H, W, 8, seed=seed)
        out = oracle.bra_forward_padded(X, Wqkv, Wo, Wlce, S=S, k=k, heads=2)
        assert out["Y"].shape == X.shape
        for b in range(2):
            Y, I, A = phantom_brute_force(X[b], Wqkv, Wo, Wlce, S, k, 2)
            assert np.abs(out["Ar"][b] - A).max() < 1e-12
            np.testing.assert_array_equal(out["Ir"][b], I)
            assert np.abs(out["Y"][b] - Y).max() < 1e-11


def test_padded_oracle_is_plain_oracle_when_s_divides():
    X, Wqkv, Wo, Wlce = make_inputs(1, 6, 8, 8, seed=5)
    a = oracle.bra_forward_padded(X, Wqkv, Wo, Wlce, S=2, k=2, heads=2)
    b = oracle.bra_forward(X, Wqkv, Wo, Wlce, S=2, k=2, heads=2)
    np.testing.assert_array_equal(a["Y"], b["Y"])
    np.testing.assert_array_equal(a["Ir"], b["Ir"])
