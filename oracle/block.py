"""TEST INFRASTRUCTURE: CPU oracle for one whole BiFormer block (forward), in float64.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this
module.  It shares nothing with the HIP library.

The block (paper Sec. 3.4, Fig. 3): a 3x3 depth-wise convolution at its start encodes
relative position, then a BRA module and a 2-layer MLP with expansion ratio e follow
one another.  The figure that fixes the normalisation and the residual links is not
part of the text this was written from; the reading taken here is the usual pre-norm
residual form of the works the section cites:

    X1 = X  + DWConv3x3(X)                 (zero padding 1, stride 1, with bias)
    X2 = X1 + BRA(LayerNorm1(X1))          (Eq. 2-7; the BRA oracle of this package)
    X3 = X2 + MLP(LayerNorm2(X2)),  MLP(t) = GELU(t W1 + b1) W2 + b2

LayerNorm normalises each token over its C channels (biased variance, eps inside the
square root, affine gamma/beta); GELU is the exact form x Phi(x).

Every step is plain numpy on float64 arrays; BRA is the C oracle called in float64.
`store="bf16"` rounds the tensor that enters BRA to bf16.  It exists for ONE purpose: a
path that stores that tensor in bf16 takes the routing decision of Eq. 5 on the rounded
values, so the affinities its index is judged against must come from the same values.
Outputs are always compared against the default, `store="f64"` (no rounding anywhere).

Pins: tests/test_oracle_block.py (library convolution / layer norm / GELU in float64,
brute-force loops on tiny inputs, closed-form values, structural special cases).
"""
from __future__ import annotations

import numpy as np
from scipy.special import erf

from . import bra_forward


def pos_encoding(X, Wpos, bpos):
    """X + depth-wise 3x3 cross-correlation of X (zero padding 1) + bias.

    X [B,H,W,C]; Wpos [C,3,3] (channel, ky, kx); bpos [C].  Sec. 3.4.
    """
    X = np.asarray(X, dtype=np.float64)
    B, H, W, C = X.shape
    Xp = np.zeros((B, H + 2, W + 2, C), dtype=np.float64)
    Xp[:, 1:H + 1, 1:W + 1, :] = X
    out = X + np.asarray(bpos, dtype=np.float64)
    for ky in range(3):
        for kx in range(3):
            out = out + Xp[:, ky:ky + H, kx:kx + W, :] * np.asarray(Wpos, dtype=np.float64)[:, ky, kx]
    return out


def layer_norm(X, gamma, beta, eps):
    """Per-token normalisation over the last axis: (x - mean) / sqrt(var + eps) * gamma + beta."""
    X = np.asarray(X, dtype=np.float64)
    mean = X.mean(axis=-1, keepdims=True)
    var = ((X - mean) ** 2).mean(axis=-1, keepdims=True)
    return (X - mean) / np.sqrt(var + eps) * np.asarray(gamma, dtype=np.float64) + np.asarray(beta, dtype=np.float64)


def gelu(t):
    """Exact GELU: t * Phi(t), Phi the standard normal distribution function."""
    t = np.asarray(t, dtype=np.float64)
    return 0.5 * t * (1.0 + erf(t / np.sqrt(2.0)))


def mlp(T, W1, b1, W2, b2):
    """2-layer per-token MLP (Sec. 3.4): GELU(T W1 + b1) W2 + b2; W1 [C,E], W2 [E,C]."""
    Hd = gelu(np.asarray(T, dtype=np.float64) @ np.asarray(W1, dtype=np.float64) + np.asarray(b1, dtype=np.float64))
    return Hd @ np.asarray(W2, dtype=np.float64) + np.asarray(b2, dtype=np.float64)


def _round_bf16(a):
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return r.view(np.float32).astype(np.float64).reshape(np.shape(a))


def block_forward(X, P, *, S, k, heads, eps=1e-6, scale=None, Ir_in=None, store="f64", threads=1):
    """One BiFormer block.  P: dict with Wpos [C,3,3], bpos [C], ln1_g, ln1_b [C], Wqkv [C,3C],
    Wo [C,C], Wlce [C,5,5], ln2_g, ln2_b [C], W1 [C,E], b1 [E], W2 [E,C], b2 [C].

    Returns a dict: "X1", "Xn" (what enters BRA), "Y" (BRA's output), "X2", "Xout", "Ir", "Ar".
    """
    X1 = pos_encoding(X, P["Wpos"], P["bpos"])
    Xn = layer_norm(X1, P["ln1_g"], P["ln1_b"], eps)
    if store == "bf16":
        Xn = _round_bf16(Xn)
    elif store != "f64":
        raise ValueError(store)
    att = bra_forward(Xn, P["Wqkv"], P["Wo"], P["Wlce"], S=S, k=k, heads=heads, scale=scale, Ir_in=Ir_in,
                      precision="f64", threads=threads)
    X2 = X1 + att["Y"]
    Xout = X2 + mlp(layer_norm(X2, P["ln2_g"], P["ln2_b"], eps), P["W1"], P["b1"], P["W2"], P["b2"])
    return {"X1": X1, "Xn": Xn, "Y": att["Y"], "X2": X2, "Xout": Xout, "Ir": att["Ir"], "Ar": att["Ar"]}
