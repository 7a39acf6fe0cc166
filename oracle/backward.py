"""TEST INFRASTRUCTURE: CPU oracle for the backward pass of BRA, in float64 numpy.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this module.
It shares nothing with the HIP library.

What is differentiated is the layer of Sec. 3.2 / Algorithm 1 with the routing index I^r held
fixed (the top-k of Eq. 5 has no derivative; the paper trains through the token-level attention
only): Y = (Attention(Q, K^g, V^g) + LCE(V)) W^o with Q, K, V = X [W^q | W^k | W^v] (Eq. 2, 3, 6, 7).
Given dY = dLoss/dY the chain rule gives, per image (T_i = the tokens of region i, G_i = the
tokens of its routed regions in I^r order, per head h with P = softmax(scale Q_h[T_i] K_h[G_i]^T)):

    dO  = dY Wo^T                      dWo = O^T dY
    dV += LCE^T(dO)                    dWlce[c,ky,kx] = sum_{y,x} dO[y,x,c] V[y+ky-2, x+kx-2, c]
    dP  = dO_h[T_i] V_h[G_i]^T         dS = P * (dP - rowsum(P * dP))
    dQ_h[T_i] += scale dS K_h[G_i]     dK_h[G_i] += scale dS^T Q_h[T_i]     dV_h[G_i] += P^T dO_h[T_i]
    dX  = dQ Wq^T + dK Wk^T + dV Wv^T  dWqkv = X^T [dQ | dK | dV]

(weight gradients summed over the batch).  Every step is written out with plain numpy loops
over images, regions and heads.

Pins: tests/test_oracle_backward.py (torch's reverse-mode differentiation of an independently
written float64 forward, central finite differences of the forward oracle, closed forms).
"""
from __future__ import annotations

import numpy as np


def region_tokens(H, W, S):
    """Flat token indices (y * W + x) of every region, row-major inside the region: [S*S, n]."""
    rh, rw = H // S, W // S
    out = np.empty((S * S, rh * rw), dtype=np.int64)
    for ry in range(S):
        for rx in range(S):
            ys, xs = np.meshgrid(np.arange(ry * rh, (ry + 1) * rh), np.arange(rx * rw, (rx + 1) * rw), indexing="ij")
            out[ry * S + rx] = (ys * W + xs).reshape(-1)
    return out


def _lce(V, Wlce):
    """5x5 depth-wise cross-correlation of V [H,W,C], zero padding 2 (Eq. 7)."""
    H, W, C = V.shape
    Vp = np.zeros((H + 4, W + 4, C))
    Vp[2:H + 2, 2:W + 2] = V
    out = np.zeros_like(V)
    for ky in range(5):
        for kx in range(5):
            out += Vp[ky:ky + H, kx:kx + W] * Wlce[:, ky, kx]
    return out


def bra_backward(X, Wqkv, Wo, Wlce, dY, Ir, *, S, heads, scale=None):
    """Gradients of sum(Y * dY) for fixed routing.  X, dY [B,H,W,C]; Ir [B,S*S,k].
    Returns dict: dX [B,H,W,C], dWqkv [C,3C], dWo [C,C], dWlce [C,5,5], and Y (the forward result)."""
    X = np.asarray(X, dtype=np.float64)
    dY = np.asarray(dY, dtype=np.float64)
    Wqkv = np.asarray(Wqkv, dtype=np.float64)
    Wo = np.asarray(Wo, dtype=np.float64)
    Wlce = np.asarray(Wlce, dtype=np.float64)
    B, H, W, C = X.shape
    d = C // heads
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    toks = region_tokens(H, W, S)
    R = S * S
    dX = np.zeros_like(X)
    dWqkv = np.zeros_like(Wqkv)
    dWo = np.zeros_like(Wo)
    dWlce = np.zeros_like(Wlce)
    Yall = np.zeros_like(X)
    for b in range(B):
        x = X[b].reshape(H * W, C)
        qkv = x @ Wqkv
        Q, K, V = qkv[:, :C], qkv[:, C:2 * C], qkv[:, 2 * C:]
        # forward, keeping P
        Oatt = np.zeros((H * W, C))
        Ps = {}
        for i in range(R):
            Ti = toks[i]
            Gi = np.concatenate([toks[j] for j in Ir[b, i]])
            for h in range(heads):
                c = slice(h * d, (h + 1) * d)
                s = scale * Q[Ti][:, c] @ K[Gi][:, c].T
                s -= s.max(axis=1, keepdims=True)
                P = np.exp(s)
                P /= P.sum(axis=1, keepdims=True)
                Ps[(i, h)] = P
                Oatt[Ti, c] = P @ V[Gi][:, c]
        O = Oatt + _lce(V.reshape(H, W, C), Wlce).reshape(H * W, C)
        Yall[b] = (O @ Wo).reshape(H, W, C)
        # backward
        dy = dY[b].reshape(H * W, C)
        dO = dy @ Wo.T
        dWo += O.T @ dy
        dQ = np.zeros_like(Q)
        dK = np.zeros_like(K)
        dV = np.zeros_like(V)
        # LCE: dV[y, x] += sum_k w[k] dO[y - (ky - 2), x - (kx - 2)];  dW[k] = sum dO[y, x] V[y + ky - 2, x + kx - 2]
        dOm = dO.reshape(H, W, C)
        dOp = np.zeros((H + 4, W + 4, C))
        dOp[2:H + 2, 2:W + 2] = dOm
        Vp = np.zeros((H + 4, W + 4, C))
        Vp[2:H + 2, 2:W + 2] = V.reshape(H, W, C)
        dVm = np.zeros((H, W, C))
        for ky in range(5):
            for kx in range(5):
                dVm += dOp[4 - ky:4 - ky + H, 4 - kx:4 - kx + W] * Wlce[:, ky, kx]
                dWlce[:, ky, kx] += (dOm * Vp[ky:ky + H, kx:kx + W]).sum(axis=(0, 1))
        dV += dVm.reshape(H * W, C)
        for i in range(R):
            Ti = toks[i]
            Gi = np.concatenate([toks[j] for j in Ir[b, i]])
            for h in range(heads):
                c = slice(h * d, (h + 1) * d)
                P = Ps[(i, h)]
                dP = dO[Ti][:, c] @ V[Gi][:, c].T
                dS = P * (dP - (P * dP).sum(axis=1, keepdims=True))
                dQ[Ti, c] += scale * dS @ K[Gi][:, c]
                np.add.at(dK, (Gi[:, None], np.arange(h * d, (h + 1) * d)[None, :]), scale * dS.T @ Q[Ti][:, c])
                np.add.at(dV, (Gi[:, None], np.arange(h * d, (h + 1) * d)[None, :]), P.T @ dO[Ti][:, c])
        dqkv = np.concatenate([dQ, dK, dV], axis=1)
        dX[b] = (dqkv @ Wqkv.T).reshape(H, W, C)
        dWqkv += x.T @ dqkv
    return {"dX": dX, "dWqkv": dWqkv, "dWo": dWo, "dWlce": dWlce, "Y": Yall}
