"""Brute-force statement of bi-level routing attention used to pin the oracle.

Formulated differently from the oracle on purpose: it never partitions tensors.
It works on the flat H*W token list of one image, computes the region affinity as
the mean of all token-pair dot products between two regions (the left-hand side of
the pooling identity, Appendix A), selects regions with a stable argsort, and runs
*dense* attention over all N tokens with a -inf mask on tokens outside the routed
regions.  LCE is scipy's 2-D cross-correlation.  float64 throughout.
"""
import numpy as np
from scipy.signal import correlate2d


def region_of(H, W, S):
    rh, rw = H // S, W // S
    ys, xs = np.meshgrid(np.arange(H), np.arange(W), indexing="ij")
    return ((ys // rh) * S + (xs // rw)).reshape(-1)


def brute_force_image(X, Wqkv, Wo, Wlce, S, k, heads, scale, Ir_forced=None):
    H, W, C = X.shape
    N, R, d = H * W, S * S, C // heads
    X = X.astype(np.float64).reshape(N, C)
    Wq, Wk, Wv = (Wqkv[:, i * C:(i + 1) * C].astype(np.float64) for i in range(3))
    Q, K, V = X @ Wq, X @ Wk, X @ Wv
    reg = region_of(H, W, S)
    members = [np.flatnonzero(reg == r) for r in range(R)]
    # affinity as the average token-to-token score between two regions
    A = np.zeros((R, R))
    for i in range(R):
        for j in range(R):
            tot = 0.0
            for t in members[i]:
                for u in members[j]:
                    tot += float(Q[t] @ K[u])
            A[i, j] = tot / (len(members[i]) * len(members[j]))
    if Ir_forced is None:
        I = np.argsort(-A, axis=1, kind="stable")[:, :k]
    else:
        I = np.asarray(Ir_forced)
    allowed = np.zeros((R, R), dtype=bool)
    for i in range(R):
        allowed[i, I[i]] = True
    mask = allowed[reg][:, reg]                      # [N, N]: may token t see token u
    O = np.zeros((N, C))
    for h in range(heads):
        sl = slice(h * d, (h + 1) * d)
        logits = (Q[:, sl] @ K[:, sl].T) * scale
        logits = np.where(mask, logits, -np.inf)
        logits -= logits.max(axis=1, keepdims=True)
        P = np.exp(logits)
        P /= P.sum(axis=1, keepdims=True)
        O[:, sl] = P @ V[:, sl]
    Vmap = V.reshape(H, W, C)
    L = np.stack([correlate2d(Vmap[:, :, c], Wlce[c].astype(np.float64), mode="same",
                              boundary="fill", fillvalue=0.0) for c in range(C)], axis=-1)
    Y = (O + L.reshape(N, C)) @ Wo.astype(np.float64)
    return Y.reshape(H, W, C), I.astype(np.int32), A
