"""Seeded synthetic inputs for the Bi-Level Routing Attention (BRA) forward path.

This module is the only code shared by the CPU oracle's tests and the HIP path's
tests / benchmark.  It draws random tensors and rounds them; it contains none of
the method's arithmetic.

The five named workloads are the BiFormer stage shapes (head width 32, top-k of
1 / 4 / 16 per stage, S = 7 for 224^2 classification inputs and S = 8 for 512^2
dense-prediction inputs; paper Sec. 3.4 and Table 1).  The paper's own inputs are
feature maps of ImageNet / ADE20K images, which are not available here; i.i.d.
Gaussian tensors of the same shapes stand in for them.

Recipe (config index c = 1..5): rng = numpy Generator(PCG64(20230308 + c)); drawn
in this order as float32: X[B,H,W,C] ~ N(0,1); Wq, Wk, Wv, Wo [C,C] ~ N(0,1)/sqrt(C);
Wlce[C,5,5] ~ N(0,1)/5; Wqkv = concat([Wq, Wk, Wv], axis=1).  For bf16 workloads
every array is rounded once to bf16 (round-to-nearest-even); both sides then see
exactly the same real values.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np

BASE_SEED = 20230308


@dataclass(frozen=True)
class BraConfig:
    name: str
    index: int          # 1-based workload index, also the seed offset
    B: int
    H: int
    W: int
    C: int
    heads: int
    S: int
    k: int
    dtype: str          # "f32" or "bf16": storage type of X, weights and Y

    @property
    def R(self) -> int:
        return self.S * self.S

    @property
    def n(self) -> int:
        return (self.H // self.S) * (self.W // self.S)

    @property
    def d(self) -> int:
        return self.C // self.heads

    @property
    def kn(self) -> int:
        return self.k * self.n

    def with_batch(self, B: int) -> "BraConfig":
        return replace(self, B=B)


CONFIGS = {
    1: BraConfig("cfg1_single_layer_f32", 1, 1, 28, 28, 64, 2, 7, 4, "f32"),
    2: BraConfig("cfg2_stage1_224", 2, 64, 56, 56, 64, 2, 7, 1, "bf16"),
    3: BraConfig("cfg3_stage2_224", 3, 64, 28, 28, 128, 4, 7, 4, "bf16"),
    4: BraConfig("cfg4_stage3_224", 4, 64, 14, 14, 256, 8, 7, 16, "bf16"),
    5: BraConfig("cfg5_dense_512", 5, 2, 128, 128, 64, 2, 8, 4, "bf16"),
}


# Further operating points of the paper (not benchmark configurations): the last stage of the
# backbones (7x7 map, S = 7: one token per region, k = S^2 is full attention) at C = 512, the
# third stage of the wider variant (C = 384), the plain-ViT adaptation of the appendix (32x32
# map, S = 8, k = 12, 12 heads of 64 channels) and S = 16 on a detection-sized first-stage map
# (a size that S divides: the paper pads otherwise).
NEXT_CONFIGS = {
    6: BraConfig("next_stage4_224", 6, 64, 7, 7, 512, 16, 7, 49, "bf16"),
    7: BraConfig("next_wide_stage3_224", 7, 64, 14, 14, 384, 12, 7, 16, "bf16"),
    8: BraConfig("next_vit_adaptation", 8, 8, 32, 32, 768, 12, 8, 12, "bf16"),
    9: BraConfig("next_detection_s16", 9, 2, 208, 304, 64, 2, 16, 4, "bf16"),
}


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even); returns float32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    return r.view(np.float32).reshape(a.shape)


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """Upper 16 bits of float32 values that are already bf16-representable."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    assert not np.any(u & np.uint32(0xFFFF)), "value is not bf16-representable"
    return (u >> np.uint32(16)).astype(np.uint16).reshape(a.shape)


def bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Inverse of bf16_bits."""
    u = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).reshape(bits.shape)


def make_inputs(B, H, W, C, *, seed, dtype="f32", smooth=False, S=None):
    """Draw X, Wqkv, Wo, Wlce (float32 arrays; bf16-representable if dtype == "bf16").

    smooth=True adds a per-region random offset (std 1) to X so that routing
    concentrates on a few regions; it needs S.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    X = rng.standard_normal((B, H, W, C), dtype=np.float32)
    Wq, Wk, Wv, Wo = (rng.standard_normal((C, C), dtype=np.float32) / np.float32(np.sqrt(C))
                      for _ in range(4))
    Wlce = rng.standard_normal((C, 5, 5), dtype=np.float32) / np.float32(5.0)
    if smooth:
        assert S is not None
        off = rng.standard_normal((B, S, S, C), dtype=np.float32)
        X = X + np.repeat(np.repeat(off, H // S, axis=1), W // S, axis=2)
    Wqkv = np.concatenate([Wq, Wk, Wv], axis=1)
    out = [X, Wqkv, Wo, Wlce]
    if dtype == "bf16":
        out = [round_to_bf16(a) for a in out]
    elif dtype != "f32":
        raise ValueError(dtype)
    return tuple(np.ascontiguousarray(a, dtype=np.float32) for a in out)


def make_config_inputs(cfg: BraConfig, *, batch=None, smooth=False):
    """Inputs of a named workload; `batch` draws only the first `batch` images.

    The first `batch` images are identical to those of the full draw because X is
    drawn image-major before the weights only when batch == cfg.B; to keep the
    weights independent of `batch`, the full X stream is always consumed.
    """
    B = cfg.B
    X, Wqkv, Wo, Wlce = make_inputs(B, cfg.H, cfg.W, cfg.C, seed=BASE_SEED + cfg.index,
                                    dtype=cfg.dtype, smooth=smooth, S=cfg.S)
    if batch is not None and batch < B:
        X = np.ascontiguousarray(X[:batch])
    return X, Wqkv, Wo, Wlce


def make_block_params(C, hidden, *, seed, dtype="f32"):
    """Draw the parameters a whole BiFormer block has beyond BRA's own (Sec. 3.4): the 3x3
    depth-wise position encoding, two LayerNorms and the 2-layer MLP (hidden = e C channels).

    rng = numpy Generator(PCG64(seed)); drawn in this order as float32: Wpos[C,3,3] ~ N(0,1)/3,
    bpos[C] ~ 0.1 N(0,1), ln1_g = 1 + 0.1 N(0,1), ln1_b ~ 0.1 N(0,1), ln2_g, ln2_b likewise,
    W1[C,hidden] ~ N(0,1)/sqrt(C), b1[hidden] ~ 0.1 N(0,1), W2[hidden,C] ~ N(0,1)/sqrt(hidden),
    b2[C] ~ 0.1 N(0,1).  The matrices (Wpos, W1, W2) are rounded to bf16 for bf16 workloads; the
    vectors stay float32 on both sides.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    n = lambda *shape: rng.standard_normal(shape, dtype=np.float32)
    P = {}
    P["Wpos"] = n(C, 3, 3) / np.float32(3.0)
    P["bpos"] = np.float32(0.1) * n(C)
    P["ln1_g"] = np.float32(1.0) + np.float32(0.1) * n(C)
    P["ln1_b"] = np.float32(0.1) * n(C)
    P["ln2_g"] = np.float32(1.0) + np.float32(0.1) * n(C)
    P["ln2_b"] = np.float32(0.1) * n(C)
    P["W1"] = n(C, hidden) / np.float32(np.sqrt(C))
    P["b1"] = np.float32(0.1) * n(hidden)
    P["W2"] = n(hidden, C) / np.float32(np.sqrt(hidden))
    P["b2"] = np.float32(0.1) * n(C)
    if dtype == "bf16":
        for key in ("Wpos", "W1", "W2"):
            P[key] = round_to_bf16(P[key])
    elif dtype != "f32":
        raise ValueError(dtype)
    return {key: np.ascontiguousarray(v, dtype=np.float32) for key, v in P.items()}


def make_block_inputs(cfg: BraConfig, *, batch=None, expansion=3):
    """X and all parameters of one block at a named workload's shape (MLP expansion ratio
    e = 3, Sec. 3.4): BRA's tensors from make_config_inputs, the rest from make_block_params
    with seed BASE_SEED + 1000 + index."""
    X, Wqkv, Wo, Wlce = make_config_inputs(cfg, batch=batch)
    P = make_block_params(cfg.C, expansion * cfg.C, seed=BASE_SEED + 1000 + cfg.index, dtype=cfg.dtype)
    P.update(Wqkv=Wqkv, Wo=Wo, Wlce=Wlce)
    return X, P
