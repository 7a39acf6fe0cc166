"""GPU parity of bra_backward (through the C ABI) against the float64 backward oracle, with the
routing index given to both sides.  Bars: float32 tensors, every gradient within 1e-4 of
max|gradient| (the float32 bar relative to the gradient's scale: sums over up to B*H*W tokens);
bf16 tensors (float32 arithmetic on bf16 inputs, dX rounded to bf16) within 2e-2 of max|gradient|
for dX and 1e-3 for the float32 weight gradients."""
import numpy as np
import pytest
import torch

import paper_2303_08810_amd as bra
from oracle import backward as obw
from parity_util import to_device, to_numpy
from synthetic_inputs import CONFIGS, make_config_inputs, make_inputs, round_to_bf16

pytestmark = pytest.mark.gpu

# (dtype, B, H, W, C, heads, S, k)
SHAPES = [
    ("f32", 1, 28, 28, 64, 2, 7, 4),
    ("f32", 2, 12, 20, 48, 3, 4, 3),
    ("f32", 2, 7, 7, 64, 1, 7, 49),
    ("f32", 3, 6, 9, 40, 5, 3, 2),
    ("f32", 1, 16, 16, 32, 1, 2, 4),
    ("bf16", 2, 14, 14, 64, 2, 7, 4),
    ("bf16", 1, 16, 24, 96, 3, 4, 2),
]


@pytest.mark.parametrize("dtype,B,H,W,C,heads,S,k", SHAPES)
def test_backward(dtype, B, H, W, C, heads, S, k):
    Xn, Wqkvn, Won, Wlcen = make_inputs(B, H, W, C, seed=6000 + H * W + C + k, dtype=dtype)
    compare_backward(Xn, Wqkvn, Won, Wlcen, dtype, heads, S, k)


def compare_backward(Xn, Wqkvn, Won, Wlcen, dtype, heads, S, k):
    B, H, W, C = Xn.shape
    print(f"backward case dtype={dtype} shape={(B, H, W, C)} heads={heads} S={S} k={k}", flush=True)
    r = np.random.Generator(np.random.PCG64(6001 + C))
    dYn = r.standard_normal(Xn.shape).astype(np.float32)
    if dtype == "bf16":
        dYn = round_to_bf16(dYn)
    Irn = np.stack([np.stack([r.permutation(S * S)[:k] for _ in range(S * S)]) for _ in range(B)]).astype(np.int32)
    X, Wqkv, Wo, Wlce, dY = (to_device(a, dtype) for a in (Xn, Wqkvn, Won, Wlcen, dYn))
    got = bra.bra_backward(X, Wqkv, Wo, Wlce, torch.from_numpy(Irn).cuda(), dY, S, heads)
    torch.cuda.synchronize()
    ref = obw.bra_backward(Xn, Wqkvn, Won, Wlcen, dYn, Irn, S=S, heads=heads)
    names = ("dX", "dWqkv", "dWo", "dWlce")
    for name, g in zip(names, got):
        gn = to_numpy(g).astype(np.float64).reshape(ref[name].shape)
        rel = float(np.abs(gn - ref[name]).max() / np.abs(ref[name]).max())
        tol = 1e-4 if dtype == "f32" else (2e-2 if name == "dX" else 1e-3)
        print(f"  {name}: max error {rel:.3e} of max|gradient|", flush=True)
        assert rel <= tol, f"{name}: {rel:.3e} > {tol}"


def random_backward_shapes(count, seed):
    import random
    rng = random.Random(seed)
    out = []
    while len(out) < count:
        S = rng.choice([1, 2, 3, 4, 5, 7])
        H, W = S * rng.choice([1, 2, 3, 4, 5, 9]), S * rng.choice([1, 2, 3, 4, 6])
        heads = rng.choice([1, 2, 3, 4])
        C = rng.choice([8, 16, 24, 32, 64]) * heads
        k = rng.choice([1, 2, 3, min(S * S, 5), S * S])
        n = (H // S) * (W // S)
        if k > S * S or H * W * C > 60000 or H * W * k * n * C > 3e7:
            continue
        out.append((rng.choice(["f32", "f32", "bf16"]), rng.choice([1, 2, 3]), H, W, C, heads, S, k))
    return out


@pytest.mark.parametrize("dtype,B,H,W,C,heads,S,k", random_backward_shapes(12, seed=20230311))
def test_backward_random_shapes(dtype, B, H, W, C, heads, S, k):
    test_backward(dtype, B, H, W, C, heads, S, k)


@pytest.mark.parametrize("idx", [1, 2, 3, 4, 5])
def test_backward_named_workloads_full_size(idx):
    # the five named workloads at their full sizes (random routing index, given to both sides)
    cfg = CONFIGS[idx]
    Xn, Wqkvn, Won, Wlcen = make_config_inputs(cfg)
    compare_backward(Xn, Wqkvn, Won, Wlcen, cfg.dtype, cfg.heads, cfg.S, cfg.k)


def test_backward_after_forward_uses_its_routing():
    B, H, W, C, heads, S, k = 2, 14, 14, 64, 2, 7, 4
    Xn, Wqkvn, Won, Wlcen = make_inputs(B, H, W, C, seed=6100)
    X, Wqkv, Wo, Wlce = (to_device(a, "f32") for a in (Xn, Wqkvn, Won, Wlcen))
    Y, Ir = bra.bra_forward(X, Wqkv, Wo, Wlce, S, k, heads, want_Ir=True)
    dY = torch.ones_like(Y)
    dX, dWqkv, dWo, dWlce = bra.bra_backward(X, Wqkv, Wo, Wlce, Ir, dY, S, heads)
    torch.cuda.synchronize()
    ref = obw.bra_backward(Xn, Wqkvn, Won, Wlcen, np.ones_like(Xn), Ir.cpu().numpy(), S=S, heads=heads)
    assert np.abs(to_numpy(Y) - ref["Y"]).max() < 1e-4
    assert np.abs(to_numpy(dX) - ref["dX"]).max() <= 1e-4 * np.abs(ref["dX"]).max()
    assert np.abs(to_numpy(dWo) - ref["dWo"]).max() <= 1e-4 * np.abs(ref["dWo"]).max()
