"""GPU parity of bra_backward (through the C ABI) against the float64 backward oracle, with the
routing index given to both sides.  Bars: float32 tensors, every gradient within 1e-4 of
max|gradient| (the float32 bar relative to the gradient's scale: sums over up to B*H*W tokens);
bf16 tensors within 2e-2 of max|gradient| for dX; their float32 weight gradients within 1e-3 on
the scalar kernels (float32 arithmetic on bf16 inputs) and within 1e-2 on the matrix-core kernels,
whose operands Q, K, V, P, dS, dO, dQ, dK, dV are each rounded to bf16 (relative error up to
2^-9 each, about 1.1e-3 rms): a gradient element is a sum over tokens of products that carry
five or so such roundings, so its error is about 2.5e-3 of a typical element in rms, and the
largest error over the matrix relative to the largest element is of that same size (measured:
3e-3 to 4e-3)."""
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


# bf16 shapes of the matrix-core backward (heads of 32 or 64 channels, C a multiple of 64): a full 64-key
# block, ragged key and query blocks (n = 49; k n = 48, 36, 2), one token per region, maps wider than
# one tile of the depth-wise kernel with a ragged last tile (W = 56, 40)
MFMA_SHAPES = [
    ("bf16", 2, 14, 14, 64, 2, 7, 4),
    ("bf16", 1, 56, 56, 64, 2, 7, 1),
    ("bf16", 2, 28, 28, 64, 2, 4, 1),
    ("bf16", 1, 16, 16, 128, 4, 4, 3),
    ("bf16", 2, 8, 8, 64, 2, 4, 9),
    ("bf16", 3, 4, 40, 128, 4, 4, 2),
    ("bf16", 1, 12, 20, 64, 2, 4, 4),
    ("bf16", 2, 7, 7, 128, 4, 7, 49),
    ("bf16", 2, 14, 14, 256, 8, 7, 16),
    ("bf16", 1, 16, 16, 256, 8, 2, 1),
    # more than 64 routed keys: key blocks taken twice by the query side; regions of more than 64 tokens
    ("bf16", 1, 32, 32, 64, 2, 4, 3),
    ("bf16", 2, 12, 20, 64, 2, 4, 16),
    ("bf16", 1, 20, 36, 128, 4, 2, 2),
    ("bf16", 1, 16, 24, 256, 8, 4, 5),
    ("bf16", 2, 7, 7, 64, 2, 7, 49),
    # wider layers: plain products for the projections
    ("bf16", 2, 14, 14, 384, 12, 7, 16),
    ("bf16", 1, 16, 24, 512, 16, 4, 3),
    ("bf16", 2, 7, 7, 512, 16, 7, 49),
    # other head counts (two heads or one per workgroup) and heads of 64 channels
    ("bf16", 2, 8, 8, 192, 6, 2, 2),
    ("bf16", 1, 12, 12, 320, 10, 3, 4),
    ("bf16", 2, 14, 14, 128, 2, 7, 4),
    ("bf16", 1, 16, 16, 64, 1, 2, 1),
    ("bf16", 1, 16, 24, 256, 4, 4, 5),
    ("bf16", 1, 20, 36, 192, 3, 2, 2),
    # 256 regions per image (1024 routing entries)
    ("bf16", 1, 32, 48, 64, 2, 16, 4),
]


@pytest.mark.parametrize("dtype,B,H,W,C,heads,S,k", SHAPES)
def test_backward(dtype, B, H, W, C, heads, S, k, path="generic"):
    Xn, Wqkvn, Won, Wlcen = make_inputs(B, H, W, C, seed=6000 + H * W + C + k, dtype=dtype)
    compare_backward(Xn, Wqkvn, Won, Wlcen, dtype, heads, S, k, path=path)


@pytest.mark.parametrize("dtype,B,H,W,C,heads,S,k", MFMA_SHAPES)
def test_backward_matrix_cores(dtype, B, H, W, C, heads, S, k):
    test_backward(dtype, B, H, W, C, heads, S, k, path="mfma")


def compare_backward(Xn, Wqkvn, Won, Wlcen, dtype, heads, S, k, path="auto"):
    B, H, W, C = Xn.shape
    print(f"backward case dtype={dtype} shape={(B, H, W, C)} heads={heads} S={S} k={k} path={path}", flush=True)
    r = np.random.Generator(np.random.PCG64(6001 + C))
    dYn = r.standard_normal(Xn.shape).astype(np.float32)
    if dtype == "bf16":
        dYn = round_to_bf16(dYn)
    Irn = np.stack([np.stack([r.permutation(S * S)[:k] for _ in range(S * S)]) for _ in range(B)]).astype(np.int32)
    X, Wqkv, Wo, Wlce, dY = (to_device(a, dtype) for a in (Xn, Wqkvn, Won, Wlcen, dYn))
    got = bra.bra_backward(X, Wqkv, Wo, Wlce, torch.from_numpy(Irn).cuda(), dY, S, heads, path=path)
    torch.cuda.synchronize()
    ref = obw.bra_backward(Xn, Wqkvn, Won, Wlcen, dYn, Irn, S=S, heads=heads)
    names = ("dX", "dWqkv", "dWo", "dWlce")
    for name, g in zip(names, got):
        gn = to_numpy(g).astype(np.float64).reshape(ref[name].shape)
        rel = float(np.abs(gn - ref[name]).max() / np.abs(ref[name]).max())
        tol = 1e-4 if dtype == "f32" else (2e-2 if name == "dX" else (1e-3 if path == "generic" else 1e-2))
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


def random_matrix_core_shapes(count, seed):
    import random
    rng = random.Random(seed)
    out = []
    while len(out) < count:
        S = rng.choice([1, 2, 3, 4, 5, 7])
        H, W = S * rng.choice([1, 2, 3, 4, 5, 9, 12]), S * rng.choice([1, 2, 3, 4, 6, 11])
        heads, d = rng.choice([1, 2, 3, 4, 6, 8]), rng.choice([32, 32, 64])
        C = d * heads
        if C % 64:
            continue
        k = rng.choice([1, 2, 3, min(S * S, 5), S * S])
        n = (H // S) * (W // S)
        if k > S * S or H * W * C > 150000 or H * W * k * n * C > 6e7:
            continue
        out.append(("bf16", rng.choice([1, 2, 3]), H, W, C, heads, S, k))
    return out


@pytest.mark.parametrize("dtype,B,H,W,C,heads,S,k", random_matrix_core_shapes(24, seed=20230312))
def test_backward_matrix_cores_random_shapes(dtype, B, H, W, C, heads, S, k):
    test_backward(dtype, B, H, W, C, heads, S, k, path="mfma")


@pytest.mark.parametrize("idx", [1, 2, 3, 4, 5])
def test_backward_named_workloads_full_size(idx):
    # the five named workloads at their full sizes (random routing index, given to both sides)
    cfg = CONFIGS[idx]
    Xn, Wqkvn, Won, Wlcen = make_config_inputs(cfg)
    # the bf16 workloads run on the matrix-core kernels, the float32 one on the scalar ones
    compare_backward(Xn, Wqkvn, Won, Wlcen, cfg.dtype, cfg.heads, cfg.S, cfg.k,
                     path="mfma" if cfg.dtype == "bf16" else "generic")


@pytest.mark.parametrize("idx", [6, 7, 8])
def test_backward_wide_workloads_full_size(idx):
    # the next-step shapes with C = 512, 384 (heads of 32 channels) and 768 (heads of 64) at their full sizes
    from synthetic_inputs import NEXT_CONFIGS
    cfg = NEXT_CONFIGS[idx]
    Xn, Wqkvn, Won, Wlcen = make_config_inputs(cfg)
    compare_backward(Xn, Wqkvn, Won, Wlcen, cfg.dtype, cfg.heads, cfg.S, cfg.k, path="mfma")


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


def test_backward_matrix_cores_repeats_bit_identical():
    # no atomic adds on this path: dK, dV are summed per key region in registers, in the order of the
    # routing entries, and the weight gradients from partial sums in a fixed order
    for (B, H, W, C, heads, S, k) in [(2, 56, 56, 64, 2, 7, 1), (2, 28, 28, 128, 4, 7, 4)]:
        Xn, Wqkvn, Won, Wlcen = make_inputs(B, H, W, C, seed=6200 + C, dtype="bf16")
        r = np.random.Generator(np.random.PCG64(6201))
        dYn = round_to_bf16(r.standard_normal(Xn.shape).astype(np.float32))
        # a skewed routing: half of the query regions attend to region 0
        Irn = np.stack([np.stack([r.permutation(S * S)[:k] for _ in range(S * S)]) for _ in range(B)]).astype(np.int32)
        for b in range(B):
            for i in range(0, S * S, 2):
                Irn[b, i] = np.concatenate(([0], 1 + r.permutation(S * S - 1)[:k - 1]))
        X, Wqkv, Wo, Wlce, dY = (to_device(a, "bf16") for a in (Xn, Wqkvn, Won, Wlcen, dYn))
        Ir = torch.from_numpy(Irn).cuda()
        first = [g.clone() for g in bra.bra_backward(X, Wqkv, Wo, Wlce, Ir, dY, S, heads, path="mfma")]
        for _ in range(3):
            again = bra.bra_backward(X, Wqkv, Wo, Wlce, Ir, dY, S, heads, path="mfma")
            torch.cuda.synchronize()
            for a, b in zip(first, again):
                assert torch.equal(a, b)
        ref = obw.bra_backward(Xn, Wqkvn, Won, Wlcen, dYn, Irn, S=S, heads=heads)
        for name, g in zip(("dX", "dWqkv", "dWo", "dWlce"), first):
            gn = to_numpy(g).astype(np.float64).reshape(ref[name].shape)
            rel = float(np.abs(gn - ref[name]).max() / np.abs(ref[name]).max())
            assert rel <= (2e-2 if name == "dX" else 1e-2), f"{name}: {rel:.3e}"


def test_backward_matrix_cores_refuses_other_shapes():
    X = torch.zeros((1, 8, 8, 96), dtype=torch.bfloat16, device="cuda")
    Wqkv = torch.zeros((96, 288), dtype=torch.bfloat16, device="cuda")
    Wo = torch.zeros((96, 96), dtype=torch.bfloat16, device="cuda")
    Wlce = torch.zeros((96, 5, 5), dtype=torch.bfloat16, device="cuda")
    Ir = torch.zeros((1, 4, 1), dtype=torch.int32, device="cuda")
    with pytest.raises(bra.BraError):
        bra.bra_backward(X, Wqkv, Wo, Wlce, Ir, X, 2, 3, path="mfma")


def test_backward_matrix_cores_crowded_key_region():
    # every query region attends to region 0 (289 routing entries name it: beyond the 256 the key
    # side sorts, so its sum runs in arrival order), and some rows name a region twice
    B, H, W, C, heads, S, k = 1, 17, 34, 64, 2, 17, 2
    Xn, Wqkvn, Won, Wlcen = make_inputs(B, H, W, C, seed=6300, dtype="bf16")
    r = np.random.Generator(np.random.PCG64(6301))
    dYn = round_to_bf16(r.standard_normal(Xn.shape).astype(np.float32))
    Irn = np.zeros((B, S * S, k), dtype=np.int32)
    Irn[:, :, 1] = r.integers(0, S * S, size=(B, S * S))
    Irn[:, 5, 1] = 0
    X, Wqkv, Wo, Wlce, dY = (to_device(a, "bf16") for a in (Xn, Wqkvn, Won, Wlcen, dYn))
    got = bra.bra_backward(X, Wqkv, Wo, Wlce, torch.from_numpy(Irn).cuda(), dY, S, heads, path="mfma")
    torch.cuda.synchronize()
    ref = obw.bra_backward(Xn, Wqkvn, Won, Wlcen, dYn, Irn, S=S, heads=heads)
    for name, g in zip(("dX", "dWqkv", "dWo", "dWlce"), got):
        gn = to_numpy(g).astype(np.float64).reshape(ref[name].shape)
        rel = float(np.abs(gn - ref[name]).max() / np.abs(ref[name]).max())
        print(f"  {name}: max error {rel:.3e} of max|gradient|", flush=True)
        assert rel <= (2e-2 if name == "dX" else 1e-2), f"{name}: {rel:.3e}"
