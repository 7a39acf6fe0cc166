"""GPU parity of the whole-block entry point (bra_block_forward, through the C ABI) against
the float64 block oracle on the same seeded inputs.

Bars: the routing index obeys parity_util.check_routing against the affinities of an oracle run
whose BRA input is LayerNorm1's output rounded to bf16 (the decision of Eq. 5 is taken on the
stored tensor; that run serves the routing comparison only); with the GPU's routing given to the
plain float64 oracle (no rounding anywhere), the block's update Xout - X is within 2e-2 of
max|Xout_ref - X| (the bf16 bar, taken on the update so that the residual copy of X cannot hide
an error in a branch), and its rms error within 8e-3 of the update's rms.
"""
import numpy as np
import pytest
import torch

import paper_2303_08810_amd as bra
from oracle import block as ob
from parity_util import TOL_BF16_REL, TOL_F32_ABS, check_routing, to_device, to_numpy
from synthetic_inputs import (BASE_SEED, CONFIGS, NEXT_CONFIGS, make_block_inputs, make_block_params,
                              make_inputs)

pytestmark = pytest.mark.gpu

EPS = 1e-6


def device_params(P, dtype="bf16"):
    out = {}
    for name in bra.BraBlockParams.FIELDS:
        if name in bra.BraBlockParams.MATRICES:
            out[name] = to_device(P[name], dtype)
        else:
            out[name] = torch.from_numpy(np.ascontiguousarray(P[name], dtype=np.float32)).cuda()
    return out


def compare_block(Xn, P, S, k, heads, path="auto", images=None, in_place=False, forced=None, dtype="bf16"):
    print(f"block case dtype={dtype} shape={Xn.shape} hidden={P['W1'].shape[1]} S={S} k={k} heads={heads} "
          f"path={path} in_place={in_place} forced={forced is not None}", flush=True)
    X = to_device(Xn, dtype)
    dP = device_params(P, dtype)
    Iin = torch.from_numpy(np.ascontiguousarray(forced, dtype=np.int32)).cuda() if forced is not None else None
    Xout, Ir = bra.bra_block_forward(X, dP, S, k, heads, eps=EPS, want_Ir=True, path=path, Ir_in=Iin,
                                     out=X if in_place else None)
    torch.cuda.synchronize()
    got, Ir = to_numpy(Xout), Ir.cpu().numpy()
    sel = np.arange(Xn.shape[0]) if images is None else np.asarray(images)
    kw = dict(S=S, k=k, heads=heads, eps=EPS, threads=8)
    if forced is None:
        free = ob.block_forward(Xn[sel], P, store="bf16" if dtype == "bf16" else "f64", **kw)
        check_routing(Ir[sel], free["Ar"], k)
    else:
        np.testing.assert_array_equal(Ir, forced)
    ref = ob.block_forward(Xn[sel], P, Ir_in=Ir[sel], store="f64", **kw)
    if dtype == "f32":
        # float32 tensors: the bar of the float32 BRA path, max-abs 1e-4, on the block's output
        err = float(np.abs(got[sel].astype(np.float64) - ref["Xout"]).max())
        print(f"  max-abs error {err:.3e}", flush=True)
        assert err <= TOL_F32_ABS, f"max-abs error {err:.3e} > {TOL_F32_ABS}"
        return err
    upd_ref = ref["Xout"] - Xn[sel]
    upd = got[sel].astype(np.float64) - Xn[sel]
    rel = float(np.abs(upd - upd_ref).max() / np.abs(upd_ref).max())
    rms = float(np.sqrt(np.mean((upd - upd_ref) ** 2)) / np.sqrt(np.mean(upd_ref ** 2)))
    print(f"  update error: max {rel:.3e} of max|update|, rms {rms:.3e} of rms(update)", flush=True)
    assert rel <= TOL_BF16_REL, f"max|d(Xout - X)| / max|Xout_ref - X| = {rel:.3e} > {TOL_BF16_REL}"
    # the bf16 roundings of the stored tensors and of the result are independent errors of relative
    # size 2^-9 (measured: rms 4e-3 of the update's rms at every shape); an error in a branch (a
    # wrong tap, a missing bias) would show in the mean long before it shows in the maximum
    assert rms <= 8e-3, f"rms error {rms:.3e} of the update's rms"
    return rel


def inputs(B, H, W, C, seed, expansion=3, dtype="bf16", hidden=None):
    X, Wqkv, Wo, Wlce = make_inputs(B, H, W, C, seed=seed, dtype=dtype)
    P = make_block_params(C, hidden or expansion * C, seed=seed + 1, dtype=dtype)
    P.update(Wqkv=Wqkv, Wo=Wo, Wlce=Wlce)
    return X, P


# (B, H, W, C, heads, S, k, expansion): one chunk per lane (C <= 512) and several (C = 192, 384,
# 768, 1024), heads of 32 and 64 channels, token counts that leave a ragged last workgroup,
# H != W, every BRA pipeline (fused k = 1, 256- and 64-token regions, small regions, general)
BLOCK_SHAPES = [
    (2, 28, 28, 64, 2, 7, 4, 3),
    (3, 56, 56, 64, 2, 7, 1, 3),
    (1, 14, 14, 256, 8, 7, 16, 3),
    (2, 28, 28, 128, 4, 7, 4, 4),
    (1, 64, 32, 64, 2, 4, 2, 3),
    (3, 7, 7, 512, 16, 7, 49, 3),
    (1, 14, 14, 384, 12, 7, 16, 3),
    (1, 12, 20, 192, 6, 4, 3, 3),
    (1, 16, 16, 768, 12, 8, 12, 3),
    (1, 8, 8, 1024, 16, 4, 5, 1),
    (5, 6, 10, 64, 2, 2, 3, 3),
    (2, 14, 14, 64, 2, 7, 4, 1),
    (1, 21, 14, 64, 2, 7, 2, 2),
    (3, 14, 28, 64, 2, 7, 4, 4),
    (1, 28, 28, 64, 2, 7, 4, 5),
]


@pytest.mark.parametrize("B,H,W,C,heads,S,k,e", BLOCK_SHAPES)
def test_block_shapes(B, H, W, C, heads, S, k, e):
    X, P = inputs(B, H, W, C, seed=4000 + C + H + k, expansion=e)
    compare_block(X, P, S, k, heads)


def random_block_shapes(count, seed):
    """Seeded random shapes within what the block is built for (C a multiple of 64, heads of 32 or
    64 channels), sized for the oracle."""
    import random
    rng = random.Random(seed)
    out = []
    while len(out) < count:
        S = rng.choice([1, 2, 3, 4, 5, 7, 8])
        H, W = S * rng.choice([1, 2, 3, 4, 5, 8, 13]), S * rng.choice([1, 2, 3, 4, 6, 8, 11])
        heads = rng.choice([1, 2, 3, 4, 6, 8, 10, 12, 16])
        C = rng.choice([32, 32, 64]) * heads
        k = rng.choice([1, 2, 3, 4, min(S * S, 12), S * S])
        B, e = rng.choice([1, 2, 3]), rng.choice([1, 2, 3, 3, 4, 5])
        n = (H // S) * (W // S)
        if C % 64 or C > 1024 or k > S * S or H * W * C > 400000 or H * W * k * n * C > 2e8 or B * H * W * C * e * C > 3e9:
            continue
        out.append((B, H, W, C, heads, S, k, e))
    return out


@pytest.mark.parametrize("B,H,W,C,heads,S,k,e", random_block_shapes(16, seed=20230309))
def test_block_random_shapes(B, H, W, C, heads, S, k, e):
    X, P = inputs(B, H, W, C, seed=4500 + H * W + C + e, expansion=e)
    compare_block(X, P, S, k, heads)


# (dtype, B, H, W, C, heads, S, k, hidden): the scalar kernels take float32 tensors and the bf16
# shapes the matrix-core kernels are not built for (C or hidden not a multiple of 64)
SCALAR_BLOCK_SHAPES = [
    ("f32", 1, 28, 28, 64, 2, 7, 4, 192),
    ("f32", 2, 12, 20, 48, 3, 4, 3, 100),
    ("f32", 1, 7, 7, 130, 2, 7, 49, 260),
    ("f32", 3, 6, 9, 32, 1, 3, 2, 32),
    ("bf16", 2, 12, 12, 48, 3, 3, 2, 144),
    ("bf16", 1, 14, 14, 64, 2, 7, 4, 100),
]


@pytest.mark.parametrize("dtype,B,H,W,C,heads,S,k,hidden", SCALAR_BLOCK_SHAPES)
def test_block_scalar_kernels(dtype, B, H, W, C, heads, S, k, hidden):
    X, P = inputs(B, H, W, C, seed=4600 + C + hidden, dtype=dtype, hidden=hidden)
    compare_block(X, P, S, k, heads, dtype=dtype)


def test_block_float32_in_place_and_forced_routing():
    X, P = inputs(2, 14, 14, 64, seed=4700, dtype="f32")
    compare_block(X, P, 7, 4, 2, dtype="f32", in_place=True)
    r = np.random.Generator(np.random.PCG64(4701))
    forced = np.stack([np.stack([r.permutation(49)[:4] for _ in range(49)]) for _ in range(2)]).astype(np.int32)
    compare_block(X, P, 7, 4, 2, dtype="f32", forced=forced)


def test_block_generic_family_for_bra():
    X, P = inputs(2, 14, 14, 64, seed=4100)
    compare_block(X, P, 7, 4, 2, path="generic")


def test_block_in_place_and_forced_routing():
    X, P = inputs(2, 28, 28, 64, seed=4200)
    compare_block(X, P, 7, 4, 2, in_place=True)
    r = np.random.Generator(np.random.PCG64(4201))
    forced = np.stack([np.stack([r.permutation(49)[:4] for _ in range(49)]) for _ in range(2)]).astype(np.int32)
    compare_block(X, P, 7, 4, 2, forced=forced)


def test_block_repeated_runs_are_bit_identical():
    X, P = inputs(2, 28, 28, 128, seed=4300)
    Xd, dP = to_device(X, "bf16"), device_params(P)
    outs = []
    for _ in range(4):
        o = bra.bra_block_forward(Xd, dP, 7, 4, 4, eps=EPS)
        torch.cuda.synchronize()
        outs.append(o.view(torch.int16).cpu().numpy().copy())
    for o in outs[1:]:
        np.testing.assert_array_equal(o, outs[0])


@pytest.mark.parametrize("idx,images", [(2, [0, 31, 63]), (3, [0, 63]), (4, [5, 63]), (5, [1]),
                                        (6, [0, 1, 62, 63]), (8, [7])])
def test_block_named_workloads_full_size(idx, images):
    cfg = CONFIGS.get(idx) or NEXT_CONFIGS[idx]
    X, P = make_block_inputs(cfg)
    compare_block(X, P, cfg.S, cfg.k, cfg.heads, images=images)


def test_block_rejects_invalid_arguments():
    X, P = inputs(1, 14, 14, 64, seed=4400)
    Xd, dP = to_device(X, "bf16"), device_params(P)
    with pytest.raises(bra.BraError) as e:
        bra.bra_block_forward(Xd, dP, 7, 4, 2, eps=-1.0)
    assert e.value.code == -2
    with pytest.raises(bra.BraError) as e:
        bra.bra_block_forward(Xd, dP, 7, 50, 2)
    assert e.value.code == -3
    with pytest.raises(ValueError):
        bra.bra_block_forward(Xd, {**dP, "W1": dP["W1"].float()}, 7, 4, 2)
