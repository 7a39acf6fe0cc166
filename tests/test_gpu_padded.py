"""GPU parity of bra_forward_padded (maps whose sides S does not divide) against the oracle's
padded variant, same bars as the other parity tests."""
import numpy as np
import pytest
import torch

import oracle
import paper_2303_08810_amd as bra
from parity_util import check_output, check_routing, to_device, to_numpy
from synthetic_inputs import make_inputs

pytestmark = pytest.mark.gpu

# (dtype, B, H, W, C, heads, S, k, path): one and both sides padded, padding that empties whole
# regions (H = 5 with S = 4 pads to 8: the last region row holds zero tokens only), the fused
# k = 1 pipeline, the general matrix-core pipeline, S = 16 on a detection-like size
PADDED = [
    ("f32", 2, 30, 45, 32, 1, 7, 4, "generic"),
    ("f32", 1, 5, 9, 16, 2, 4, 3, "generic"),
    ("bf16", 2, 30, 45, 64, 2, 7, 4, "auto"),
    ("bf16", 2, 50, 56, 64, 2, 7, 1, "auto"),
    ("bf16", 1, 100, 90, 64, 2, 8, 4, "auto"),
    ("bf16", 1, 13, 14, 256, 8, 7, 16, "auto"),
    ("bf16", 1, 200, 300, 64, 2, 16, 4, "auto"),
    ("bf16", 3, 28, 28, 128, 4, 7, 4, "auto"),      # S divides: the plain path, no copies
]


@pytest.mark.parametrize("dtype,B,H,W,C,heads,S,k,path", PADDED)
def test_padded_forward(dtype, B, H, W, C, heads, S, k, path):
    print(f"padded case dtype={dtype} shape={(B, H, W, C)} S={S} k={k} heads={heads} path={path}", flush=True)
    Xn, Wqkvn, Won, Wlcen = make_inputs(B, H, W, C, seed=5000 + H + W + k, dtype=dtype)
    X, Wqkv, Wo, Wlce = (to_device(a, dtype) for a in (Xn, Wqkvn, Won, Wlcen))
    Y, Ir = bra.bra_forward_padded(X, Wqkv, Wo, Wlce, S, k, heads, want_Ir=True, path=path)
    torch.cuda.synchronize()
    Y, Ir = to_numpy(Y), Ir.cpu().numpy()
    assert Y.shape == Xn.shape
    kw = dict(S=S, k=k, heads=heads, threads=8)
    free = oracle.bra_forward_padded(Xn, Wqkvn, Won, Wlcen, **kw)
    check_routing(Ir, free["Ar"], k)
    ref = oracle.bra_forward_padded(Xn, Wqkvn, Won, Wlcen, Ir_in=Ir, **kw)
    check_output(Y, ref["Y"], dtype)


def random_padded_shapes(count, seed):
    import random
    rng = random.Random(seed)
    out = []
    while len(out) < count:
        S = rng.choice([2, 3, 4, 5, 7, 8, 16])
        H, W = rng.randint(max(1, S // 2), 70), rng.randint(max(1, S // 2), 70)
        dtype = rng.choice(["bf16", "bf16", "f32"])
        heads = rng.choice([1, 2, 4, 8])
        C = rng.choice([16, 32, 32, 64]) * heads
        k = rng.choice([1, 2, 3, 4, min(S * S, 9)])
        Hp, Wp = -(-H // S) * S, -(-W // S) * S
        n = (Hp // S) * (Wp // S)
        if C > 512 or Hp * Wp * C > 500000 or Hp * Wp * k * n * C > 2e8:
            continue
        out.append((dtype, rng.choice([1, 2]), H, W, C, heads, S, k, "auto"))
    return out


@pytest.mark.parametrize("dtype,B,H,W,C,heads,S,k,path", random_padded_shapes(16, seed=20230310))
def test_padded_forward_random_shapes(dtype, B, H, W, C, heads, S, k, path):
    test_padded_forward(dtype, B, H, W, C, heads, S, k, path)


def test_padded_forward_forced_routing():
    B, H, W, C, heads, S, k = 2, 20, 26, 64, 2, 4, 3
    Xn, Wqkvn, Won, Wlcen = make_inputs(B, H, W, C, seed=5100, dtype="bf16")
    r = np.random.Generator(np.random.PCG64(5101))
    forced = np.stack([np.stack([r.permutation(S * S)[:k] for _ in range(S * S)]) for _ in range(B)]).astype(np.int32)
    X, Wqkv, Wo, Wlce = (to_device(a, "bf16") for a in (Xn, Wqkvn, Won, Wlcen))
    Y, Ir = bra.bra_forward_padded(X, Wqkv, Wo, Wlce, S, k, heads, want_Ir=True,
                                   Ir_in=torch.from_numpy(forced).cuda())
    torch.cuda.synchronize()
    np.testing.assert_array_equal(Ir.cpu().numpy(), forced)
    ref = oracle.bra_forward_padded(Xn, Wqkvn, Won, Wlcen, S=S, k=k, heads=heads, Ir_in=forced, threads=8)
    check_output(to_numpy(Y), ref["Y"], "bf16")
