"""GPU test of bra_forward_static (the entry point that allocates nothing: its scratch memory is a
buffer inside the library's code object): same bits as bra_forward, on two calls in a row that
share the buffer, the second with a smaller input; then the other kernel families."""
import numpy as np
import pytest
import torch

import paper_2303_08810_amd as bra
from parity_util import to_device
from synthetic_inputs import CONFIGS, make_config_inputs, make_inputs

pytestmark = pytest.mark.gpu


def both(Xn, Wqkvn, Won, Wlcen, dtype, S, k, heads, Ir_in=None):
    X, Wqkv, Wo, Wlce = (to_device(a, dtype) for a in (Xn, Wqkvn, Won, Wlcen))
    B = X.shape[0]
    Y0, I0 = bra.bra_forward(X, Wqkv, Wo, Wlce, S, k, heads, want_Ir=True, Ir_in=Ir_in)
    Y1 = torch.full_like(X, 7.0)
    I1 = torch.full((B, S * S, k), -1, dtype=torch.int32, device=X.device)
    bra.bra_forward_static(X, Wqkv, Wo, Wlce, S, k, heads, out=Y1, Ir_out=I1, Ir_in=Ir_in)
    torch.cuda.synchronize()
    as_bits = lambda t: t.view(torch.int16 if t.dtype == torch.bfloat16 else torch.int32).cpu().numpy()
    np.testing.assert_array_equal(as_bits(Y1), as_bits(Y0))
    np.testing.assert_array_equal(I1.cpu().numpy(), I0.cpu().numpy())


def test_static_scratch_two_calls_second_smaller():
    cfg = CONFIGS[3]                      # projection -> routing -> attention: Q, K, V, partial sums in scratch
    Xn, Wqkvn, Won, Wlcen = make_config_inputs(cfg, batch=8)
    print("static scratch: workload 3 shape, 8 images", flush=True)
    both(Xn, Wqkvn, Won, Wlcen, cfg.dtype, cfg.S, cfg.k, cfg.heads)
    print("static scratch: workload 3 shape, 3 images (smaller, same buffer)", flush=True)
    both(Xn[:3].copy(), Wqkvn, Won, Wlcen, cfg.dtype, cfg.S, cfg.k, cfg.heads)


@pytest.mark.parametrize("idx,batch", [(1, 1), (2, 6), (4, 8), (5, 2)])
def test_static_scratch_other_pipelines(idx, batch):
    cfg = CONFIGS[idx]
    Xn, Wqkvn, Won, Wlcen = make_config_inputs(cfg, batch=batch)
    print(f"static scratch: workload {idx} shape, {batch} images", flush=True)
    both(Xn, Wqkvn, Won, Wlcen, cfg.dtype, cfg.S, cfg.k, cfg.heads)


def test_static_scratch_forced_routing_and_limit():
    Xn, Wqkvn, Won, Wlcen = make_inputs(2, 28, 28, 64, seed=99, dtype="bf16")
    Ir_in = torch.from_numpy(np.broadcast_to(np.arange(4, dtype=np.int32)[None, None, :], (2, 49, 4)).copy()).cuda()
    both(Xn, Wqkvn, Won, Wlcen, "bf16", 7, 4, 2, Ir_in=Ir_in)
    cfg = CONFIGS[3]
    X = torch.zeros((64, cfg.H, cfg.W, cfg.C), dtype=torch.bfloat16, device="cuda")
    W = [to_device(a, "bf16") for a in make_config_inputs(cfg, batch=1)[1:]]
    with pytest.raises(bra.BraError) as e:
        bra.bra_forward_static(X, *W, cfg.S, cfg.k, cfg.heads, out=torch.empty_like(X))
    assert e.value.code == -8
