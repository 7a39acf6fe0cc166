"""Helpers shared by the GPU parity tests (comparison rules only, no BRA arithmetic)."""
import numpy as np
import torch

import oracle
from synthetic_inputs import bf16_bits, bits_to_f32

GAP = 1e-3          # affinity gap above which routing indices must match bit for bit
TOL_F32_ABS = 1e-4  # max-abs bound on Y for float32 tensors
TOL_BF16_REL = 2e-2 # bound on max|dY| / max|Y_ref| for bf16 tensors
TOL_BF16_RMS = 8e-3 # bound on rms(dY) / rms(Y_ref) for bf16 tensors
TOL_BF16_FRAC = 0.999   # share of elements with |dY| <= 2e-2 |Y_ref| + 2e-2 rms(Y_ref), at least


def to_device(a, dtype):
    """float32 numpy array -> device tensor of the workload's storage type (exact)."""
    if dtype == "bf16":
        return torch.from_numpy(bf16_bits(a).view(np.int16)).view(torch.bfloat16).cuda()
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def to_numpy(t):
    if t.dtype == torch.bfloat16:
        return bits_to_f32(t.cpu().view(torch.int16).numpy().view(np.uint16))
    return t.cpu().numpy()


def check_routing(Ir_gpu, Ar_ref, k, gap=GAP):
    """Routing rule: per row with oracle affinities sorted s_1 >= ... >= s_R,
    (i) indices are in range and distinct; (ii) if s_k - s_{k+1} > gap the index SET
    equals the oracle's; (iii) position p matches exactly when both neighbouring
    gaps exceed `gap`; (iv) otherwise every pick has affinity >= s_k - gap.
    Returns the number of rows that differ from the oracle's exact order."""
    Ir_gpu = np.asarray(Ir_gpu)
    B, R, _ = Ar_ref.shape
    assert Ir_gpu.shape == (B, R, k)
    assert Ir_gpu.min() >= 0 and Ir_gpu.max() < R
    order = np.argsort(-Ar_ref, axis=-1, kind="stable")
    s = np.take_along_axis(Ar_ref, order, axis=-1)               # descending
    srt = np.sort(Ir_gpu, axis=-1)
    assert np.all(srt[..., 1:] != srt[..., :-1]), "duplicate region in a routing row"
    ref = order[..., :k]
    picked = np.take_along_axis(Ar_ref, Ir_gpu.astype(np.int64), axis=-1)
    assert np.all(picked >= s[..., k - 1:k] - gap), "picked a region below the k-th affinity"
    if k < R:
        clear = (s[..., k - 1] - s[..., k]) > gap
    else:
        clear = np.ones((B, R), dtype=bool)
    same_set = np.all(np.sort(ref, axis=-1) == srt, axis=-1)
    assert np.all(same_set[clear]), "index set differs where the boundary gap is clear"
    # positions whose neighbours are both further than gap away must match exactly
    d = s[..., :-1] - s[..., 1:] if R > 1 else np.zeros((B, R, 0))
    big = np.full((B, R, 1), np.inf)
    up = np.concatenate([big, d], axis=-1)[..., :k]               # gap to the previous value
    dn = np.concatenate([d, big], axis=-1)[..., :k]               # gap to the next value
    must = (up > gap) & (dn > gap)
    assert np.all((Ir_gpu == ref)[must]), "position differs where both neighbouring gaps are clear"
    return int(np.any(Ir_gpu != ref, axis=-1).sum())


def run_oracle(X, Wqkv, Wo, Wlce, cfgkw, Ir_in=None, threads=8, precision="f64", want=()):
    return oracle.bra_forward(X, Wqkv, Wo, Wlce, Ir_in=Ir_in, threads=threads, precision=precision,
                              want=want, **cfgkw)


def check_output(Y_gpu, Y_ref, dtype):
    """float32 tensors: max-abs bound.  bf16 tensors: three bounds.  The maximum norm is the stated
    bar; the rms bound and the element-wise share catch what it lets through (a localised defect
    of up to 2 % of max|Y|: one wrong tap at an image border, one mis-weighted key).  The bf16
    roundings of the stored intermediates and of Y are independent errors of relative size 2^-9,
    which puts the rms error at 3-4e-3 of rms(Y); 8e-3 leaves a factor of two."""
    d = Y_gpu.astype(np.float64) - Y_ref
    err = float(np.abs(d).max())
    if dtype == "f32":
        assert err <= TOL_F32_ABS, f"max-abs error {err:.3e} > {TOL_F32_ABS}"
        return err
    rel = err / float(np.abs(Y_ref).max())
    assert rel <= TOL_BF16_REL, f"max|dY|/max|Y| = {rel:.3e} > {TOL_BF16_REL}"
    ref_rms = float(np.sqrt(np.mean(Y_ref ** 2)))
    if ref_rms > 0:
        rms = float(np.sqrt(np.mean(d ** 2))) / ref_rms
        frac = float(np.mean(np.abs(d) <= 2e-2 * np.abs(Y_ref) + 2e-2 * ref_rms))
        print(f"  rms(dY)/rms(Y) = {rms:.3e}; share within 2e-2|Y| + 2e-2 rms(Y): {frac:.6f}", flush=True)
        assert rms <= TOL_BF16_RMS, f"rms(dY)/rms(Y) = {rms:.3e} > {TOL_BF16_RMS}"
        assert frac >= TOL_BF16_FRAC, f"only {frac:.6f} of the elements within 2e-2|Y| + 2e-2 rms(Y)"
    return err
