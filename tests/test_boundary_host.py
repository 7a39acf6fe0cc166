"""Host-side checks of the C-ABI library: it loads, exports every symbol that
include/bra.h declares, and turns invalid arguments into error codes before any
GPU work (none of these calls reaches a kernel launch)."""
import ctypes
import os
import re

import pytest

import paper_2303_08810_amd as bra

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "bra.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(bra_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = bra.lib()
    names = declared_functions()
    assert set(names) == set(bra.EXPORTS)
    for name in names:
        assert getattr(L, name) is not None
    assert L.bra_version() >= 100


def ws_bytes(**kw):
    base = dict(B=1, H=28, W=28, C=64, heads=2, S=7, k=4, dtype=bra.BRA_F32, scale=None, path="auto")
    base.update(kw)
    shape = bra.make_shape(**base)
    out = ctypes.c_size_t(0)
    return bra.lib().bra_workspace_bytes(ctypes.byref(shape), ctypes.byref(out)), out.value


def test_workspace_query_and_error_codes():
    rc, n = ws_bytes()
    assert rc == 0 and n > 0 and n % 256 == 0
    assert ws_bytes(S=5)[0] == -2            # S does not divide H
    assert ws_bytes(heads=3)[0] == -2        # heads does not divide C
    assert ws_bytes(B=0)[0] == -2
    assert ws_bytes(k=0)[0] == -3
    assert ws_bytes(k=50)[0] == -3
    assert ws_bytes(k=49)[0] == 0
    assert ws_bytes(dtype=7)[0] == -4
    assert ws_bytes(path="mfma")[0] == -6    # matrix-core kernels are bf16 only
    assert bra.lib().bra_workspace_bytes(None, None) == -1
    for code in range(0, -9, -1):
        assert bra.strerror(code) != "unknown error code"
    assert bra.strerror(-99) == "unknown error code"


def test_kernel_family_selection_by_shape():
    """Which shapes the matrix-core family accepts (path "mfma" fails with -6 otherwise)."""
    def mfma(**kw):
        return ws_bytes(dtype=bra.BRA_BF16, path="mfma", **kw)[0]
    # the five named bf16 workloads' shapes
    assert mfma(B=64, H=56, W=56, C=64, heads=2, S=7, k=1) == 0
    assert mfma(B=64, H=28, W=28, C=128, heads=4, S=7, k=4) == 0
    assert mfma(B=64, H=14, W=14, C=256, heads=8, S=7, k=16) == 0
    assert mfma(B=2, H=128, W=128, C=64, heads=2, S=8, k=4) == 0
    # other channel counts: multiples of 64 with heads of 32 channels and small regions
    assert mfma(B=64, H=7, W=7, C=512, heads=16, S=7, k=49) == 0
    assert mfma(B=2, H=14, W=14, C=384, heads=12, S=7, k=16) == 0
    assert mfma(B=2, H=28, W=28, C=512, heads=16, S=7, k=4) == 0       # regions of 16 tokens at C = 512
    assert mfma(B=2, H=14, W=14, C=384, heads=6, S=7, k=4) == 0        # heads of 64 channels
    assert mfma(B=1, H=32, W=32, C=64, heads=2, S=16, k=4) == 0        # 256 regions: routed by the generic kernels
    assert mfma(B=2, H=21, W=14, C=64, heads=2, S=7, k=2) == 0         # regions of 6 tokens
    assert mfma(B=2, H=14, W=14, C=96, heads=3, S=7, k=4) == -6        # C not a multiple of 64
    assert mfma(B=2, H=14, W=14, C=128, heads=8, S=7, k=4) == -6       # heads of 16 channels
    # maps beyond the 32-bit element offsets / exact divisions of the matrix-core kernels
    assert mfma(B=1, H=8192, W=8192, C=64, heads=2, S=8, k=1) == -6    # 2^32 elements per image
    assert mfma(B=1, H=4096, W=4096, C=64, heads=2, S=2, k=1) == -6    # 2^22 tokens per region
    assert mfma(B=1, H=2048, W=2048, C=64, heads=2, S=8, k=64) == -6   # 2^22 keys per query
    # every rejected shape still runs on the generic family
    for kw in (dict(H=14, W=14, C=96, heads=3, S=7, k=4), dict(H=14, W=14, C=128, heads=8, S=7, k=4)):
        rc, n = ws_bytes(dtype=bra.BRA_BF16, path="auto", B=2, **kw)
        assert rc == 0 and n > 0


def test_entry_points_reject_bad_arguments_before_launching():
    L = bra.lib()
    shape = bra.make_shape(1, 28, 28, 64, 2, 7, 4, bra.BRA_F32)
    fake = ctypes.c_void_p(4096)             # never dereferenced: checks fail first
    assert L.bra_forward(ctypes.byref(shape), None, fake, fake, fake, fake, None, None, fake, 1 << 30, None) == -1
    assert L.bra_route(ctypes.byref(shape), fake, fake, None, None, fake, 1 << 30, None) == -1
    # workspace NULL / misaligned / too small
    assert L.bra_forward(ctypes.byref(shape), fake, fake, fake, fake, fake, None, None, None, 1 << 30, None) == -5
    assert L.bra_forward(ctypes.byref(shape), fake, fake, fake, fake, fake, None, None,
                         ctypes.c_void_p(4096 + 8), 1 << 30, None) == -5
    assert L.bra_forward(ctypes.byref(shape), fake, fake, fake, fake, fake, None, None, fake, 16, None) == -5
    assert L.bra_route(ctypes.byref(shape), fake, fake, fake, None, fake, 16, None) == -5
    bad = bra.make_shape(1, 28, 28, 64, 2, 7, 50, bra.BRA_F32)
    assert L.bra_forward(ctypes.byref(bad), fake, fake, fake, fake, fake, None, None, fake, 1 << 30, None) == -3
    assert L.bra_forward(None, fake, fake, fake, fake, fake, None, None, fake, 1 << 30, None) == -1


def test_static_scratch_entry_point_rejects_before_launching():
    L = bra.lib()
    fake = ctypes.c_void_p(4096)
    ok = bra.make_shape(1, 28, 28, 64, 2, 7, 4, bra.BRA_F32)
    assert L.bra_forward_static(ctypes.byref(ok), None, fake, fake, fake, fake, None, None, None) == -1
    assert L.bra_forward_static(None, fake, fake, fake, fake, fake, None, None, None) == -1
    bad = bra.make_shape(1, 28, 28, 64, 2, 7, 50, bra.BRA_F32)
    assert L.bra_forward_static(ctypes.byref(bad), fake, fake, fake, fake, fake, None, None, None) == -3
    # a batch whose workspace exceeds the built-in buffer: refused, nothing enqueued
    big = bra.make_shape(64, 28, 28, 128, 4, 7, 4, bra.BRA_BF16)
    assert ws_bytes(B=64, C=128, heads=4, dtype=bra.BRA_BF16)[1] > bra.STATIC_SCRATCH_BYTES
    assert L.bra_forward_static(ctypes.byref(big), fake, fake, fake, fake, fake, None, None, None) == -8
    assert "scratch" in bra.strerror(-8)


def test_block_and_padded_workspace_queries():
    L = bra.lib()
    out = ctypes.c_size_t(0)

    def block(hidden, **kw):
        base = dict(B=2, H=28, W=28, C=64, heads=2, S=7, k=4, dtype=bra.BRA_BF16, scale=None, path="auto")
        base.update(kw)
        shape = bra.make_shape(**base)
        return L.bra_block_workspace_bytes(ctypes.byref(shape), hidden, ctypes.byref(out)), out.value

    rc, n = block(192)
    inner = ws_bytes(B=2, dtype=bra.BRA_BF16)[1]
    tokens = 2 * 28 * 28
    # X1, LayerNorm1's output, BRA's output, the hidden layer, BRA's own workspace
    assert rc == 0 and n % 256 == 0 and n >= inner + tokens * (3 * 64 + 192) * 2
    assert block(0)[0] == -2 and block(-64)[0] == -2                  # hidden < 1
    # float32 tensors and sizes that are not multiples of 64 run on the scalar kernels
    assert block(100)[0] == 0 and block(192, dtype=bra.BRA_F32)[0] == 0 and block(144, C=48, heads=3)[0] == 0
    assert block(192, dtype=bra.BRA_F32)[1] >= 2 * 28 * 28 * (3 * 64 + 192) * 4
    assert block(192, H=30)[0] == -2 and block(192, k=50)[0] == -3    # BRA's own checks come first
    assert L.bra_block_workspace_bytes(None, 192, ctypes.byref(out)) == -1

    def padded(**kw):
        base = dict(B=1, H=30, W=45, C=64, heads=2, S=7, k=4, dtype=bra.BRA_BF16, scale=None, path="auto")
        base.update(kw)
        shape = bra.make_shape(**base)
        return L.bra_padded_workspace_bytes(ctypes.byref(shape), ctypes.byref(out)), out.value

    rc, n = padded()
    inner = ws_bytes(H=35, W=49, dtype=bra.BRA_BF16)[1]
    assert rc == 0 and n >= inner + 2 * 35 * 49 * 64 * 2                # padded X and Y beside BRA's workspace
    assert padded(H=35, W=49) == (0, inner)                           # S divides: no copies, bra_forward's size
    assert padded(H=0)[0] == -2 and padded(k=50)[0] == -3 and padded(S=0)[0] == -2
    # the padded call turns the same invalid arguments into codes before any launch
    shape = bra.make_shape(1, 30, 45, 64, 2, 7, 4, bra.BRA_BF16)
    assert L.bra_forward_padded(ctypes.byref(shape), None, None, None, None, None, None, None, None, 0, None) == -1
    fake = ctypes.c_void_p(256)
    assert L.bra_forward_padded(ctypes.byref(shape), fake, fake, fake, fake, fake, None, None, None, 0, None) == -5


def test_backward_workspace_query_and_error_codes():
    L = bra.lib()
    out = ctypes.c_size_t(0)
    shape = bra.make_shape(2, 28, 28, 64, 2, 7, 4, bra.BRA_F32)
    assert L.bra_backward_workspace_bytes(ctypes.byref(shape), ctypes.byref(out)) == 0
    # Q|K|V, O, dO and dQ|dK|dV in float32: 8 C floats per token
    assert out.value >= 2 * 28 * 28 * 8 * 64 * 4 and out.value % 256 == 0
    wide = bra.make_shape(1, 8, 8, 256, 2, 2, 2, bra.BRA_F32)          # heads of 128 channels
    assert L.bra_backward_workspace_bytes(ctypes.byref(wide), ctypes.byref(out)) == -6
    bad = bra.make_shape(1, 28, 28, 64, 2, 7, 50, bra.BRA_F32)
    assert L.bra_backward_workspace_bytes(ctypes.byref(bad), ctypes.byref(out)) == -3
    fake = ctypes.c_void_p(4096)
    args = [fake] * 11
    assert L.bra_backward(ctypes.byref(shape), *args, 16, None) == -5          # workspace too small
    args[4] = None                                                              # Ir missing
    assert L.bra_backward(ctypes.byref(shape), *args, 1 << 30, None) == -1


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(bra, "_lib", None)
    monkeypatch.setattr(bra, "LIB_PATH", str(tmp_path / "libbra.so"))
    with pytest.raises(ImportError):
        bra.lib()
