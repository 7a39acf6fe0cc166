"""Host-side checks of the harness files: the seeded generators are deterministic and round as
documented, and bench.py refuses more than one GPU before it touches a device."""
import os
import subprocess
import sys

import numpy as np

from synthetic_inputs import (CONFIGS, NEXT_CONFIGS, bf16_bits, bits_to_f32, make_block_params, make_inputs,
                              round_to_bf16)

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_generators_are_deterministic_and_bf16_exact():
    a = make_inputs(2, 6, 8, 16, seed=77, dtype="bf16")
    b = make_inputs(2, 6, 8, 16, seed=77, dtype="bf16")
    for x, y in zip(a, b):
        np.testing.assert_array_equal(x, y)
        np.testing.assert_array_equal(bits_to_f32(bf16_bits(x)), x)          # representable: the round trip is exact
    c = make_inputs(2, 6, 8, 16, seed=78, dtype="bf16")
    assert not np.array_equal(a[0], c[0])
    P = make_block_params(16, 48, seed=5, dtype="bf16")
    Q = make_block_params(16, 48, seed=5, dtype="bf16")
    assert set(P) == {"Wpos", "bpos", "ln1_g", "ln1_b", "ln2_g", "ln2_b", "W1", "b1", "W2", "b2"}
    for key in P:
        np.testing.assert_array_equal(P[key], Q[key])
        assert P[key].dtype == np.float32
    for key in ("Wpos", "W1", "W2"):                                          # matrices rounded, vectors not
        np.testing.assert_array_equal(round_to_bf16(P[key]), P[key])
    assert P["W1"].shape == (16, 48) and P["W2"].shape == (48, 16) and P["Wpos"].shape == (16, 3, 3)


def test_round_to_bf16_is_round_to_nearest_even():
    one = np.float32(1.0)
    ulp = np.float32(2.0 ** -7)                      # bf16 spacing in [1, 2)
    x = np.array([one + ulp / 2, one + 3 * ulp / 2, one + ulp / 4, one + 3 * ulp / 4], dtype=np.float32)
    np.testing.assert_array_equal(round_to_bf16(x), np.array([one, one + 2 * ulp, one, one + ulp], dtype=np.float32))


def test_named_workloads_are_valid_shapes():
    for cfg in list(CONFIGS.values()) + list(NEXT_CONFIGS.values()):
        assert cfg.H % cfg.S == 0 and cfg.W % cfg.S == 0 and cfg.C % cfg.heads == 0 and 1 <= cfg.k <= cfg.R
        assert cfg.dtype in ("f32", "bf16")
