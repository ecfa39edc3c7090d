"""Pins of oracle/cache.py.  No GPU."""
import numpy as np
import torch

from oracle import cache as C


def test_bf16_rounding_hand_values():
    """bf16 keeps 8 significand bits: spacing 2^-7 in [1, 2).  Ties go to the even neighbour."""
    x = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20, 1.0 + 2.0 ** -7,
                  -(1.0 + 3 * 2.0 ** -8), 0.0, 3.0e38, 1e-40], dtype=np.float32)
    want = np.array([1.0, 1.0, 1.0 + 2 * 2.0 ** -7, 1.0 + 2.0 ** -7, 1.0 + 2.0 ** -7, -(1.0 + 2 * 2.0 ** -7), 0.0,
                     2.9908e38, 0.0], dtype=np.float32)
    got = C.to_bf16_nearest_even(x)
    assert np.array_equal(got[:7], want[:7])
    assert abs(got[7] - 3.0e38) <= 3.0e38 * 2.0 ** -8 and abs(got[8] - 1e-40) <= 2.0 ** -134


def test_bf16_rounding_matches_an_independent_library():
    rng = np.random.default_rng(3)
    x = np.concatenate([rng.standard_normal(100000).astype(np.float32) * 10.0 ** rng.integers(-20, 20, 100000),
                        np.array([np.inf, -np.inf, 65504.0, 1.0039062, 1.0117188], dtype=np.float32)])
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(C.to_bf16_nearest_even(x), want)


def test_append_and_emit_touch_only_their_rows():
    rng = np.random.default_rng(4)
    kc = np.full((2, 10, 8), -1.0, dtype=np.float32); vc = kc.copy()
    ks = rng.standard_normal((2, 3, 8)).astype(np.float32); vs = rng.standard_normal((2, 3, 8)).astype(np.float32)
    C.kv_append(ks, vs, 4, kc, vc)
    assert np.array_equal(kc[:, 4:7], ks) and np.array_equal(vc[:, 4:7], vs)
    assert (kc[:, :4] == -1).all() and (kc[:, 7:] == -1).all() and (vc[:, :4] == -1).all() and (vc[:, 7:] == -1).all()
    dk, dv = C.kv_grad_emit(kc, vc, 4, 3, "f32")
    assert np.array_equal(dk, ks) and np.array_equal(dv, vs)
    dk, dv = C.kv_grad_emit(kc, vc, 4, 3, "bf16")
    assert np.array_equal(dk, C.to_bf16_nearest_even(ks)) and np.abs(dk - ks).max() <= np.abs(ks).max() * 2.0 ** -8
