"""Oracle for the two data movements around a segment's attention calls (test infrastructure, not the product):
appending a segment's K/V rows to the prefix cache, and emitting the final rows of the fp32 dK/dV accumulators
in the tensors' element type (Section 3.2).  Plain numpy slicing; bf16 conversion written out on the bits."""
from __future__ import annotations

import numpy as np


def to_bf16_nearest_even(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 (returned as fp32 holding the rounded value): keep the upper 16 bits, round to nearest,
    ties to the even upper half."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    upper, lower = u >> 16, u & 0xFFFF
    up = (lower > 0x8000) | ((lower == 0x8000) & ((upper & 1) == 1))
    r = ((upper + up.astype(np.uint64)) << 16).astype(np.uint32)
    return r.view(np.float32).reshape(np.shape(x))


def kv_append(k_seg: np.ndarray, v_seg: np.ndarray, seg_off: int, k_cache: np.ndarray, v_cache: np.ndarray) -> None:
    """k_seg, v_seg [H, seg_len, D] -> rows [seg_off, seg_off + seg_len) of k_cache, v_cache [H, capacity, D]."""
    n = k_seg.shape[1]
    k_cache[:, seg_off:seg_off + n] = k_seg
    v_cache[:, seg_off:seg_off + n] = v_seg


def kv_grad_emit(dk_acc: np.ndarray, dv_acc: np.ndarray, seg_off: int, seg_len: int, dtype: str):
    """Rows [seg_off, seg_off + seg_len) of the fp32 accumulators [H, capacity, D] in `dtype` ("f32" | "bf16")."""
    dk = np.asarray(dk_acc[:, seg_off:seg_off + seg_len], dtype=np.float32)
    dv = np.asarray(dv_acc[:, seg_off:seg_off + seg_len], dtype=np.float32)
    if dtype == "bf16":
        return to_bf16_nearest_even(dk), to_bf16_nearest_even(dv)
    return dk.copy(), dv.copy()
