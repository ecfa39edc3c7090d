"""CPU-only checks of the boundary: the shared library loads, exports every symbol the header declares,
validates arguments before touching a device, and its partitioner agrees bit for bit with the oracle."""
import ctypes
import os
import re

import pytest

import paper_2406_03488_amd as s1f
from paper_2406_03488_amd import binding
from oracle import partition as P

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "s1f.h")).read()
    names = set(re.findall(r"\b(s1f_[a-z_0-9]+)\s*\(", header))
    assert {"s1f_partition", "s1f_seg_attn_fwd", "s1f_seg_attn_bwd", "s1f_bwd_workspace_bytes", "s1f_strerror",
            "s1f_version"} <= names
    lib = s1f.load_library()
    for name in names:
        assert hasattr(lib, name), name
    assert s1f.version() >= 100


@pytest.mark.parametrize("args", [(8, 2, 1, 1), (6, 3, 1, 1), (100, 4, 8, 2), (1000, 7, 64, 8), (4096, 8, 512, 8),
                                  (999, 3, 1, 1), (37, 1, 16, 4), (9, 9, 16, 4), (8192, 4, 2560, 32),
                                  (32768, 8, 4096, 32), (65536, 16, 7168, 56), (131072, 32, 8192, 64),
                                  (64, 4, 10**6, 1), (10000, 5, 1, 1), (24, 23, 3, 1), (50, 49, 1, 1)])
def test_partition_matches_oracle_bit_exact(args):
    assert s1f.partition(*args) == P.partition(*args)


def test_partition_matches_oracle_sweep():
    for n in range(1, 40):
        for k in range(1, min(n, 6) + 1):
            for hidden in (1, 2, 5, 64):
                assert s1f.partition(n, k, hidden, 1) == P.partition(n, k, hidden, 1), (n, k, hidden)


def test_partition_rejects_bad_arguments():
    for bad in ((8, 0, 4, 1), (3, 4, 4, 1), (8, 2, 0, 1), (8, 2, 4, 0), (8, 2, 6, 4)):
        with pytest.raises(s1f.S1FError) as e:
            s1f.partition(*bad)
        assert e.value.status == 1
    lib = s1f.load_library()
    assert lib.s1f_partition(8, 2, 4, 1, None) == 1


def _desc(**kw):
    base = dict(batch=1, n_q_heads=4, n_kv_heads=2, head_dim=64, dtype=1, reserved=0, q_stride_b=4 * 256 * 64,
                q_stride_h=256 * 64, q_stride_s=64, kv_stride_b=2 * 512 * 64, kv_stride_h=512 * 64, kv_stride_s=64,
                kv_capacity=512)
    base.update(kw)
    return binding.Desc(**base)


def test_attention_entry_points_validate_before_any_launch():
    """Every call below must fail in validation (no GPU is present or needed)."""
    lib = s1f.load_library()
    p = ctypes.c_void_p(4096)   # non-null, 16-byte aligned, never dereferenced

    def fwd(desc, seg_off=0, seg_len=256, q=p, lse=p):
        return lib.s1f_seg_attn_fwd(ctypes.byref(desc), q, p, p, seg_off, seg_len, p, lse, None)

    assert fwd(_desc(), q=None) == 1
    assert fwd(_desc(), lse=None) == 1
    assert fwd(_desc(), q=ctypes.c_void_p(4100)) == 1            # misaligned
    assert fwd(_desc(n_kv_heads=3)) == 1
    assert fwd(_desc(q_stride_s=60)) == 1
    assert fwd(_desc(kv_stride_h=513 * 64 + 1)) == 1
    assert fwd(_desc(reserved=1)) == 1
    assert fwd(_desc(head_dim=96)) == 2
    assert fwd(_desc(dtype=7)) == 2
    assert fwd(_desc(), seg_off=-1) == 3
    assert fwd(_desc(), seg_len=0) == 3
    assert fwd(_desc(), seg_off=300, seg_len=256) == 3            # past kv_capacity
    assert lib.s1f_seg_attn_fwd(None, p, p, p, 0, 1, p, p, None) == 1

    def bwd(desc, seg_off=0, seg_len=256, ws=p, ws_bytes=1 << 20):
        return lib.s1f_seg_attn_bwd(ctypes.byref(desc), p, p, p, p, p, p, seg_off, seg_len, p, p, p, ws, ws_bytes, None)

    assert bwd(_desc(), ws=None) == 1
    assert bwd(_desc(), ws_bytes=4 * 256 * 4 - 1) == 1
    assert bwd(_desc(), seg_off=400, seg_len=200) == 3
    assert bwd(_desc(head_dim=32)) == 2
    assert lib.s1f_bwd_workspace_bytes(ctypes.byref(_desc()), 0, 256) == 2 * 4 * 256 * 4
    assert lib.s1f_bwd_workspace_bytes(ctypes.byref(_desc()), 500, 256) == 0
    for code in range(0, 6):
        assert isinstance(s1f.strerror(code), str) and s1f.strerror(code)


def test_seq1f1b_order_matches_oracle():
    """The library enumerates the order in closed form; the oracle simulates the queue of Section 3.2."""
    from oracle import schedule as SCH
    for P_ in (1, 2, 3, 4, 8):
        for i in range(1, P_ + 1):
            for M in (1, 2, 3, 4, 7, 9, 16, 33):
                for k in (1, 2, 3, 4, 8):
                    assert s1f.seq1f1b_warmup(P_, i, M, k) == SCH.warmup_count(P_, i, M, k), (P_, i, M, k)
                    assert s1f.seq1f1b_order(P_, i, M, k) == SCH.stage_order(P_, i, M, k), (P_, i, M, k)


def test_seq1f1b_rejects_bad_arguments():
    for bad in ((0, 1, 4, 2), (4, 0, 4, 2), (4, 5, 4, 2), (4, 1, 0, 2), (4, 1, 4, 0)):
        with pytest.raises(s1f.S1FError) as e:
            s1f.seq1f1b_order(*bad)
        assert e.value.status == 1
        with pytest.raises(s1f.S1FError):
            s1f.seq1f1b_warmup(*bad)
    lib = s1f.load_library()
    n = ctypes.c_int64(0)
    buf = (binding.Pass * 4)()
    assert lib.s1f_seq1f1b_order(2, 1, 3, 2, buf, 4, ctypes.byref(n)) == 1      # too small: size reported
    assert n.value == 12
    assert lib.s1f_seq1f1b_order(2, 1, 3, 2, None, 0, ctypes.byref(n)) == 1 and n.value == 12
