"""The backward entry point that allocates nothing (s1f_seg_attn_bwd_noalloc: row statistics in a device array
built into the library) against s1f_seg_attn_bwd with a caller-owned workspace: same kernels, so the fp32
accumulators must agree bit for bit, and dQ too unless the two cut the dQ launch into different key chunks (the
built-in scratch holds fewer partial rows), which reorders fp32 sums: then to the contract's bf16 tolerance.  Two calls in a row, the second on a smaller segment, so that whatever
the first call left in the shared array cannot leak into the second."""
import ctypes

import pytest
import torch

import paper_2406_03488_amd as s1f
import s1f_synth as S
from paper_2406_03488_amd import binding

pytestmark = pytest.mark.gpu


def _segment(seed, hq, hkv, off, m, d, dtype):
    from gpu_harness import to_device
    n = off + m
    q, do = (to_device(S.tensor(seed, t, hq, n, d, dtype)[:, off:], dtype)[None].contiguous() for t in ("q", "dout"))
    k, v = (to_device(S.tensor(seed, t, hkv, n, d, dtype), dtype)[None] for t in ("k", "v"))
    out = torch.empty_like(q)
    lse = torch.empty((1, hq, m), dtype=torch.float32, device="cuda")
    s1f.seg_attn_fwd(q, k, v, off, out, lse)
    return q, k, v, do, out, lse


@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("f32", 64)])
def test_noalloc_backward_equals_workspace_backward(dtype, d):
    lib = s1f.load_library()
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    for seed, (hq, hkv, off, m) in enumerate([(8, 2, 700, 900), (4, 4, 130, 77)]):   # second call: smaller input
        q, k, v, do, out, lse = _segment(60 + seed, hq, hkv, off, m, d, dtype)
        got = {}
        for mode in ("workspace", "noalloc"):
            dq = torch.full_like(q, float("nan"))
            dk = torch.full((1, hkv, off + m, d), 0.25, dtype=torch.float32, device="cuda")
            dv = torch.full_like(dk, -0.5)
            desc = binding.make_desc(q, k)
            common = (ctypes.byref(desc), do.data_ptr(), q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(),
                      lse.data_ptr(), off, m, dq.data_ptr(), dk.data_ptr(), dv.data_ptr())
            if mode == "workspace":
                ws = torch.empty(s1f.bwd_workspace_bytes(q, k, off), dtype=torch.uint8, device="cuda")
                rc = lib.s1f_seg_attn_bwd(*common, ws.data_ptr(), ws.numel(), stream)
            else:
                rc = lib.s1f_seg_attn_bwd_noalloc(*common, stream)
            assert rc == 0, (mode, rc, s1f.strerror(rc))
            torch.cuda.synchronize()
            got[mode] = (dq, dk, dv)
        for a, b, name in zip(got["workspace"], got["noalloc"], ("dq", "dk", "dv")):
            assert torch.isfinite(b).all(), name
            if name == "dq" and not torch.equal(a, b):
                diff = (a.float() - b.float()).abs().max().item()
                assert diff <= (2e-2 if dtype == "bf16" else 1e-4), f"dq differs by {diff} (call {seed})"
            else:
                assert torch.equal(a, b), f"{name} differs between the two entry points (call {seed})"
