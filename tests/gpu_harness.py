"""Drives the library through its Python binding the way a pipeline stage would (Sections 3.1-3.2):
forward of segments in order, then backward in reverse order with fp32 dK/dV accumulation.  Used by the
GPU parity tests; holds no attention arithmetic of its own."""
import numpy as np
import torch

import paper_2406_03488_amd as s1f


def to_device(x: np.ndarray, dtype: str) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32))
    if dtype == "bf16":
        t = t.to(torch.bfloat16)      # exact: the generator already rounded the values to bf16
    return t.cuda()


def run_schedule(q, k, v, dout, boundaries, dtype, capacity=None, layout="bhsd", finality=None):
    """q, dout [Hq, n, D]; k, v [Hkv, n, D] numpy fp32.  Returns dict of numpy fp64 results.

    layout "bshd" stores the tensors as [B, S, H, D] and hands permuted views to the library, which
    exercises the stride arguments.  `finality`, if a list, receives (segment index, dk copy, dv copy)
    after each backward call.
    """
    hq, n, d = q.shape
    hkv = k.shape[0]
    cap = n if capacity is None else capacity
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32

    def alloc(h, s, dt, fill=None):
        if layout == "bshd":
            t = torch.empty((1, s, h, d), dtype=dt, device="cuda").permute(0, 2, 1, 3)
        else:
            t = torch.empty((1, h, s, d), dtype=dt, device="cuda")
        if fill is not None:
            t.fill_(fill)
        return t

    kc, vc = alloc(hkv, cap, tdt, 0.0), alloc(hkv, cap, tdt, 0.0)
    kc[0, :, :n].copy_(to_device(k, dtype)); vc[0, :, :n].copy_(to_device(v, dtype))
    dk_acc, dv_acc = alloc(hkv, cap, torch.float32, 0.0), alloc(hkv, cap, torch.float32, 0.0)
    if cap > n:   # rows past the sequence must never be touched
        dk_acc[0, :, n:] = 777.0; dv_acc[0, :, n:] = 777.0
    qd, dod = to_device(q, dtype), to_device(dout, dtype)
    nseg = len(boundaries) - 1
    saved = []
    for i in range(nseg):
        a, b = boundaries[i], boundaries[i + 1]
        qs = alloc(hq, b - a, tdt); qs[0].copy_(qd[:, a:b])
        out = alloc(hq, b - a, tdt, float("nan"))
        lse = torch.full((1, hq, b - a), float("nan"), dtype=torch.float32, device="cuda")
        s1f.seg_attn_fwd(qs, kc, vc, a, out, lse)
        saved.append((qs, out, lse))
    outs = np.empty((hq, n, d)); lses = np.empty((hq, n)); dqs = np.empty((hq, n, d))
    for i in reversed(range(nseg)):
        a, b = boundaries[i], boundaries[i + 1]
        qs, out, lse = saved[i]
        dos = alloc(hq, b - a, tdt); dos[0].copy_(dod[:, a:b])
        dq = alloc(hq, b - a, tdt, float("nan"))
        ws = torch.empty(s1f.bwd_workspace_bytes(qs, kc, a), dtype=torch.uint8, device="cuda")
        s1f.seg_attn_bwd(dos, qs, kc, vc, out, lse, a, dq, dk_acc, dv_acc, ws)
        outs[:, a:b] = out[0].float().cpu().numpy(); lses[:, a:b] = lse[0].cpu().numpy()
        dqs[:, a:b] = dq[0].float().cpu().numpy()
        if finality is not None:
            finality.append((i, dk_acc[0].cpu().numpy().copy(), dv_acc[0].cpu().numpy().copy()))
    torch.cuda.synchronize()
    return {"out": outs, "lse": lses, "dq": dqs, "dk": dk_acc[0].cpu().numpy().astype(np.float64),
            "dv": dv_acc[0].cpu().numpy().astype(np.float64)}


def errors(got: np.ndarray, want: np.ndarray):
    """(max abs error, relative Frobenius error)."""
    diff = np.asarray(got, dtype=np.float64) - np.asarray(want, dtype=np.float64)
    return float(np.abs(diff).max()), float(np.linalg.norm(diff) / max(np.linalg.norm(want), 1e-300))
