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


def _alloc(layout, batch, h, s, d, dt, fill=None):
    if layout == "bshd":
        t = torch.empty((batch, s, h, d), dtype=dt, device="cuda").permute(0, 2, 1, 3)
    else:
        t = torch.empty((batch, h, s, d), dtype=dt, device="cuda")
    if fill is not None:
        t.fill_(fill)
    return t


def forward(qs, kc, vc, seg_off, out, lse, with_workspace=True):
    """s1f_seg_attn_fwd_ws with a workspace of the size the library asks for (the path the benchmark times), or the
    plain s1f_seg_attn_fwd."""
    if not with_workspace:
        s1f.seg_attn_fwd(qs, kc, vc, seg_off, out, lse)
        return
    nbytes = s1f.fwd_workspace_bytes(qs, kc, seg_off)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda") if nbytes else None
    s1f.seg_attn_fwd_ws(qs, kc, vc, seg_off, out, lse, ws)


def run_schedule_batched(q, k, v, dout, boundaries, dtype, capacity=None, layout="bhsd", finality=None,
                         cache_kernels=False, fwd_workspace=True):
    """q, dout [B, Hq, n, D]; k, v [B, Hkv, n, D] numpy fp32: B independent sequences in one set of calls.
    Returns dict of numpy fp64 results with the same leading batch dimension.

    layout "bshd" stores the tensors as [B, S, H, D] and hands permuted views to the library, which
    exercises the stride arguments.  `finality`, if a list, receives (segment index, dk copy, dv copy)
    after each backward call.  With `cache_kernels` the K/V rows of a segment reach the cache through
    s1f_kv_append right before its forward pass (rows not yet appended hold NaN), and its final dK/dV rows
    are emitted by s1f_kv_grad_emit right after its backward pass ("dk_emit", "dv_emit" in the result).
    """
    nb, hq, n, d = q.shape
    hkv = k.shape[1]
    cap = n if capacity is None else capacity
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32

    def alloc(h, s, dt, fill=None):
        return _alloc(layout, nb, h, s, d, dt, fill)

    kd, vd = to_device(k, dtype), to_device(v, dtype)
    if cache_kernels:
        kc, vc = alloc(hkv, cap, tdt, float("nan")), alloc(hkv, cap, tdt, float("nan"))
    else:
        kc, vc = alloc(hkv, cap, tdt, 0.0), alloc(hkv, cap, tdt, 0.0)
        kc[:, :, :n].copy_(kd); vc[:, :, :n].copy_(vd)
    dk_acc, dv_acc = alloc(hkv, cap, torch.float32, 0.0), alloc(hkv, cap, torch.float32, 0.0)
    if cap > n:   # rows past the sequence must never be touched
        dk_acc[:, :, n:] = 777.0; dv_acc[:, :, n:] = 777.0
    dk_emit = alloc(hkv, n, tdt, float("nan")) if cache_kernels else None
    dv_emit = alloc(hkv, n, tdt, float("nan")) if cache_kernels else None
    qd, dod = to_device(q, dtype), to_device(dout, dtype)
    nseg = len(boundaries) - 1
    saved = []
    for i in range(nseg):
        a, b = boundaries[i], boundaries[i + 1]
        if cache_kernels:
            ks = alloc(hkv, b - a, tdt); ks.copy_(kd[:, :, a:b])
            vs = alloc(hkv, b - a, tdt); vs.copy_(vd[:, :, a:b])
            s1f.kv_append(ks, vs, a, kc, vc)
        qs = alloc(hq, b - a, tdt); qs.copy_(qd[:, :, a:b])
        out = alloc(hq, b - a, tdt, float("nan"))
        lse = torch.full((nb, hq, b - a), float("nan"), dtype=torch.float32, device="cuda")
        forward(qs, kc, vc, a, out, lse, fwd_workspace)
        saved.append((qs, out, lse))
    outs = np.empty((nb, hq, n, d)); lses = np.empty((nb, hq, n)); dqs = np.empty((nb, hq, n, d))
    for i in reversed(range(nseg)):
        a, b = boundaries[i], boundaries[i + 1]
        qs, out, lse = saved[i]
        dos = alloc(hq, b - a, tdt); dos.copy_(dod[:, :, a:b])
        dq = alloc(hq, b - a, tdt, float("nan"))
        ws = torch.empty(s1f.bwd_workspace_bytes(qs, kc, a), dtype=torch.uint8, device="cuda")
        s1f.seg_attn_bwd(dos, qs, kc, vc, out, lse, a, dq, dk_acc, dv_acc, ws)
        if cache_kernels:
            s1f.kv_grad_emit(dk_acc, dv_acc, a, dk_emit[:, :, a:b], dv_emit[:, :, a:b])
        outs[:, :, a:b] = out.float().cpu().numpy(); lses[:, :, a:b] = lse.cpu().numpy()
        dqs[:, :, a:b] = dq.float().cpu().numpy()
        if finality is not None:
            finality.append((i, dk_acc.cpu().numpy().copy(), dv_acc.cpu().numpy().copy()))
    torch.cuda.synchronize()
    res = {"out": outs, "lse": lses, "dq": dqs, "dk": dk_acc.cpu().numpy().astype(np.float64),
           "dv": dv_acc.cpu().numpy().astype(np.float64)}
    if cache_kernels:
        res["dk_emit"] = dk_emit.float().cpu().numpy().astype(np.float64)
        res["dv_emit"] = dv_emit.float().cpu().numpy().astype(np.float64)
        res["k_cache"] = kc.float().cpu().numpy(); res["v_cache"] = vc.float().cpu().numpy()
    return res


def run_schedule(q, k, v, dout, boundaries, dtype, capacity=None, layout="bhsd", finality=None, fwd_workspace=True):
    """One sequence: q, dout [Hq, n, D]; k, v [Hkv, n, D] numpy fp32.  Results without a batch dimension;
    `finality` entries are (segment index, dk [Hkv, cap, D], dv)."""
    fin = [] if finality is not None else None
    res = run_schedule_batched(q[None], k[None], v[None], dout[None], boundaries, dtype, capacity, layout, fin,
                               fwd_workspace=fwd_workspace)
    if finality is not None:
        finality.extend((i, dk[0], dv[0]) for i, dk, dv in fin)
    return {name: x[0] for name, x in res.items()}


def run_segment(q_seg, k, v, dout_seg, seg_off, dtype, layout="bhsd", fwd_workspace=True):
    """One forward and one backward call for a single segment at offset seg_off: q_seg, dout_seg [Hq, m, D];
    k, v [Hkv, seg_off + m, D].  dk/dv are what this segment's rows alone add to zeroed accumulators."""
    hq, m, d = q_seg.shape
    hkv, c, _ = k.shape
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    kc, vc = _alloc(layout, 1, hkv, c, d, tdt), _alloc(layout, 1, hkv, c, d, tdt)
    kc[0].copy_(to_device(k, dtype)); vc[0].copy_(to_device(v, dtype))
    qs, dos = _alloc(layout, 1, hq, m, d, tdt), _alloc(layout, 1, hq, m, d, tdt)
    qs[0].copy_(to_device(q_seg, dtype)); dos[0].copy_(to_device(dout_seg, dtype))
    out, dq = _alloc(layout, 1, hq, m, d, tdt, float("nan")), _alloc(layout, 1, hq, m, d, tdt, float("nan"))
    lse = torch.full((1, hq, m), float("nan"), dtype=torch.float32, device="cuda")
    dk_acc, dv_acc = _alloc(layout, 1, hkv, c, d, torch.float32, 0.0), _alloc(layout, 1, hkv, c, d, torch.float32, 0.0)
    forward(qs, kc, vc, seg_off, out, lse, fwd_workspace)
    ws = torch.empty(s1f.bwd_workspace_bytes(qs, kc, seg_off), dtype=torch.uint8, device="cuda")
    s1f.seg_attn_bwd(dos, qs, kc, vc, out, lse, seg_off, dq, dk_acc, dv_acc, ws)
    torch.cuda.synchronize()
    f = lambda t: t[0].float().cpu().numpy().astype(np.float64)
    return {"out": f(out), "lse": f(lse), "dq": f(dq), "dk": f(dk_acc), "dv": f(dv_acc)}


def errors(got: np.ndarray, want: np.ndarray):
    """(max abs error, relative Frobenius error)."""
    diff = np.asarray(got, dtype=np.float64) - np.asarray(want, dtype=np.float64)
    return float(np.abs(diff).max()), float(np.linalg.norm(diff) / max(np.linalg.norm(want), 1e-300))
