"""ctypes binding of the C ABI declared in include/s1f.h (same names, same argument order)."""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libs1f.so")
_lib = None

S1F_F32, S1F_BF16 = 0, 1


class S1FError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: status {status} ({strerror(status)})")


class Desc(ctypes.Structure):
    """Mirror of s1f_desc."""
    _fields_ = [("batch", ctypes.c_int32), ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("dtype", ctypes.c_int32), ("reserved", ctypes.c_int32),
                ("q_stride_b", ctypes.c_int64), ("q_stride_h", ctypes.c_int64), ("q_stride_s", ctypes.c_int64),
                ("kv_stride_b", ctypes.c_int64), ("kv_stride_h", ctypes.c_int64), ("kv_stride_s", ctypes.c_int64),
                ("kv_capacity", ctypes.c_int64)]


class Pass(ctypes.Structure):
    _fields_ = [("micro_batch", ctypes.c_int32), ("segment", ctypes.c_int32), ("backward", ctypes.c_int32)]


class StagePass(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int32), ("micro_batch", ctypes.c_int32), ("segment", ctypes.c_int32),
                ("chunk", ctypes.c_int32)]


class PipelineDesc(ctypes.Structure):
    """Mirror of s1f_pipeline_desc."""
    _fields_ = [("pp_size", ctypes.c_int32), ("n_micro", ctypes.c_int32), ("n_seg", ctypes.c_int32),
                ("n_chunks", ctypes.c_int32), ("split_weight_grad", ctypes.c_int32), ("reserved", ctypes.c_int32),
                ("max_pending_wgrad", ctypes.c_int64), ("t_comm", ctypes.c_int64),
                ("t_fwd", ctypes.POINTER(ctypes.c_int64)), ("t_bwd", ctypes.POINTER(ctypes.c_int64)),
                ("t_wgrad", ctypes.POINTER(ctypes.c_int64)), ("seg_tokens", ctypes.POINTER(ctypes.c_int64))]


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libs1f.so (built in-tree by paper_2406_03488_amd.build).  Raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} not found: build it with `python -m paper_2406_03488_amd.build` "
                          "(there is no fallback implementation)")
    lib = ctypes.CDLL(_LIB_PATH)
    i64, i32, vp, sz = ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p, ctypes.c_size_t
    dp = ctypes.POINTER(Desc)
    lib.s1f_partition.argtypes = [i64, i32, i32, i32, ctypes.POINTER(i64)]
    lib.s1f_partition.restype = ctypes.c_int
    lib.s1f_partition_ex.argtypes = [i64, i32, i32, i32, i32, i64, ctypes.POINTER(i64)]
    lib.s1f_partition_ex.restype = ctypes.c_int
    lib.s1f_partition_rebalance.argtypes = [i32, ctypes.POINTER(i64), ctypes.POINTER(i64), i64, ctypes.POINTER(i64)]
    lib.s1f_partition_rebalance.restype = ctypes.c_int
    lib.s1f_seg_attn_fwd.argtypes = [dp, vp, vp, vp, i64, i64, vp, vp, vp]
    lib.s1f_seg_attn_fwd.restype = ctypes.c_int
    lib.s1f_seg_attn_fwd_ws.argtypes = [dp, vp, vp, vp, i64, i64, vp, vp, vp, sz, vp]
    lib.s1f_seg_attn_fwd_ws.restype = ctypes.c_int
    lib.s1f_fwd_workspace_bytes.argtypes = [dp, i64, i64]
    lib.s1f_fwd_workspace_bytes.restype = sz
    lib.s1f_seg_attn_bwd.argtypes = [dp, vp, vp, vp, vp, vp, vp, i64, i64, vp, vp, vp, vp, sz, vp]
    lib.s1f_seg_attn_bwd.restype = ctypes.c_int
    lib.s1f_seg_attn_bwd_dq.argtypes = [dp, vp, vp, vp, vp, vp, vp, i64, i64, vp, vp, sz, vp]
    lib.s1f_seg_attn_bwd_dq.restype = ctypes.c_int
    lib.s1f_seg_attn_bwd_dkdv.argtypes = [dp, vp, vp, vp, vp, vp, i64, i64, vp, vp, vp, sz, vp]
    lib.s1f_seg_attn_bwd_dkdv.restype = ctypes.c_int
    lib.s1f_seg_attn_bwd_noalloc.argtypes = [dp, vp, vp, vp, vp, vp, vp, i64, i64, vp, vp, vp, vp]
    lib.s1f_seg_attn_bwd_noalloc.restype = ctypes.c_int
    lib.s1f_static_scratch_rows.argtypes = []
    lib.s1f_static_scratch_rows.restype = sz
    lib.s1f_bwd_workspace_bytes.argtypes = [dp, i64, i64]
    lib.s1f_bwd_workspace_bytes.restype = sz
    lib.s1f_kv_append.argtypes = [dp, vp, vp, i64, i64, i64, i64, i64, vp, vp, vp]
    lib.s1f_kv_append.restype = ctypes.c_int
    lib.s1f_kv_grad_emit.argtypes = [dp, vp, vp, i64, i64, vp, vp, i64, i64, i64, vp]
    lib.s1f_kv_grad_emit.restype = ctypes.c_int
    lib.s1f_seq1f1b_warmup.argtypes = [i32, i32, i32, i32, ctypes.POINTER(i64)]
    lib.s1f_seq1f1b_warmup.restype = ctypes.c_int
    lib.s1f_seq1f1b_order.argtypes = [i32, i32, i32, i32, ctypes.POINTER(Pass), i64, ctypes.POINTER(i64)]
    lib.s1f_seq1f1b_order.restype = ctypes.c_int
    lib.s1f_seq1f1b_interleaved_warmup.argtypes = [i32, i32, i32, i32, i32, ctypes.POINTER(i64)]
    lib.s1f_seq1f1b_interleaved_warmup.restype = ctypes.c_int
    lib.s1f_seq1f1b_interleaved_order.argtypes = [i32, i32, i32, i32, i32, ctypes.POINTER(StagePass), i64,
                                                  ctypes.POINTER(i64)]
    lib.s1f_seq1f1b_interleaved_order.restype = ctypes.c_int
    lib.s1f_seq1f1b_peak_memory_share.argtypes = [i32, i32, i32, i32, ctypes.POINTER(i64), ctypes.POINTER(i64)]
    lib.s1f_seq1f1b_peak_memory_share.restype = ctypes.c_int
    lib.s1f_pipeline_simulate.argtypes = [ctypes.POINTER(PipelineDesc), ctypes.POINTER(i64), ctypes.POINTER(i64),
                                          ctypes.POINTER(i64), ctypes.POINTER(i64), ctypes.POINTER(ctypes.c_double)]
    lib.s1f_pipeline_simulate.restype = ctypes.c_int
    lib.s1f_strerror.argtypes = [ctypes.c_int]
    lib.s1f_strerror.restype = ctypes.c_char_p
    lib.s1f_version.argtypes = []
    lib.s1f_version.restype = ctypes.c_int
    _lib = lib
    return lib


def strerror(status: int) -> str:
    return load_library().s1f_strerror(int(status)).decode()


def version() -> int:
    return int(load_library().s1f_version())


def partition(seq_len: int, n_seg: int, hidden: int, heads: int):
    """s1f_partition: list of n_seg + 1 boundaries."""
    lib = load_library()
    out = (ctypes.c_int64 * (max(int(n_seg), 0) + 1))()
    rc = lib.s1f_partition(int(seq_len), int(n_seg), int(hidden), int(heads), out)
    if rc != 0:
        raise S1FError(rc, "s1f_partition")
    return list(out)


COST_ADDITIVE, COST_LITERAL = 0, 1


def partition_ex(seq_len: int, n_seg: int, hidden: int, heads: int, cost_model: int = COST_ADDITIVE, align: int = 1):
    """s1f_partition_ex: list of n_seg + 1 boundaries under the chosen cost model and alignment."""
    out = (ctypes.c_int64 * (max(int(n_seg), 0) + 1))()
    rc = load_library().s1f_partition_ex(int(seq_len), int(n_seg), int(hidden), int(heads), int(cost_model),
                                         int(align), out)
    if rc != 0:
        raise S1FError(rc, "s1f_partition_ex")
    return list(out)


def partition_rebalance(boundaries, seg_cost, align: int = 1):
    """s1f_partition_rebalance: new boundaries from the measured integer cost of each segment."""
    k = len(boundaries) - 1
    if k < 1 or len(seg_cost) != k:
        raise S1FError(1, "s1f_partition_rebalance")
    b_in = (ctypes.c_int64 * (k + 1))(*[int(x) for x in boundaries])
    cost = (ctypes.c_int64 * k)(*[int(x) for x in seg_cost])
    out = (ctypes.c_int64 * (k + 1))()
    rc = load_library().s1f_partition_rebalance(k, b_in, cost, int(align), out)
    if rc != 0:
        raise S1FError(rc, "s1f_partition_rebalance")
    return list(out)


def seq1f1b_warmup(pp_size: int, device: int, n_micro: int, n_seg: int) -> int:
    """s1f_seq1f1b_warmup: sub-sequences forwarded before the first backward pass."""
    w = ctypes.c_int64(0)
    rc = load_library().s1f_seq1f1b_warmup(int(pp_size), int(device), int(n_micro), int(n_seg), ctypes.byref(w))
    if rc != 0:
        raise S1FError(rc, "s1f_seq1f1b_warmup")
    return int(w.value)


def seq1f1b_peak_memory_share(pp_size: int, device: int, n_micro: int, n_seg: int):
    """s1f_seq1f1b_peak_memory_share: (numerator, denominator) of w_i / sum_j w_j."""
    num, den = ctypes.c_int64(0), ctypes.c_int64(0)
    rc = load_library().s1f_seq1f1b_peak_memory_share(int(pp_size), int(device), int(n_micro), int(n_seg),
                                                      ctypes.byref(num), ctypes.byref(den))
    if rc != 0:
        raise S1FError(rc, "s1f_seq1f1b_peak_memory_share")
    return int(num.value), int(den.value)


def seq1f1b_order(pp_size: int, device: int, n_micro: int, n_seg: int):
    """s1f_seq1f1b_order: list of ("F" | "B", micro_batch, segment) in execution order."""
    lib = load_library()
    n = ctypes.c_int64(0)
    cap = 2 * max(int(n_micro), 0) * max(int(n_seg), 0)
    buf = (Pass * max(cap, 1))()
    rc = lib.s1f_seq1f1b_order(int(pp_size), int(device), int(n_micro), int(n_seg), buf, cap, ctypes.byref(n))
    if rc != 0:
        raise S1FError(rc, "s1f_seq1f1b_order")
    return [("B" if buf[i].backward else "F", int(buf[i].micro_batch), int(buf[i].segment)) for i in range(n.value)]


def seq1f1b_interleaved_warmup(pp_size: int, device: int, n_micro: int, n_seg: int, n_chunks: int) -> int:
    """s1f_seq1f1b_interleaved_warmup: sub-sequences forwarded before the first backward pass (Eq. 5-6)."""
    w = ctypes.c_int64(0)
    rc = load_library().s1f_seq1f1b_interleaved_warmup(int(pp_size), int(device), int(n_micro), int(n_seg),
                                                       int(n_chunks), ctypes.byref(w))
    if rc != 0:
        raise S1FError(rc, "s1f_seq1f1b_interleaved_warmup")
    return int(w.value)


def seq1f1b_interleaved_order(pp_size: int, device: int, n_micro: int, n_seg: int, n_chunks: int):
    """s1f_seq1f1b_interleaved_order: list of ("F" | "B", micro_batch, segment, chunk) in execution order."""
    n = ctypes.c_int64(0)
    cap = 2 * max(int(n_micro), 0) * max(int(n_seg), 0) * max(int(n_chunks), 0)
    buf = (StagePass * max(cap, 1))()
    rc = load_library().s1f_seq1f1b_interleaved_order(int(pp_size), int(device), int(n_micro), int(n_seg),
                                                      int(n_chunks), buf, cap, ctypes.byref(n))
    if rc != 0:
        raise S1FError(rc, "s1f_seq1f1b_interleaved_order")
    return [("B" if buf[i].kind else "F", int(buf[i].micro_batch), int(buf[i].segment), int(buf[i].chunk))
            for i in range(n.value)]


def pipeline_simulate(pp_size: int, n_micro: int, n_seg: int, n_chunks: int, t_fwd, t_bwd, t_wgrad=None,
                      t_comm: int = 0, max_pending_wgrad: int = 0, seg_tokens=None):
    """s1f_pipeline_simulate: dict with makespan, busy, peak_live, peak_pending (lists over devices) and
    bubble_ratio, all as the library returns them."""
    k, P = int(n_seg), int(pp_size)
    if k < 1 or P < 1 or len(t_fwd) != k or len(t_bwd) != k or (t_wgrad is not None and len(t_wgrad) != k) or (
            seg_tokens is not None and len(seg_tokens) != k):
        raise S1FError(1, "s1f_pipeline_simulate")
    arr = lambda xs: (ctypes.c_int64 * k)(*[int(x) for x in xs])
    keep = [arr(t_fwd), arr(t_bwd), arr(t_wgrad) if t_wgrad is not None else None,
            arr(seg_tokens) if seg_tokens is not None else None]
    desc = PipelineDesc(P, int(n_micro), k, int(n_chunks), 1 if t_wgrad is not None else 0, 0, int(max_pending_wgrad),
                        int(t_comm), keep[0], keep[1], keep[2], keep[3])
    span = ctypes.c_int64(0)
    busy, live, pend = ((ctypes.c_int64 * P)() for _ in range(3))
    bubble = ctypes.c_double(0.0)
    rc = load_library().s1f_pipeline_simulate(ctypes.byref(desc), ctypes.byref(span), busy, live, pend,
                                              ctypes.byref(bubble))
    if rc != 0:
        raise S1FError(rc, "s1f_pipeline_simulate")
    return {"makespan": int(span.value), "busy": list(busy), "peak_live": list(live), "peak_pending": list(pend),
            "bubble_ratio": float(bubble.value)}


def _dtype_code(t):
    import torch
    if t.dtype == torch.float32:
        return S1F_F32
    if t.dtype == torch.bfloat16:
        return S1F_BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def make_desc(q_like, kv_like) -> Desc:
    """Descriptor from a [B, Hq, S, D] query-shaped tensor and a [B, Hkv, C, D] prefix-shaped tensor."""
    if q_like.dim() != 4 or kv_like.dim() != 4 or q_like.stride(3) != 1 or kv_like.stride(3) != 1:
        raise ValueError("expected [batch, heads, seq, head_dim] tensors with contiguous head_dim")
    b, hq, _, d = q_like.shape
    return Desc(batch=b, n_q_heads=hq, n_kv_heads=kv_like.shape[1], head_dim=d, dtype=_dtype_code(q_like), reserved=0,
                q_stride_b=q_like.stride(0), q_stride_h=q_like.stride(1), q_stride_s=q_like.stride(2),
                kv_stride_b=kv_like.stride(0), kv_stride_h=kv_like.stride(1), kv_stride_s=kv_like.stride(2),
                kv_capacity=kv_like.shape[2])


def _stream_ptr():
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _same_layout(ref, *others):
    for t in others:
        if t.shape != ref.shape or t.stride() != ref.stride() or t.dtype != ref.dtype:
            raise ValueError("tensors sharing a stride set must have identical shape, strides and dtype")


def seg_attn_fwd(q_seg, k_prefix, v_prefix, seg_off: int, out, lse):
    """s1f_seg_attn_fwd on torch device tensors.

    q_seg/out [B, Hq, seg_len, D]; k_prefix/v_prefix [B, Hkv, capacity, D] (row 0 of the cache);
    lse [B, Hq, seg_len] fp32 contiguous.  Enqueued on torch's current stream.
    """
    lib = load_library()
    _same_layout(q_seg, out)
    _same_layout(k_prefix, v_prefix)
    if not lse.is_contiguous() or lse.shape != q_seg.shape[:3]:
        raise ValueError("lse must be a contiguous [B, Hq, seg_len] fp32 tensor")
    desc = make_desc(q_seg, k_prefix)
    rc = lib.s1f_seg_attn_fwd(ctypes.byref(desc), q_seg.data_ptr(), k_prefix.data_ptr(), v_prefix.data_ptr(),
                              int(seg_off), int(q_seg.shape[2]), out.data_ptr(), lse.data_ptr(), _stream_ptr())
    if rc != 0:
        raise S1FError(rc, "s1f_seg_attn_fwd")


def fwd_workspace_bytes(q_seg, k_prefix, seg_off: int) -> int:
    desc = make_desc(q_seg, k_prefix)
    return int(load_library().s1f_fwd_workspace_bytes(ctypes.byref(desc), int(seg_off), int(q_seg.shape[2])))


def seg_attn_fwd_ws(q_seg, k_prefix, v_prefix, seg_off: int, out, lse, workspace):
    """s1f_seg_attn_fwd_ws on torch device tensors: seg_attn_fwd with a device workspace of at least
    fwd_workspace_bytes(...) bytes (None is accepted when that is 0)."""
    lib = load_library()
    _same_layout(q_seg, out)
    _same_layout(k_prefix, v_prefix)
    _check_lse(lse, q_seg)
    desc = make_desc(q_seg, k_prefix)
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    rc = lib.s1f_seg_attn_fwd_ws(ctypes.byref(desc), q_seg.data_ptr(), k_prefix.data_ptr(), v_prefix.data_ptr(),
                                 int(seg_off), int(q_seg.shape[2]), out.data_ptr(), lse.data_ptr(), ws_ptr, ws_bytes,
                                 _stream_ptr())
    if rc != 0:
        raise S1FError(rc, "s1f_seg_attn_fwd_ws")


def bwd_workspace_bytes(q_seg, k_prefix, seg_off: int) -> int:
    desc = make_desc(q_seg, k_prefix)
    return int(load_library().s1f_bwd_workspace_bytes(ctypes.byref(desc), int(seg_off), int(q_seg.shape[2])))


def _check_lse(lse, q_seg):
    import torch
    if lse.dtype != torch.float32:
        raise TypeError("lse is fp32")
    if not lse.is_contiguous() or lse.shape != q_seg.shape[:3]:
        raise ValueError("lse must be a contiguous [B, Hq, seg_len] fp32 tensor")


def _check_acc(k_prefix, v_prefix, dk_prefix_acc, dv_prefix_acc):
    import torch
    _same_layout(k_prefix, v_prefix)
    _same_layout(dk_prefix_acc, dv_prefix_acc)
    if dk_prefix_acc.shape != k_prefix.shape or dk_prefix_acc.stride() != k_prefix.stride():
        raise ValueError("gradient accumulators must have the shape and strides of k_prefix")
    if dk_prefix_acc.dtype != torch.float32:
        raise TypeError("accumulators are fp32")


def _check_bwd_tensors(dout, q_seg, k_prefix, v_prefix, out, lse, dq, dk_prefix_acc, dv_prefix_acc):
    _same_layout(q_seg, dout, out, dq)
    _check_acc(k_prefix, v_prefix, dk_prefix_acc, dv_prefix_acc)
    _check_lse(lse, q_seg)


def seg_attn_bwd(dout, q_seg, k_prefix, v_prefix, out, lse, seg_off: int, dq, dk_prefix_acc, dv_prefix_acc, workspace):
    """s1f_seg_attn_bwd on torch device tensors.

    dk_prefix_acc/dv_prefix_acc are fp32 tensors with the shape and strides of k_prefix; workspace is any
    device tensor of at least bwd_workspace_bytes(...) bytes.
    """
    lib = load_library()
    _check_bwd_tensors(dout, q_seg, k_prefix, v_prefix, out, lse, dq, dk_prefix_acc, dv_prefix_acc)
    desc = make_desc(q_seg, k_prefix)
    rc = lib.s1f_seg_attn_bwd(ctypes.byref(desc), dout.data_ptr(), q_seg.data_ptr(), k_prefix.data_ptr(),
                              v_prefix.data_ptr(), out.data_ptr(), lse.data_ptr(), int(seg_off), int(q_seg.shape[2]),
                              dq.data_ptr(), dk_prefix_acc.data_ptr(), dv_prefix_acc.data_ptr(),
                              workspace.data_ptr(), workspace.numel() * workspace.element_size(), _stream_ptr())
    if rc != 0:
        raise S1FError(rc, "s1f_seg_attn_bwd")


def static_scratch_rows() -> int:
    return int(load_library().s1f_static_scratch_rows())


def seg_attn_bwd_noalloc(dout, q_seg, k_prefix, v_prefix, out, lse, seg_off: int, dq, dk_prefix_acc, dv_prefix_acc):
    """s1f_seg_attn_bwd_noalloc on torch device tensors: s1f_seg_attn_bwd without a workspace argument."""
    lib = load_library()
    _check_bwd_tensors(dout, q_seg, k_prefix, v_prefix, out, lse, dq, dk_prefix_acc, dv_prefix_acc)
    desc = make_desc(q_seg, k_prefix)
    rc = lib.s1f_seg_attn_bwd_noalloc(ctypes.byref(desc), dout.data_ptr(), q_seg.data_ptr(), k_prefix.data_ptr(),
                                      v_prefix.data_ptr(), out.data_ptr(), lse.data_ptr(), int(seg_off),
                                      int(q_seg.shape[2]), dq.data_ptr(), dk_prefix_acc.data_ptr(),
                                      dv_prefix_acc.data_ptr(), _stream_ptr())
    if rc != 0:
        raise S1FError(rc, "s1f_seg_attn_bwd_noalloc")


def seg_attn_bwd_dq(dout, q_seg, k_prefix, v_prefix, out, lse, seg_off: int, dq, workspace):
    """s1f_seg_attn_bwd_dq: first half of the backward (dq, and delta into the workspace)."""
    lib = load_library()
    _same_layout(q_seg, dout, out, dq)
    _same_layout(k_prefix, v_prefix)
    _check_lse(lse, q_seg)
    desc = make_desc(q_seg, k_prefix)
    rc = lib.s1f_seg_attn_bwd_dq(ctypes.byref(desc), dout.data_ptr(), q_seg.data_ptr(), k_prefix.data_ptr(),
                                 v_prefix.data_ptr(), out.data_ptr(), lse.data_ptr(), int(seg_off),
                                 int(q_seg.shape[2]), dq.data_ptr(), workspace.data_ptr(),
                                 workspace.numel() * workspace.element_size(), _stream_ptr())
    if rc != 0:
        raise S1FError(rc, "s1f_seg_attn_bwd_dq")


def seg_attn_bwd_dkdv(dout, q_seg, k_prefix, v_prefix, lse, seg_off: int, dk_prefix_acc, dv_prefix_acc, workspace):
    """s1f_seg_attn_bwd_dkdv: second half of the backward (prefix dK/dV accumulation)."""
    lib = load_library()
    _same_layout(q_seg, dout)
    _check_acc(k_prefix, v_prefix, dk_prefix_acc, dv_prefix_acc)
    _check_lse(lse, q_seg)
    desc = make_desc(q_seg, k_prefix)
    rc = lib.s1f_seg_attn_bwd_dkdv(ctypes.byref(desc), dout.data_ptr(), q_seg.data_ptr(), k_prefix.data_ptr(),
                                   v_prefix.data_ptr(), lse.data_ptr(), int(seg_off), int(q_seg.shape[2]),
                                   dk_prefix_acc.data_ptr(), dv_prefix_acc.data_ptr(), workspace.data_ptr(),
                                   workspace.numel() * workspace.element_size(), _stream_ptr())
    if rc != 0:
        raise S1FError(rc, "s1f_seg_attn_bwd_dkdv")


def _kv_desc(cache) -> Desc:
    """Descriptor for the cache-side calls: only the kv_* fields, dtype, batch and head_dim are read."""
    if cache.dim() != 4 or cache.stride(3) != 1:
        raise ValueError("expected a [batch, kv_heads, capacity, head_dim] tensor with contiguous head_dim")
    b, h, cap, d = cache.shape
    return Desc(batch=b, n_q_heads=h, n_kv_heads=h, head_dim=d, dtype=0, reserved=0, q_stride_b=0, q_stride_h=0,
                q_stride_s=d, kv_stride_b=cache.stride(0), kv_stride_h=cache.stride(1), kv_stride_s=cache.stride(2),
                kv_capacity=cap)


def kv_append(k_seg, v_seg, seg_off: int, k_cache, v_cache):
    """s1f_kv_append: rows of the segment -> rows [seg_off, seg_off + seg_len) of the caches."""
    lib = load_library()
    _same_layout(k_seg, v_seg)
    _same_layout(k_cache, v_cache)
    desc = _kv_desc(k_cache)
    desc.dtype = _dtype_code(k_cache)
    if k_seg.dtype != k_cache.dtype or k_seg.stride(3) != 1:
        raise ValueError("segment and cache must share the element type; head_dim must be contiguous")
    rc = lib.s1f_kv_append(ctypes.byref(desc), k_seg.data_ptr(), v_seg.data_ptr(), k_seg.stride(0), k_seg.stride(1),
                           k_seg.stride(2), int(seg_off), k_seg.shape[2], k_cache.data_ptr(), v_cache.data_ptr(),
                           _stream_ptr())
    if rc != 0:
        raise S1FError(rc, "s1f_kv_append")


def kv_grad_emit(dk_prefix_acc, dv_prefix_acc, seg_off: int, dk_seg, dv_seg):
    """s1f_kv_grad_emit: final rows [seg_off, seg_off + seg_len) of the fp32 accumulators -> dk_seg, dv_seg."""
    import torch
    lib = load_library()
    _same_layout(dk_prefix_acc, dv_prefix_acc)
    _same_layout(dk_seg, dv_seg)
    if dk_prefix_acc.dtype != torch.float32 or dk_seg.stride(3) != 1:
        raise ValueError("accumulators must be fp32; head_dim must be contiguous")
    desc = _kv_desc(dk_prefix_acc)
    desc.dtype = _dtype_code(dk_seg)
    rc = lib.s1f_kv_grad_emit(ctypes.byref(desc), dk_prefix_acc.data_ptr(), dv_prefix_acc.data_ptr(), int(seg_off),
                              dk_seg.shape[2], dk_seg.data_ptr(), dv_seg.data_ptr(), dk_seg.stride(0), dk_seg.stride(1),
                              dk_seg.stride(2), _stream_ptr())
    if rc != 0:
        raise S1FError(rc, "s1f_kv_grad_emit")
