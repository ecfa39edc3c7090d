#!/usr/bin/env python3
"""Benchmark of the segmented causal attention hot path on one MI355X.

One step = one pass of the whole path over one synthetic sequence: the host partitioner, the forward of
every segment in order, the zero-fill of the fp32 dK/dV accumulators, and the backward of every segment
in reverse order (Sections 3.1, 3.2 and 3.4 of the Seq1F1B paper).  Inputs are resident in HBM before
the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload gqa|30b|7b|2.7b|30b-uniform|tiny]

The headline workload is the largest one of the contract that fits one GPU (gqa: 131072 tokens, 32 segments, 64
query heads on 8 K/V heads); the 7b, 30b and 2.7b workloads are run briefly in the same command and reported under
"other_workloads".
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_F32_TFLOPS = 157.3     # MI355X fp32 matrix


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="gqa")
    ap.add_argument("--others", default="7b,30b,2.7b", help="workloads reported briefly next to the headline ('' for none)")
    ap.add_argument("--constant-data", action="store_true",
                    help="fill Q, K, V and dO with one constant instead of N(0,1): same instructions, hardly a bit "
                         "toggling (shows how much of the kernels' time is the chip's power limit)")
    ap.add_argument("--probe-atomics", action="store_true",
                    help="also measure the rate of fp32 global atomic adds in the access shape a fused dQ would use")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-unsegmented", action="store_true")
    ap.add_argument("--no-graph", action="store_true", help="skip the replay of the step recorded as one HIP graph")
    ap.add_argument("--no-balance", action="store_true", help="skip the cwp-vs-uniform load-balance report")
    ap.add_argument("--no-mfma-probe", action="store_true", help="skip the measured matrix-peak microbenchmark")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run one 1 GiB device-to-device copy first (reference for HBM byte counters)")
    return ap.parse_args()


def measured_traffic(kernel, workload):
    """HBM bytes per launch of `kernel` measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE for this workload
    (recorded in the summaries under profiles/), or None if no profile covers it."""
    import glob
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*.txt"))):
        for line in open(path):
            f = line.split()
            if len(f) == 4 and f[0] == "traffic_bytes_per_launch" and f[1] == kernel and f[2] == workload:
                return float(f[3])
    return None


def seg_pairs(bounds):
    """Causal (query, key) pairs per head of each segment."""
    return [(b - a) * a + (b - a) * (b - a + 1) // 2 for a, b in zip(bounds[:-1], bounds[1:])]


def measured_mfma_peak(torch):
    """TFLOP/s of register-resident back-to-back v_mfma_f32_32x32x16_bf16 on every SIMD (two waves per SIMD),
    measured in this run with the probe kernel of libs1f_probe.so: (constant operands, operands that change from
    instruction to instruction).  The second is the rate the matrix pipe sustains under the chip's power limit
    when the data toggles like real activations."""
    import ctypes
    lib = ctypes.CDLL(os.path.join(ROOT, "paper_2406_03488_amd", "libs1f_probe.so"))
    lib.s1f_probe_mfma_bf16.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
    lib.s1f_probe_mfma_bf16.restype = ctypes.c_int
    wgs, iters = 512, 4000
    sink = torch.zeros(wgs * 256, dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    best = [0.0, 0.0]
    for varied in (0, 1):
        for rep in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            if lib.s1f_probe_mfma_bf16(wgs, iters, varied, sink.data_ptr(), stream) != 0:
                raise RuntimeError("matrix-peak probe failed to launch")
            e1.record()
            torch.cuda.synchronize()
            flops = wgs * 4 * 16.0 * iters * 32768.0
            best[varied] = max(best[varied], flops / (e0.elapsed_time(e1) * 1e-3) / 1e12)
    return best


KERNEL_NAMES = {"fwd": "seg_attn_fwd_kernel", "bwd_dq": "seg_attn_bwd_dq_kernel", "bwd_dkdv": "seg_attn_bwd_dkdv_kernel"}


class Stage:
    """Device buffers of one pipeline stage's attention for one sequence, and the step that uses them."""

    def __init__(self, w, torch, s1f, constant_data=False):
        self.w, self.torch, self.s1f = w, torch, s1f
        dt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
        gen = torch.Generator(device="cuda")
        gen.manual_seed(w.seed)
        n, d = w.seq_len, w.head_dim

        def rnd(h):
            if constant_data:
                return torch.full((1, h, n, d), 0.5, device="cuda", dtype=dt)
            return torch.randn((1, h, n, d), generator=gen, device="cuda", dtype=torch.float32).to(dt)

        self.q, self.dout = rnd(w.n_q_heads), rnd(w.n_q_heads)
        self.k, self.v = rnd(w.n_kv_heads), rnd(w.n_kv_heads)
        self.out = torch.empty_like(self.q)
        self.dq = torch.empty_like(self.q)
        self.dk = torch.empty((1, w.n_kv_heads, n, d), device="cuda", dtype=torch.float32)
        self.dv = torch.empty_like(self.dk)
        self.lse_flat = torch.empty(w.n_q_heads * n, device="cuda", dtype=torch.float32)
        # workspaces at the library's upper limits (row statistics + 512 MiB of partial rows; 513 MiB forward), so that
        # any list of boundaries fits; every call still checks its own size
        self.ws = torch.empty(2 * w.n_q_heads * (n + 64) + (513 << 18), device="cuda", dtype=torch.float32)
        self.fwd_ws = torch.empty(514 << 20, device="cuda", dtype=torch.uint8)
        self.events = []     # (kind, segment, start, end) recorded inside timed steps

    def boundaries(self, n_seg=None, kind=None):
        w = self.w
        n_seg = w.n_seg if n_seg is None else n_seg
        kind = w.partition if kind is None else kind
        if isinstance(kind, (list, tuple)):           # explicit boundaries
            return list(kind)
        if kind == "cwp":
            return self.s1f.partition(w.seq_len, n_seg, w.hidden, w.n_q_heads)
        if kind == "cwp_literal":                      # Eq. 8's per-segment line as printed
            return self.s1f.partition_ex(w.seq_len, n_seg, w.hidden, w.n_q_heads, self.s1f.COST_LITERAL, 1)
        if kind.startswith("cwp_aligned"):             # boundaries on multiples of e.g. 128 tokens
            return self.s1f.partition_ex(w.seq_len, n_seg, w.hidden, w.n_q_heads, self.s1f.COST_ADDITIVE,
                                         int(kind[len("cwp_aligned"):]))
        return [(i * w.seq_len) // n_seg for i in range(n_seg + 1)]

    def step(self, n_seg=None, kind=None, record=False):
        torch, s1f, w = self.torch, self.s1f, self.w
        bounds = self.boundaries(n_seg, kind)
        segs = []
        off = 0
        for a, b in zip(bounds[:-1], bounds[1:]):
            lse = self.lse_flat[off:off + w.n_q_heads * (b - a)].view(1, w.n_q_heads, b - a)
            off += w.n_q_heads * (b - a)
            segs.append((a, b, lse))

        def timed(kind_, i, fn):
            if not record:
                fn()
                return
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(); fn(); e1.record()
            self.events.append((kind_, i, e0, e1))

        for i, (a, b, lse) in enumerate(segs):
            timed("fwd", i, lambda: s1f.seg_attn_fwd_ws(self.q[:, :, a:b], self.k, self.v, a, self.out[:, :, a:b], lse,
                                                         self.fwd_ws))
        self.dk.zero_(); self.dv.zero_()
        for i in reversed(range(len(segs))):
            a, b, lse = segs[i]
            qs, dos = self.q[:, :, a:b], self.dout[:, :, a:b]
            timed("bwd_dq", i, lambda: s1f.seg_attn_bwd_dq(dos, qs, self.k, self.v, self.out[:, :, a:b], lse, a,
                                                            self.dq[:, :, a:b], self.ws))
            timed("bwd_dkdv", i, lambda: s1f.seg_attn_bwd_dkdv(dos, qs, self.k, self.v, lse, a, self.dk, self.dv,
                                                                self.ws))
        return bounds

    def run(self, steps, warmup, **kw):
        torch = self.torch
        for _ in range(warmup):
            self.step(**kw)
        torch.cuda.synchronize()
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
        t0 = time.perf_counter()
        marks[0].record()
        for i in range(steps):
            self.step(record=True, **kw)
            marks[i + 1].record()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / steps
        self.step_ms = [marks[i].elapsed_time(marks[i + 1]) for i in range(steps)]
        return ms


def cache_kernels_report(stage, w, torch, s1f, bounds):
    """The data movements around the attention calls (K/V append before each forward, final dK/dV rows emitted
    after each backward), timed outside the step: HBM-bound, reported against the 8 TB/s peak."""
    e = 2 if w.dtype == "bf16" else 4
    kc, vc = torch.empty_like(stage.k), torch.empty_like(stage.v)
    dko, dvo = torch.empty_like(stage.k), torch.empty_like(stage.v)
    segs = list(zip(bounds[:-1], bounds[1:]))

    def timed(fn, reps=5):
        fn(); torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record(); torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    t_app = timed(lambda: [s1f.kv_append(stage.k[:, :, a:b], stage.v[:, :, a:b], a, kc, vc) for a, b in segs])
    t_emit = timed(lambda: [s1f.kv_grad_emit(stage.dk, stage.dv, a, dko[:, :, a:b], dvo[:, :, a:b]) for a, b in segs])
    elems = 2.0 * w.seq_len * w.n_kv_heads * w.head_dim          # K and V
    return {"kv_append": {"ms_per_sequence": t_app, "GB_per_s": elems * 2 * e / (t_app * 1e-3) / 1e9},
            "kv_grad_emit": {"ms_per_sequence": t_emit, "GB_per_s": elems * (4 + e) / (t_emit * 1e-3) / 1e9},
            "bound": "hbm", "peak_GB_per_s": 8000.0, "launches_per_sequence": len(segs)}


PP_SIZE, N_MICRO = 4, 16


def balance_report(stage, w, seg_ms, bounds, kernels, args):
    """Load balance of the partition (Section 3.4): max/mean over segments of attention time (measured,
    forward + backward of the segment) plus linear-layer time.  The linear layers are not built here: their
    time is MODELLED as 3 * 24 * hidden^2 * n_i FLOPs (forward + backward of one layer's matrices) at the
    TFLOP/s this run achieved on attention.  The uniform partition is measured the same way for comparison."""
    def ratio(bnds, per_seg_ms):
        att = [sum(per_seg_ms[k][i] for k in per_seg_ms) for i in range(len(bnds) - 1)]
        tot_att_flops = 14.0 * w.head_dim * w.n_q_heads * (w.seq_len * (w.seq_len + 1) // 2)
        rate = tot_att_flops / (sum(att) * 1e-3)                       # FLOP/s achieved on attention
        lin = [72.0 * w.hidden ** 2 * (b - a) / rate * 1e3 for a, b in zip(bnds[:-1], bnds[1:])]
        both = [x + y for x, y in zip(att, lin)]
        # what the imbalance costs a pipeline: bubble ratio of the sequence-level schedule on PP_SIZE devices with
        # N_MICRO micro-batches (the paper's 7B setting, Table 1), every stage taking these per-segment times
        t_f = [int(1e6 * (per_seg_ms["fwd"][i] + lin[i] / 3)) for i in range(len(att))]
        t_b = [int(1e6 * (per_seg_ms["bwd_dq"][i] + per_seg_ms["bwd_dkdv"][i] + 2 * lin[i] / 3)) for i in range(len(att))]
        sim = stage.s1f.pipeline_simulate(PP_SIZE, N_MICRO, len(att), 1, t_f, t_b)
        ideal = (PP_SIZE - 1) / (N_MICRO * len(att) + PP_SIZE - 1)     # equal segments
        return {"attention_only_max_over_mean": max(att) / (sum(att) / len(att)),
                "pipeline_bubble_ratio": sim["bubble_ratio"], "pipeline_bubble_ratio_equal_segments": ideal,
                "with_modelled_linear_max_over_mean": max(both) / (sum(both) / len(both)),
                "attention_total_ms": sum(att), "attention_ms": att, "modelled_linear_ms": lin}
    rep = {"partition": w.partition, "this": ratio(bounds, seg_ms), "linear_term": "modelled, not measured"}
    if w.partition != "cwp":
        return rep
    steps = 2

    def measure(kind):
        stage.events = []
        stage.run(steps, 1, kind=kind)
        b = stage.boundaries(kind=kind)
        seg = {}
        for knd, i, e0, e1 in stage.events:
            seg.setdefault(knd, [0.0] * (len(b) - 1))[i] += e0.elapsed_time(e1) / steps
        r = ratio(b, seg)
        r["boundaries"] = b
        return r
    rep["uniform"] = measure("uniform")
    rep["cwp_literal"] = measure("cwp_literal")
    rep["cwp_aligned128"] = measure("cwp_aligned128")
    # boundaries re-balanced twice on the measured time of each segment (attention measured + linear modelled)
    cur = dict(rep["this"], boundaries=list(bounds))
    for _ in range(2):
        cost_ns = [int(1e6 * (x + y)) for x, y in zip(cur["attention_ms"], cur["modelled_linear_ms"])]
        cur = measure(stage.s1f.partition_rebalance(cur["boundaries"], cost_ns, 1))
    rep["cwp_rebalanced_on_measured_time"] = cur
    return rep


def graph_report(stage, torch, flops, steps):
    """The same step recorded once as a HIP graph and replayed `steps` times: what the launches cost on top of the
    kernels (it matters for the small workloads, whose step is 24 launches of ~0.1 ms)."""
    stage.step()                      # warm: every kernel has run once outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        stage.step()
    graph.replay()
    torch.cuda.synchronize()
    steps = min(steps, 5)
    t0 = time.perf_counter()
    for _ in range(steps):
        graph.replay()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    return {"ms_per_step": ms, "tflops": flops / (ms * 1e-3) / 1e12, "replays": steps}


def cpu_baseline(stage, torch):
    """The row oracle, as it stands, timed on this machine's host cores on a bounded sample of the workload: one K/V
    group (its query heads share one K/V head, as in the workload) over the first `ns` tokens, full causal
    forward + backward, `ns` chosen for about 5e8 (query, key) pairs in all."""
    from oracle import rows
    w = stage.w
    grp = w.n_q_heads // w.n_kv_heads
    ns = min(w.seq_len, int(math.sqrt(2 * 5.4e8 / grp)))
    pairs = ns * (ns + 1) // 2
    rows.build()
    q = stage.q[0, :grp, :ns].float().cpu().numpy()
    do = stage.dout[0, :grp, :ns].float().cpu().numpy()
    k = stage.k[0, :1, :ns].float().cpu().numpy()
    v = stage.v[0, :1, :ns].float().cpu().numpy()
    t0 = time.perf_counter()
    for h in range(grp):
        rows.forward_rows(q, k, v, h, 0, ns)
        rows.dq_rows(q, k, v, do, h, 0, ns)
    rows.dkdv_keys(q, k, v, do, 0, 0, ns)
    dt = time.perf_counter() - t0
    flops = 14.0 * w.head_dim * pairs * grp
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": rows.threads(), "kind": "oracle",
            "sample": f"fp64 row oracle, one K/V group ({grp} query head(s) on 1 K/V head), first {ns} tokens of the "
                      f"{w.name} workload, full causal forward+backward ({dt:.1f} s)", "seconds": dt}


def measure_workload(w, torch, s1f, steps, warmup, constant_data=False):
    """Runs `steps` timed steps of workload w.  Returns (stage, result dict with the headline fields)."""
    stage = Stage(w, torch, s1f, constant_data)
    ms = stage.run(steps, warmup)
    bounds = stage.boundaries()
    pairs = seg_pairs(bounds)
    d, hq = w.head_dim, w.n_q_heads
    tot_pairs = sum(pairs)
    assert tot_pairs == w.seq_len * (w.seq_len + 1) // 2
    flops = 14.0 * d * hq * tot_pairs
    peak = PEAK_BF16_TFLOPS if w.dtype == "bf16" else PEAK_F32_TFLOPS
    # per-kernel durations from the events recorded inside the timed steps
    per = {"fwd": [0.0, 0, 4.0], "bwd_dq": [0.0, 0, 2.0], "bwd_dkdv": [0.0, 0, 8.0]}   # ms, launches, flops/(pair*D)
    seg_ms = {}
    for kind, i, e0, e1 in stage.events:
        t = e0.elapsed_time(e1)
        per[kind][0] += t; per[kind][1] += 1
        seg_ms.setdefault(kind, [0.0] * len(pairs))[i] += t / steps
    kernels = {}
    for kind, (t, cnt, fpp) in per.items():
        alg = fpp * d * hq * tot_pairs * steps          # algorithmic flops over all timed launches
        kernels[kind] = {"avg_launch_ms": t / cnt, "launches_per_step": cnt // steps,
                         "alg_tflops": alg / (t * 1e-3) / 1e12, "ms_per_step": t / steps}
    # executed rate of the dQ kernel: it runs three products (S, dP, dQ) where one is credited
    kernels["bwd_dq"]["executed_tflops"] = 3.0 * kernels["bwd_dq"]["alg_tflops"]
    sm = stage.step_ms
    mean = sum(sm) / len(sm)
    res = {"value": flops / (ms * 1e-3) / 1e12, "ms_per_step": ms, "pct_of_peak": 100.0 * flops / (ms * 1e-3) / 1e12 / peak,
           "config": {"workload": w.name, "seq_len": w.seq_len, "n_seg": w.n_seg, "partition": w.partition,
                      "n_q_heads": hq, "n_kv_heads": w.n_kv_heads, "head_dim": d, "boundaries": bounds},
           "fwd_tflops": 4.0 * d * hq * tot_pairs / (kernels["fwd"]["ms_per_step"] * 1e-3) / 1e12,
           "bwd_tflops": 10.0 * d * hq * tot_pairs /
                         ((kernels["bwd_dq"]["ms_per_step"] + kernels["bwd_dkdv"]["ms_per_step"]) * 1e-3) / 1e12,
           "kernels": kernels, "segment_ms": seg_ms, "step_ms_mean": mean,
           "step_ms_std": (sum((x - mean) ** 2 for x in sm) / max(1, len(sm) - 1)) ** 0.5}
    return stage, res, flops, peak


def unsegmented_report(stage, ms, steps):
    """One unsegmented pass (a single segment at offset 0) over the same sequence, and what segmentation costs."""
    stage.events = []
    ms1 = stage.run(steps, 1, n_seg=1, kind="uniform")
    per_kernel = {}
    for kind, _, e0, e1 in stage.events:
        per_kernel[kind] = per_kernel.get(kind, 0.0) + e0.elapsed_time(e1) / steps
    return {"unsegmented_ms": ms1, "segmentation_overhead": ms / ms1 - 1.0, "unsegmented_kernels_ms": per_kernel}


def atomics_probe(torch):
    """TB/s of fp32 global atomic adds (and of plain stores of the same shape) when every wave adds 32 rows x 32
    floats per step into a [rows, 128] fp32 array shared by the workgroups of a head, heads spread over the XCDs the
    way the kernels spread them: the traffic a dK/dV kernel that also produced dQ would put on the L2."""
    import ctypes
    lib = ctypes.CDLL(os.path.join(ROOT, "paper_2406_03488_amd", "libs1f_probe.so"))
    lib.s1f_probe_dq_atomics.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                         ctypes.c_void_p, ctypes.c_void_p]
    lib.s1f_probe_dq_atomics.restype = ctypes.c_int
    rows, heads, steps, wgs = 4096, 32, 128, 2048
    acc = torch.zeros(heads * rows * 128, dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    out = {}
    for mode, name in ((0, "atomic_add_f32_TB_per_s"), (1, "plain_store_TB_per_s")):
        best = 0.0
        for rep in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            if lib.s1f_probe_dq_atomics(wgs, rows, heads, steps, mode, acc.data_ptr(), stream) != 0:
                raise RuntimeError("atomics probe failed to launch")
            e1.record()
            torch.cuda.synchronize()
            best = max(best, wgs * 4 * steps * 16 * 64 * 4.0 / (e0.elapsed_time(e1) * 1e-3) / 1e12)
        out[name] = best
    out["shape"] = f"{wgs} workgroups x 4 waves x {steps} steps x 16 instructions of 64 lanes x 4 bytes"
    return out


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU: the path has no collectives and this build runs on a single MI355X; "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)
    import torch
    import s1f_synth as S
    import paper_2406_03488_amd as s1f
    s1f.load_library()            # fails loudly if the HIP library is missing; there is no fallback
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    w = S.WORKLOADS[args.workload]
    if args.calibrate_copy:   # a plain copy of known size: 1 GiB read + 1 GiB written
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").fill_(1.0)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    stage, res, flops, peak = measure_workload(w, torch, s1f, args.steps, args.warmup, args.constant_data)
    ms, bounds, kernels, seg_ms = res["ms_per_step"], res["config"]["boundaries"], res["kernels"], res["segment_ms"]

    dom = max(kernels, key=lambda kk: kernels[kk]["ms_per_step"])
    roofline = {"bound": "mfma", "kernel": KERNEL_NAMES[dom],
                "achieved": kernels[dom]["alg_tflops"], "peak": peak, "unit": "TFLOP/s",
                "frac": kernels[dom]["alg_tflops"] / peak, "traffic": measured_traffic(KERNEL_NAMES[dom], w.name),
                "traffic_unit": "bytes per launch", "avg_launch_ms": kernels[dom]["avg_launch_ms"]}
    result = {
        "metric": "segmented causal attn fwd+bwd TFLOP/s on 1 GPU; % of bf16 MFMA peak",
        "value": res["value"], "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": w.dtype, "data": "synthetic, constant" if args.constant_data else "synthetic",
        "config": res["config"], "pct_of_peak": res["pct_of_peak"], "fwd_tflops": res["fwd_tflops"],
        "bwd_tflops": res["bwd_tflops"], "kernels": kernels, "segment_ms": seg_ms, "roofline": roofline,
        "step_ms_mean": res["step_ms_mean"], "step_ms_std": res["step_ms_std"],
    }
    for kind in kernels:
        kernels[kind]["traffic_bytes_per_launch"] = measured_traffic(KERNEL_NAMES[kind], w.name)
    if not args.no_mfma_probe and w.dtype == "bf16":
        mp, mp_varied = measured_mfma_peak(torch)
        result["measured_mfma_peak_tflops"] = mp
        result["measured_mfma_peak_varied_data_tflops"] = mp_varied
        result["pct_of_measured_peak"] = 100.0 * result["value"] / mp
        result["pct_of_measured_peak_varied_data"] = 100.0 * result["value"] / mp_varied
        roofline["frac_of_measured_peak"] = roofline["achieved"] / mp
        roofline["frac_of_measured_peak_varied_data"] = roofline["achieved"] / mp_varied
    if args.probe_atomics:
        result["dq_atomics_probe"] = atomics_probe(torch)
    result["cache_kernels"] = cache_kernels_report(stage, w, torch, s1f, bounds)
    if not args.no_balance:
        result["balance"] = balance_report(stage, w, seg_ms, bounds, kernels, args)
    if not args.no_unsegmented:
        result.update(unsegmented_report(stage, ms, 2))
    if not args.no_graph:
        result["hip_graph"] = graph_report(stage, torch, flops, args.steps)
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(stage, torch)
    del stage
    torch.cuda.empty_cache()
    # the other workloads of the target range, briefly: same step, same kernels
    others = {}
    for name in [x for x in args.others.split(",") if x and x != w.name]:
        short = S.WORKLOADS[name].seq_len < 32768      # a step of a few milliseconds: more of them
        st2, r2, _, _ = measure_workload(S.WORKLOADS[name], torch, s1f, 20 if short else 3, 3 if short else 1,
                                         args.constant_data)
        if not args.no_unsegmented:
            r2.update(unsegmented_report(st2, r2["ms_per_step"], 2))
        r2["kernels"] = {k: {"alg_tflops": v["alg_tflops"], "ms_per_step": v["ms_per_step"],
                             "avg_launch_ms": v["avg_launch_ms"]} for k, v in r2["kernels"].items()}
        r2["config"] = {k: v for k, v in r2["config"].items() if k != "boundaries"}
        del r2["segment_ms"]
        others[name] = r2
        del st2
        torch.cuda.empty_cache()
    if others:
        result["other_workloads"] = others
    print(json.dumps(result))


if __name__ == "__main__":
    main()
