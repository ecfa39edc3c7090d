"""GPU parity beyond one sequence and beyond hand-picked boundaries: several independent sequences in one set
of calls (batch > 1), launches that take the XCD-aware workgroup order in both of its variants, prefix
accumulation over many launches compared element by element, and a seeded random sweep over offsets,
lengths, head dimensions, head groupings and layouts.  Tolerances are the contract's (see test_gpu_parity)."""
import numpy as np
import pytest

import s1f_synth as S
from oracle import attention as A

pytestmark = pytest.mark.gpu

F32_MAXABS = 1e-4
BF16_MAXABS, BF16_RELFRO = 2e-2, 1e-2
LSE_MAXABS_BF16 = 1e-3


def _check(res, want, dtype, where=""):
    from gpu_harness import errors
    for name in ("out", "lse", "dq", "dk", "dv"):
        assert np.isfinite(res[name]).all(), f"{where}{name} has non-finite values"
        mx, fro = errors(res[name], want[name])
        if dtype == "f32":
            assert mx <= F32_MAXABS, f"{where}{name}: max abs {mx}"
        elif name == "lse":
            assert mx <= LSE_MAXABS_BF16, f"{where}lse: max abs {mx}"
        else:
            assert mx <= BF16_MAXABS and fro <= BF16_RELFRO, f"{where}{name}: max abs {mx} rel fro {fro}"


def _sequence(seed, hq, hkv, n, d, dtype):
    return (S.tensor(seed, "q", hq, n, d, dtype), S.tensor(seed, "k", hkv, n, d, dtype),
            S.tensor(seed, "v", hkv, n, d, dtype), S.tensor(seed, "dout", hq, n, d, dtype))


def _oracle(q, k, v, do):
    out, lse = A.full_forward(q, k, v)
    dq, dk, dv = A.full_backward(do, q, k, v)
    return {"out": out, "lse": lse, "dq": dq, "dk": dk, "dv": dv}


# A short first segment (workgroups ordered tile by tile inside an XCD) followed by segments behind a prefix longer
# than themselves (ordered head by head), with unaligned boundaries and a ragged tail.
BOUNDS = [0, 300, 500, 1100, 1357]


@pytest.mark.parametrize("dtype,d,layout", [("bf16", 128, "bhsd"), ("bf16", 80, "bshd"), ("f32", 64, "bshd"),
                                            ("f32", 128, "bhsd")])
@pytest.mark.parametrize("nb,hq,hkv", [(3, 8, 2), (2, 4, 4)])
def test_several_sequences_in_one_call(dtype, d, layout, nb, hq, hkv):
    """Every batch entry is a sequence of its own (distinct data) and must equal full causal attention on it.
    3 x 8 query heads give 24 (batch, head) pairs: the forward and dQ kernels take the XCD-aware order; 2 x 4
    K/V heads do the same for the dK/dV kernel.  The K/V rows travel through s1f_kv_append and the final
    gradient rows through s1f_kv_grad_emit."""
    from gpu_harness import run_schedule_batched
    n = BOUNDS[-1]
    seqs = [_sequence(300 + 17 * b + d, hq, hkv, n, d, dtype) for b in range(nb)]
    q, k, v, do = (np.stack([s[i] for s in seqs]) for i in range(4))
    fin = []
    res = run_schedule_batched(q, k, v, do, BOUNDS, dtype, capacity=n + 40, layout=layout, finality=fin,
                               cache_kernels=True)
    assert (res["dk"][:, :, n:] == 777.0).all() and (res["dv"][:, :, n:] == 777.0).all()
    assert np.array_equal(res["k_cache"][:, :, :n], k) and np.array_equal(res["v_cache"][:, :, :n], v)
    from gpu_harness import errors
    for b in range(nb):
        want = _oracle(*seqs[b])
        got = {name: res[name][b][:, :n] if name in ("dk", "dv") else res[name][b] for name in want}
        _check(got, want, dtype, where=f"batch entry {b}: ")
        # rows emitted right after each segment's backward pass are already the gradient of the whole sequence
        # (Section 3.1's order constraint), rounded once more to the element type in bf16 mode
        for name in ("dk", "dv"):
            mx, fro = errors(res[name + "_emit"][b], want[name])
            if dtype == "f32":
                assert mx <= F32_MAXABS, (name, b, mx)
            else:
                assert mx <= BF16_MAXABS + 2.0 ** -8 * np.abs(want[name]).max() and fro <= BF16_RELFRO, (name, b, mx, fro)
    assert len(fin) == len(BOUNDS) - 1


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_eight_heads_both_workgroup_orders(dtype):
    """One sequence, 8 query heads on 8 K/V heads: all three kernels take the XCD-aware order, tile-major for the
    first segment and head-major behind the long prefix; compared element by element."""
    from gpu_harness import run_schedule
    q, k, v, do = _sequence(911, 8, 8, BOUNDS[-1], 128, dtype)
    _check(run_schedule(q, k, v, do, BOUNDS, dtype), _oracle(q, k, v, do), dtype)


@pytest.mark.parametrize("n_seg,hq,hkv,hidden", [(32, 64, 8, 8192), (16, 56, 56, 7168)])
def test_prefix_accumulation_over_every_launch(n_seg, hq, hkv, hidden):
    """16384 tokens in 32 (16) equal-cost segments with the head structure of the two largest workloads, driven by
    the same Stage object the benchmark times.  The keys of the FIRST segment receive a += from every one of the 32
    (16) backward launches; their dK/dV are compared element by element with the row oracle, as are keys at later
    boundaries and the outputs and dQ of rows spread over the sequence."""
    import torch
    import bench
    import paper_2406_03488_amd as s1f
    from gpu_harness import errors
    from oracle import rows

    n, d = 16384, 128
    w = S.Workload(f"acc{n_seg}", n, n_seg, hq, hkv, d, hidden, "bf16", "cwp", 20240700 + n_seg)
    stage = bench.Stage(w, torch, s1f)
    bounds = stage.step()
    torch.cuda.synchronize()
    assert len(bounds) == n_seg + 1
    grp = hq // hkv
    g = hkv - 3
    heads = list(range(g * grp, (g + 1) * grp))
    q = stage.q[0, heads].float().cpu().numpy(); do = stage.dout[0, heads].float().cpu().numpy()
    k = stage.k[0, g:g + 1].float().cpu().numpy(); v = stage.v[0, g:g + 1].float().cpu().numpy()
    key_sets = [(0, 24), (bounds[1] - 12, bounds[1] + 12), (bounds[n_seg // 2] - 8, bounds[n_seg // 2] + 8), (n - 24, n)]
    for j0, j1 in key_sets:
        print(f"  keys {j0}..{j1} of kv head {g}", flush=True)
        dk_ref, dv_ref = rows.dkdv_keys(q, k, v, do, 0, j0, j1)
        for name, got, ref in (("dk", stage.dk, dk_ref), ("dv", stage.dv, dv_ref)):
            mx, fro = errors(got[0, g, j0:j1].cpu().numpy(), ref)
            assert mx <= BF16_MAXABS and fro <= BF16_RELFRO, (name, j0, mx, fro)
    hl = grp - 1
    for r0, r1 in [(0, 16), (bounds[1] - 8, bounds[1] + 8), (bounds[-2] - 8, bounds[-2] + 8), (n - 16, n)]:
        o_ref, _ = rows.forward_rows(q, k, v, hl, r0, r1)
        dq_ref = rows.dq_rows(q, k, v, do, hl, r0, r1)
        for name, got, ref in (("out", stage.out, o_ref), ("dq", stage.dq, dq_ref)):
            mx, fro = errors(got[0, heads[hl], r0:r1].float().cpu().numpy(), ref)
            assert mx <= BF16_MAXABS and fro <= BF16_RELFRO, (name, r0, mx, fro)


def _sweep_cases(count, seed):
    """(seg_off, seg_len, head_dim, Hq, Hkv, dtype, layout): lengths of one to three row tiles (128 rows) plus or
    minus a token and a few tiny ones, offsets from 0 to a few key tiles (aligned and not)."""
    rng = np.random.Generator(np.random.Philox(seed))
    lens = [1, 2, 31, 33, 127, 128, 129, 255, 256, 257, 383, 384, 385]
    offs = [0, 0, 1, 31, 32, 63, 64, 65, 127, 128, 255, 256, 257, 300, 511, 512, 640, 777]
    groups = [(1, 1), (2, 1), (2, 2), (4, 2), (3, 3), (8, 2), (6, 1)]
    cases = []
    for _ in range(count):
        hq, hkv = groups[rng.integers(len(groups))]
        cases.append((int(offs[rng.integers(len(offs))]), int(lens[rng.integers(len(lens))]),
                      int((64, 80, 128)[rng.integers(3)]), hq, hkv, ("f32", "bf16")[rng.integers(2)],
                      ("bhsd", "bshd")[rng.integers(2)]))
    return cases


def test_random_sweep_single_segment_calls():
    """64 seeded random single-segment calls (forward + backward at an arbitrary offset) against the oracle's
    segment-wise definition; stops at the first failure and names the case."""
    from gpu_harness import run_segment
    for idx, (off, m, d, hq, hkv, dtype, layout) in enumerate(_sweep_cases(64, 20240611)):
        case = f"case {idx}: seg_off={off} seg_len={m} D={d} heads={hq}/{hkv} {dtype} {layout}: "
        print(case, flush=True)
        n = off + m
        q, k, v, do = _sequence(5000 + idx, hq, hkv, n, d, dtype)
        res = run_segment(q[:, off:], k, v, do[:, off:], off, dtype, layout)
        out, lse = A.segment_forward(q[:, off:], k, v, off)
        dq, dk, dv = A.segment_backward(do[:, off:], q[:, off:], k, v, off)
        _check(res, {"out": out, "lse": lse, "dq": dq, "dk": dk, "dv": dv}, dtype, where=case)


@pytest.mark.parametrize("d", [64, 80, 128])
@pytest.mark.parametrize("hq,hkv,off,m", [(2, 1, 2100, 333), (4, 4, 1800, 140), (3, 1, 4500, 129), (8, 2, 1290, 256),
                                          (2, 2, 3000, 1)])
def test_key_split_row_tiles_match_oracle(d, hq, hkv, off, m):
    """Few row tiles behind a long prefix: the library cuts every one of them into chunks along the keys (forward
    through its workspace entry point, dQ through the backward's workspace) and merges the partial results; the
    result must still equal the oracle, and the forward must agree with the entry point that never splits."""
    import torch
    import paper_2406_03488_amd as s1f
    from gpu_harness import errors, run_segment, to_device
    n = off + m
    q, k, v, do = _sequence(7000 + d + off, hq, hkv, n, d, "bf16")
    kd = to_device(k, "bf16")[None]
    qd = to_device(q[:, off:], "bf16")[None].contiguous()
    assert s1f.fwd_workspace_bytes(qd, kd, off) > 0, "this shape is meant to be split"
    assert s1f.bwd_workspace_bytes(qd, kd, off) > 2 * 4 * hq * m + 256, "this shape is meant to be split"
    res = run_segment(q[:, off:], k, v, do[:, off:], off, "bf16")
    out, lse = A.segment_forward(q[:, off:], k, v, off)
    dq, dk, dv = A.segment_backward(do[:, off:], q[:, off:], k, v, off)
    _check(res, {"out": out, "lse": lse, "dq": dq, "dk": dk, "dv": dv}, "bf16")
    plain = run_segment(q[:, off:], k, v, do[:, off:], off, "bf16", fwd_workspace=False)
    assert errors(res["out"], plain["out"])[0] <= 2.0 ** -7 * np.abs(plain["out"]).max()   # one bf16 rounding apart
    assert errors(res["lse"], plain["lse"])[0] <= 1e-5


def _rising(seed, hq, hkv, n, d, dtype, levels=4):
    """Inputs whose scores climb along the sequence: key j carries a_j * u (a_j rising from 0 to 2 in `levels` steps,
    u a fixed vector of +-1) and query r carries c_r * u with c_r in [-2, 2], both on top of 0.6 * N(0, 1)
    noise.  Row r's scaled scores step up by 2 c_r * sqrt(d) / (levels - 1) from level to level (tens of nats for the
    rows with large c_r, far beyond what N(0, 1) operands ever produce), and fall as steeply for the rows with c_r < 0."""
    q, k, v, do = _sequence(seed, hq, hkv, n, d, dtype)
    u = np.where(S.head_tensor(seed + 1, "q", 0, 1, d, "f32")[0] >= 0, 1.0, -1.0).astype(np.float32)
    a = 2.0 * (np.arange(n) * levels // n).astype(np.float32) / (levels - 1)
    c = np.clip(S.tensor(seed + 2, "q", hq, n, 1, "f32")[..., 0] * 1.5, -2.0, 2.0)
    k = 0.6 * k + a[None, :, None] * u
    q = 0.6 * q + c[:, :, None] * u
    if dtype == "bf16":
        q, k = S.round_to_bf16(q), S.round_to_bf16(k)
    return q.astype(np.float32), k.astype(np.float32), v, do


@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("bf16", 64), ("bf16", 80), ("f32", 128)])
def test_rising_scores_raise_the_running_maximum(dtype, d):
    """The forward keeps a running row maximum and rescales its accumulators when a later block of keys exceeds it
    by a wide margin; N(0, 1) operands never make it do so.  Here the scores of many rows climb by tens of nats along
    the keys (and fall as far for others, whose late probabilities underflow to zero), through several segments and
    through a launch whose row tiles are cut along the keys, where the chunks of one row differ as much in their
    maxima."""
    from gpu_harness import run_schedule, run_segment
    hq, hkv, n = 4, 2, BOUNDS[-1]
    q, k, v, do = _rising(910 + d, hq, hkv, n, d, dtype)
    scores = np.einsum("hrd,hjd->hrj", q.astype(np.float64), np.repeat(k, hq // hkv, axis=0)) / np.sqrt(d)
    rows = range(n // 2, n)
    climb = np.array([[scores[h, r, 32:r + 1].max() - scores[h, r, :32].max() for r in rows] for h in range(hq)])
    fall = np.array([[scores[h, r, r - 31:r + 1].max() - scores[h, r, :32].max() for r in rows] for h in range(hq)])
    assert (climb > 10.0).mean() > 0.15 and (fall < -10.0).mean() > 0.15   # the data does what the test is about
    res = run_schedule(q, k, v, do, BOUNDS, dtype)
    _check(res, _oracle(q, k, v, do), dtype, where="schedule: ")
    if dtype == "bf16":   # few row tiles behind a long prefix: forward and dQ launches are split along the keys
        off, m = 2100, 333
        q, k, v, do = _rising(920 + d, 2, 1, off + m, d, dtype)
        res = run_segment(q[:, off:], k, v, do[:, off:], off, dtype)
        out, lse = A.segment_forward(q[:, off:], k, v, off)
        dq, dk, dv = A.segment_backward(do[:, off:], q[:, off:], k, v, off)
        _check(res, {"out": out, "lse": lse, "dq": dq, "dk": dk, "dv": dv}, dtype, where="key-split: ")


def test_results_do_not_depend_on_the_run():
    """No kernel uses atomics and every accumulator element has one owner, so the same call on the same data must give
    the same bits every time, key-split launches included (their merge adds the chunks in a fixed order)."""
    from gpu_harness import run_segment
    hq, hkv, off, m, d = 8, 2, 2300, 300, 128
    q, k, v, do = _sequence(4242, hq, hkv, off + m, d, "bf16")
    runs = [run_segment(q[:, off:], k, v, do[:, off:], off, "bf16") for _ in range(3)]
    for other in runs[1:]:
        for name in ("out", "lse", "dq", "dk", "dv"):
            assert np.array_equal(runs[0][name], other[name]), name
