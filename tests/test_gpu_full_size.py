"""GPU parity at the contract's full sizes, in the launch configuration bench.py times (same Stage
object, same entry points): outputs the row oracle can compute one by one are compared on sampled rows
and keys, and invariants that hold at any size are checked on all heads."""
import os
import sys

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BF16_MAXABS, BF16_RELFRO = 2e-2, 1e-2


def _errors(got, want):
    diff = np.asarray(got, np.float64) - np.asarray(want, np.float64)
    return float(np.abs(diff).max()), float(np.linalg.norm(diff) / max(np.linalg.norm(want), 1e-300))


@pytest.mark.parametrize("name,second_keys", [("2.7b", "first-boundary"), ("7b", "first-boundary"),
                                              ("30b", "last-boundary"), ("30b-uniform", "last-boundary"),
                                              ("gqa", "late")])
def test_full_size_workload_sampled_against_row_oracle(name, second_keys):
    import torch
    import bench
    import s1f_synth as S
    import paper_2406_03488_amd as s1f
    from oracle import rows

    w = S.WORKLOADS[name]
    print(f"workload {name}: n={w.seq_len} segs={w.n_seg} heads={w.n_q_heads}/{w.n_kv_heads} d={w.head_dim}", flush=True)
    stage = bench.Stage(w, torch, s1f)
    bounds = stage.step()
    torch.cuda.synchronize()
    n, d, grp = w.seq_len, w.head_dim, w.n_q_heads // w.n_kv_heads

    # ---- invariants on every head (any size) ----
    for t in (stage.out, stage.dq, stage.dk, stage.dv):
        assert torch.isfinite(t).all()
    # dV columns: every dO row is distributed in full over the values it saw
    do_sum = stage.dout.float().view(1, w.n_kv_heads, grp, n, d).sum(dim=(2, 3)).double().cpu().numpy()
    dv_sum = stage.dv.double().sum(dim=2).cpu().numpy()
    assert _errors(dv_sum, do_sum)[1] <= BF16_RELFRO
    # dK sums to zero over keys (shift invariance of the softmax), relative to the size of its terms
    dk_sum = stage.dk.double().sum(dim=2).abs().max().item()
    dk_abs = stage.dk.double().abs().sum(dim=2).max().item()
    assert dk_sum <= 1e-2 * dk_abs
    # out rows are convex combinations of the values they saw: bounded by the running extremes of v
    h_chk = w.n_q_heads - 1
    vmax = torch.cummax(stage.v[0, h_chk // grp].float(), dim=0).values
    vmin = torch.cummin(stage.v[0, h_chk // grp].float(), dim=0).values
    o = stage.out[0, h_chk].float()
    assert (o <= vmax + 2e-2).all() and (o >= vmin - 2e-2).all()

    # ---- sampled rows / keys against the fp64 row oracle ----
    h = w.n_q_heads - 1 if name != "7b" else 17
    g = h // grp
    heads = list(range(g * grp, (g + 1) * grp))
    q = stage.q[0, heads].float().cpu().numpy(); do = stage.dout[0, heads].float().cpu().numpy()
    k = stage.k[0, g:g + 1].float().cpu().numpy(); v = stage.v[0, g:g + 1].float().cpu().numpy()
    hl = h - g * grp     # index of head h inside the extracted group
    # rows straddling segment boundaries and tile edges, plus the first and last rows
    row_sets = [(0, 40), (bounds[1] - 20, bounds[1] + 20), (bounds[-2] - 20, bounds[-2] + 20), (n - 40, n)]
    mid = bounds[len(bounds) // 2]
    row_sets.append((mid + 250, mid + 290))
    for r0, r1 in row_sets:
        print(f"  rows {r0}..{r1} of head {h}", flush=True)
        o_ref, lse_ref = rows.forward_rows(q, k, v, hl, r0, r1)
        dq_ref = rows.dq_rows(q, k, v, do, hl, r0, r1)
        mx, fro = _errors(stage.out[0, h, r0:r1].float().cpu().numpy(), o_ref)
        assert mx <= BF16_MAXABS and fro <= BF16_RELFRO, ("out", r0, mx, fro)
        mx, fro = _errors(stage.dq[0, h, r0:r1].float().cpu().numpy(), dq_ref)
        assert mx <= BF16_MAXABS and fro <= BF16_RELFRO, ("dq", r0, mx, fro)
    # lse of the last rows (saved per segment, segment-major in the flat buffer)
    a, b = bounds[-2], bounds[-1]
    lse_last = stage.lse_flat[w.n_q_heads * a:].view(w.n_q_heads, b - a)[h, -40:].cpu().numpy()
    _, lse_ref = rows.forward_rows(q, k, v, hl, n - 40, n)
    assert np.abs(lse_last - lse_ref).max() <= 1e-3
    # keys: the last keys (cheap for the oracle) and, where affordable, keys that receive gradient from
    # every segment (they need the oracle's forward of all later rows)
    key_sets = [(n - 48, n)]
    if second_keys == "first-boundary":     # gradient arrives from every segment
        key_sets.append((bounds[1] - 8, bounds[1] + 8))
    elif second_keys == "last-boundary":    # gradient arrives from the last two segments
        key_sets.append((bounds[-2] - 8, bounds[-2] + 8))
    else:                                   # the oracle's cost grows with (rows after the key) x heads in the group
        key_sets.append((n - 400, n - 384))
    for j0, j1 in key_sets:
        print(f"  keys {j0}..{j1} of kv head {g}", flush=True)
        dk_ref, dv_ref = rows.dkdv_keys(q, k, v, do, 0, j0, j1)
        mx, fro = _errors(stage.dk[0, g, j0:j1].cpu().numpy(), dk_ref)
        assert mx <= BF16_MAXABS and fro <= BF16_RELFRO, ("dk", j0, mx, fro)
        mx, fro = _errors(stage.dv[0, g, j0:j1].cpu().numpy(), dv_ref)
        assert mx <= BF16_MAXABS and fro <= BF16_RELFRO, ("dv", j0, mx, fro)


def test_one_long_launch_without_segments():
    """A single launch over a whole sequence that is many rounds of row tiles long (128 tiles x 56 heads): the
    forward and dQ kernels then order their workgroups head by head although the launch starts at offset 0.  Sampled
    rows and keys against the row oracle, invariants on every head."""
    import torch
    import bench
    import s1f_synth as S
    import paper_2406_03488_amd as s1f
    from oracle import rows

    w = S.Workload("one-pass", 16384, 1, 56, 56, 128, 7168, "bf16", "uniform", 20240611)
    stage = bench.Stage(w, torch, s1f)
    bounds = stage.step()
    torch.cuda.synchronize()
    assert bounds == [0, w.seq_len]
    n, d = w.seq_len, w.head_dim
    for t in (stage.out, stage.dq, stage.dk, stage.dv):
        assert torch.isfinite(t).all()
    do_sum = stage.dout.float().sum(dim=2).double().cpu().numpy()
    assert _errors(stage.dv.double().sum(dim=2).cpu().numpy(), do_sum)[1] <= BF16_RELFRO
    assert stage.dk.double().sum(dim=2).abs().max().item() <= 1e-2 * stage.dk.double().abs().sum(dim=2).max().item()
    for h in (0, 29, 55):
        q = stage.q[0, h:h + 1].float().cpu().numpy(); do = stage.dout[0, h:h + 1].float().cpu().numpy()
        k = stage.k[0, h:h + 1].float().cpu().numpy(); v = stage.v[0, h:h + 1].float().cpu().numpy()
        for r0, r1 in [(0, 24), (4090, 4110), (n - 24, n)]:
            print(f"  head {h} rows {r0}..{r1}", flush=True)
            o_ref, lse_ref = rows.forward_rows(q, k, v, 0, r0, r1)
            dq_ref = rows.dq_rows(q, k, v, do, 0, r0, r1)
            for name, got, ref in (("out", stage.out, o_ref), ("dq", stage.dq, dq_ref)):
                mx, fro = _errors(got[0, h, r0:r1].float().cpu().numpy(), ref)
                assert mx <= BF16_MAXABS and fro <= BF16_RELFRO, (name, h, r0, mx, fro)
            assert np.abs(stage.lse_flat.view(w.n_q_heads, n)[h, r0:r1].cpu().numpy() - lse_ref).max() <= 1e-3
        j0, j1 = n - 40, n
        dk_ref, dv_ref = rows.dkdv_keys(q, k, v, do, 0, j0, j1)
        for name, got, ref in (("dk", stage.dk, dk_ref), ("dv", stage.dv, dv_ref)):
            mx, fro = _errors(got[0, h, j0:j1].cpu().numpy(), ref)
            assert mx <= BF16_MAXABS and fro <= BF16_RELFRO, (name, h, mx, fro)
