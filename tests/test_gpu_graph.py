"""A whole step (K/V append, forward of every segment, backward in reverse order, gradient emit) recorded once into
a HIP graph and replayed (launches split along the keys and their merge kernels included): every replay must
reproduce the eager results bit for bit (the kernels use no atomics),
with eager work and synchronisations between the replays, and on fresh inputs written into the same buffers."""
import numpy as np
import pytest
import torch

import paper_2406_03488_amd as s1f
import s1f_synth as S
from gpu_harness import to_device

pytestmark = pytest.mark.gpu


def test_step_in_a_graph_matches_eager_on_every_replay():
    hq, hkv, n, d, dtype = 4, 2, 3300, 128, "bf16"
    bounds = s1f.partition(n, 3, 64, 4)
    segs = list(zip(bounds[:-1], bounds[1:]))

    def inputs(seed):
        return [to_device(S.tensor(seed, t, hh, n, d, dtype), dtype)[None]
                for t, hh in (("q", hq), ("k", hkv), ("v", hkv), ("dout", hq))]

    qd, kd, vd, dod = inputs(21)
    kc = torch.zeros((1, hkv, n, d), dtype=torch.bfloat16, device="cuda"); vc = torch.zeros_like(kc)
    out = torch.empty_like(qd); dq = torch.empty_like(qd)
    dk_acc = torch.zeros((1, hkv, n, d), dtype=torch.float32, device="cuda"); dv_acc = torch.zeros_like(dk_acc)
    dk_out = torch.empty_like(kc); dv_out = torch.empty_like(kc)
    lses = [torch.empty((1, hq, b - a), dtype=torch.float32, device="cuda") for a, b in segs]
    wss = [torch.empty(s1f.bwd_workspace_bytes(qd[:, :, a:b], kc, a), dtype=torch.uint8, device="cuda") for a, b in segs]
    fwd_bytes = [s1f.fwd_workspace_bytes(qd[:, :, a:b], kc, a) for a, b in segs]
    assert max(fwd_bytes) > 0, "a launch of this step is meant to be split along the keys (merge kernels in the graph)"
    fwss = [torch.empty(nb, dtype=torch.uint8, device="cuda") if nb else None for nb in fwd_bytes]

    def step():
        for (a, b), lse, fws in zip(segs, lses, fwss):
            s1f.kv_append(kd[:, :, a:b], vd[:, :, a:b], a, kc, vc)
            s1f.seg_attn_fwd_ws(qd[:, :, a:b], kc, vc, a, out[:, :, a:b], lse, fws)
        dk_acc.zero_(); dv_acc.zero_()          # a fill kernel, not a memset node
        for i in reversed(range(len(segs))):
            a, b = segs[i]
            s1f.seg_attn_bwd(dod[:, :, a:b], qd[:, :, a:b], kc, vc, out[:, :, a:b], lses[i], a, dq[:, :, a:b],
                             dk_acc, dv_acc, wss[i])
            s1f.kv_grad_emit(dk_acc, dv_acc, a, dk_out[:, :, a:b], dv_out[:, :, a:b])

    def results():
        torch.cuda.synchronize()
        return [t.clone() for t in (out, dq, dk_out, dv_out, dk_acc, dv_acc, *lses)]

    def scrub():
        for t in (out, dq, dk_out, dv_out):
            t.fill_(float("nan"))
        dk_acc.fill_(3.0); dv_acc.fill_(-3.0)
        for t in lses:
            t.fill_(float("nan"))

    step()
    eager = results()
    graph = torch.cuda.CUDAGraph()
    scrub()
    with torch.cuda.graph(graph):
        step()
    for replay in range(3):
        scrub()
        _ = (qd.float() @ qd.float().transpose(-1, -2)).sum().item()     # eager work and a synchronisation in between
        graph.replay()
        got = results()
        for g, e in zip(got, eager):
            assert torch.equal(g, e), f"replay {replay} differs from the eager run"
    # new inputs in the same buffers: the graph holds pointers, not data
    q2, k2, v2, do2 = inputs(22)
    qd.copy_(q2); kd.copy_(k2); vd.copy_(v2); dod.copy_(do2)
    scrub()
    step()
    eager2 = results()
    assert not torch.equal(eager2[0], eager[0])
    scrub()
    graph.replay()
    for g, e in zip(results(), eager2):
        assert torch.equal(g, e)
