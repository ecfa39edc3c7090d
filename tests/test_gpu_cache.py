"""K/V append and final-gradient emit on the GPU against the oracle: bit-exact data movement, and the
end-to-end use around the attention calls (rows of a segment are final after its backward pass)."""
import numpy as np
import pytest
import torch

import paper_2406_03488_amd as s1f
import s1f_synth as S
from gpu_harness import errors, to_device
from oracle import attention as A
from oracle import cache as C

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("d", [64, 80, 128])
def test_append_and_emit_bit_exact(dtype, d):
    h, cap, off, n = 3, 300, 77, 131
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    ks, vs = S.tensor(7, "k", h, n, d, dtype), S.tensor(7, "v", h, n, d, dtype)
    # caches stored [B, S, H, D] and handed over as permuted views: exercises the strides
    kc = torch.full((1, cap, h, d), 5.0, dtype=tdt, device="cuda").permute(0, 2, 1, 3)
    vc = torch.full((1, cap, h, d), 5.0, dtype=tdt, device="cuda").permute(0, 2, 1, 3)
    s1f.kv_append(to_device(ks, dtype)[None], to_device(vs, dtype)[None], off, kc, vc)
    kco = np.full((h, cap, d), 5.0, dtype=np.float32); vco = kco.copy()
    C.kv_append(ks, vs, off, kco, vco)
    assert np.array_equal(kc[0].float().cpu().numpy(), kco) and np.array_equal(vc[0].float().cpu().numpy(), vco)

    acc_k = (S.tensor(8, "k", h, cap, d, "f32") * 3.7).astype(np.float32)
    acc_v = (S.tensor(8, "v", h, cap, d, "f32") * 0.013).astype(np.float32)
    dk = torch.full((1, h, n, d), float("nan"), dtype=tdt, device="cuda")
    dv = torch.full((1, h, n, d), float("nan"), dtype=tdt, device="cuda")
    s1f.kv_grad_emit(torch.from_numpy(acc_k)[None].cuda(), torch.from_numpy(acc_v)[None].cuda(), off, dk, dv)
    wk, wv = C.kv_grad_emit(acc_k, acc_v, off, n, dtype)
    assert np.array_equal(dk[0].float().cpu().numpy(), wk) and np.array_equal(dv[0].float().cpu().numpy(), wv)


def test_around_the_attention_calls():
    """Cache filled segment by segment (rows past the segment are NaN until appended); after the backward of
    segment i its emitted dK/dV rows already equal the gradient of the whole sequence."""
    hq, hkv, n, d, dtype = 4, 2, 600, 128, "bf16"
    bounds = s1f.partition(n, 3, 64, 4)
    q, k, v, do = (S.tensor(11, t, hh, n, d, dtype) for t, hh in (("q", hq), ("k", hkv), ("v", hkv), ("dout", hq)))
    qd, kd, vd, dod = (to_device(x, dtype)[None] for x in (q, k, v, do))
    kc = torch.full((1, hkv, n, d), float("nan"), dtype=torch.bfloat16, device="cuda"); vc = kc.clone()
    out = torch.empty_like(qd); dq = torch.empty_like(qd)
    dk_acc = torch.zeros((1, hkv, n, d), dtype=torch.float32, device="cuda"); dv_acc = torch.zeros_like(dk_acc)
    dk_out = torch.empty_like(kc); dv_out = torch.empty_like(kc)
    lses = []
    for a, b in zip(bounds[:-1], bounds[1:]):
        s1f.kv_append(kd[:, :, a:b], vd[:, :, a:b], a, kc, vc)
        lse = torch.empty((1, hq, b - a), dtype=torch.float32, device="cuda")
        s1f.seg_attn_fwd(qd[:, :, a:b], kc, vc, a, out[:, :, a:b], lse)
        lses.append(lse)
    for i in reversed(range(len(bounds) - 1)):
        a, b = bounds[i], bounds[i + 1]
        ws = torch.empty(s1f.bwd_workspace_bytes(qd[:, :, a:b], kc, a), dtype=torch.uint8, device="cuda")
        s1f.seg_attn_bwd(dod[:, :, a:b], qd[:, :, a:b], kc, vc, out[:, :, a:b], lses[i], a, dq[:, :, a:b], dk_acc, dv_acc, ws)
        s1f.kv_grad_emit(dk_acc, dv_acc, a, dk_out[:, :, a:b], dv_out[:, :, a:b])
    torch.cuda.synchronize()
    _, wdk, wdv = A.full_backward(do, q, k, v)
    for name, got, want in (("dk", dk_out, wdk), ("dv", dv_out, wdv)):
        mx, fro = errors(got[0].float().cpu().numpy(), want)
        assert mx <= 2e-2 + 2.0 ** -8 * np.abs(want).max() and fro <= 1e-2, (name, mx, fro)
