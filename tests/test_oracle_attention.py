"""Pins of the attention oracle (oracle/attention.py and oracle/attn_rows.c) against things other than
itself: a hand-worked example, closed forms, invariants, finite differences, an independent library
routine, and the paper's claim that segment-wise execution leaves results unchanged (Sections 3.1-3.2)."""
import math

import numpy as np
import pytest
import torch

import s1f_synth as S
from oracle import attention as A
from oracle import rows as R


def _rand(hq, hkv, n, d, seed=7, dtype="f32"):
    return (S.tensor(seed, "q", hq, n, d, dtype).astype(np.float64),
            S.tensor(seed, "k", hkv, n, d, dtype).astype(np.float64),
            S.tensor(seed, "v", hkv, n, d, dtype).astype(np.float64),
            S.tensor(seed, "dout", hq, n, d, dtype).astype(np.float64))


def _golden(golden_dir):
    vals = {}
    for line in open(f"{golden_dir}/two_token_attention.txt"):
        if line.startswith("#") or not line.strip():
            continue
        key, *nums = line.split()
        vals[key] = np.array([float(x) for x in nums])
    return vals


def test_two_token_worked_example(golden_dir):
    g = _golden(golden_dir)
    q = np.array([[[1.0], [2.0]]]); k = np.array([[[1.0], [3.0]]]); v = np.array([[[2.0], [5.0]]])
    do = np.ones((1, 2, 1))
    o, lse = A.full_forward(q, k, v)
    dq, dk, dv = A.full_backward(do, q, k, v)
    for name, got in (("o", o), ("lse", lse), ("dq", dq), ("dk", dk), ("dv", dv)):
        np.testing.assert_allclose(got.reshape(-1), g[name], rtol=1e-14, atol=1e-15, err_msg=name)
    # the C rows oracle on the same example
    o2, lse2 = R.forward_rows(q, k, v, 0, 0, 2)
    np.testing.assert_allclose(o2.reshape(-1), g["o"], rtol=1e-14)
    np.testing.assert_allclose(lse2, g["lse"], rtol=1e-14)
    np.testing.assert_allclose(R.dq_rows(q, k, v, do, 0, 0, 2).reshape(-1), g["dq"], rtol=1e-13, atol=1e-15)
    dk2, dv2 = R.dkdv_keys(q, k, v, do, 0, 0, 2)
    np.testing.assert_allclose(dk2.reshape(-1), g["dk"], rtol=1e-13)
    np.testing.assert_allclose(dv2.reshape(-1), g["dv"], rtol=1e-13)


def test_probability_rows_sum_to_one_and_are_causal():
    q, k, _, _ = _rand(1, 1, 40, 8)
    p, _ = A._probabilities(q[0, 10:30], k[0], 10)
    np.testing.assert_allclose(p.sum(axis=1), 1.0, rtol=1e-14)
    for r in range(20):
        assert np.all(p[r, 10 + r + 1:] == 0.0) and np.all(p[r, :10 + r + 1] > 0.0)


def test_first_token_sees_only_itself():
    q, k, v, _ = _rand(3, 3, 9, 4)
    o, lse = A.full_forward(q, k, v)
    np.testing.assert_allclose(o[:, 0], v[:, 0], rtol=1e-15)
    np.testing.assert_allclose(lse[:, 0], (q[:, 0] * k[:, 0]).sum(-1) / 2.0, rtol=1e-14)


def test_identical_keys_give_running_mean():
    q, k, v, do = _rand(2, 2, 33, 8)
    k[:] = k[:, :1]
    o, lse = A.full_forward(q, k, v)
    mean = np.cumsum(v, axis=1) / np.arange(1, 34)[None, :, None]
    np.testing.assert_allclose(o, mean, rtol=1e-12, atol=1e-13)
    s = (q * k).sum(-1) / math.sqrt(8)
    np.testing.assert_allclose(lse, s + np.log(np.arange(1, 34))[None], rtol=1e-12, atol=1e-12)
    dq, dk, dv = A.full_backward(do, q, k, v)
    np.testing.assert_allclose(dq, 0.0, atol=1e-13)          # uniform softmax: no score gradient reaches q
    o2, lse2 = R.forward_rows(q, k, v, 1, 0, 33)
    np.testing.assert_allclose(o2, mean[1], rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(R.dq_rows(q, k, v, do, 1, 0, 33), 0.0, atol=1e-13)


def test_constant_values_give_constant_output():
    q, k, v, _ = _rand(2, 1, 20, 8)
    v[:] = v[:, :1]
    o, _ = A.full_forward(q, k, v)
    np.testing.assert_allclose(o, np.broadcast_to(v[0, 0], o.shape), rtol=1e-13)


@pytest.mark.parametrize("hq,hkv,n,d", [(2, 2, 48, 16), (4, 2, 37, 8), (8, 1, 25, 80)])
def test_against_library_attention_and_autograd(hq, hkv, n, d):
    """Second opinion: torch's scaled_dot_product_attention (CPU, fp64, is_causal) and its autograd."""
    q, k, v, do = _rand(hq, hkv, n, d, seed=11)
    tq, tk, tv = (torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in (q, k, v))
    rep = hq // hkv
    to = torch.nn.functional.scaled_dot_product_attention(
        tq[None], tk.repeat_interleave(rep, 0)[None], tv.repeat_interleave(rep, 0)[None], is_causal=True)[0]
    (to * torch.tensor(do)).sum().backward()
    o, lse = A.full_forward(q, k, v)
    dq, dk, dv = A.full_backward(do, q, k, v)
    np.testing.assert_allclose(o, to.detach().numpy(), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(dq, tq.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dk, tk.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dv, tv.grad.numpy(), rtol=1e-10, atol=1e-12)
    # lse against a direct logsumexp of the visible scores
    for h in range(hq):
        s = torch.tensor(q[h] @ k[h // rep].T / math.sqrt(d))
        for i in (0, n // 2, n - 1):
            assert abs(torch.logsumexp(s[i, :i + 1], 0).item() - lse[h, i]) < 1e-12
    # C rows oracle against the same library results
    for h in (0, hq - 1):
        o2, lse2 = R.forward_rows(q, k, v, h, 3, n)
        np.testing.assert_allclose(o2, to.detach().numpy()[h, 3:], rtol=1e-11, atol=1e-12)
        np.testing.assert_allclose(lse2, lse[h, 3:], rtol=1e-12)
        np.testing.assert_allclose(R.dq_rows(q, k, v, do, h, 0, n - 2), tq.grad.numpy()[h, :n - 2],
                                   rtol=1e-10, atol=1e-12)
    for g in (0, hkv - 1):
        dk2, dv2 = R.dkdv_keys(q, k, v, do, g, 2, n)
        np.testing.assert_allclose(dk2, tk.grad.numpy()[g, 2:], rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose(dv2, tv.grad.numpy()[g, 2:], rtol=1e-10, atol=1e-12)


def test_backward_matches_finite_differences():
    hq, hkv, n, d = 4, 2, 12, 6
    q, k, v, do = _rand(hq, hkv, n, d, seed=3)
    dq, dk, dv = A.full_backward(do, q, k, v)

    def loss(q_, k_, v_):
        return float((A.full_forward(q_, k_, v_)[0] * do).sum())

    rng = np.random.default_rng(0)
    eps = 1e-6
    for arr, grad, which in ((q, dq, 0), (k, dk, 1), (v, dv, 2)):
        for _ in range(25):
            idx = tuple(rng.integers(0, s) for s in arr.shape)
            plus = [q.copy(), k.copy(), v.copy()]; minus = [q.copy(), k.copy(), v.copy()]
            plus[which][idx] += eps; minus[which][idx] -= eps
            fd = (loss(*plus) - loss(*minus)) / (2 * eps)
            assert abs(fd - grad[idx]) < 1e-7 * max(1.0, abs(fd)), (which, idx, fd, grad[idx])


def test_gradient_invariants():
    hq, hkv, n, d = 6, 2, 50, 8
    q, k, v, do = _rand(hq, hkv, n, d, seed=5)
    dq, dk, dv = A.full_backward(do, q, k, v)
    # columns of a row-stochastic P: every dO row is distributed in full over the values it saw
    np.testing.assert_allclose(dv.sum(axis=1), do.reshape(hkv, 3, n, d).sum(axis=(1, 2)), rtol=1e-12, atol=1e-12)
    # softmax is shift invariant in the scores: moving all keys by a common vector changes nothing
    np.testing.assert_allclose(dk.sum(axis=1), 0.0, atol=1e-12)


@pytest.mark.parametrize("boundaries", [[0, 16, 32, 48, 64], [0, 1, 2, 64], [0, 23, 24, 50, 64], [0, 64]])
def test_segmentwise_execution_equals_full_sequence(boundaries):
    """The paper's equivalence claim: forward in order / backward in reverse with accumulation gives
    exactly full-sequence attention and gradients; after the backward of segment i its dK/dV rows are final."""
    hq, hkv, n, d = 4, 2, 64, 8
    q, k, v, do = _rand(hq, hkv, n, d, seed=9)
    o, lse = A.full_forward(q, k, v)
    dq, dk, dv = A.full_backward(do, q, k, v)
    o2, lse2, dq2, dk2, dv2, trace = A.segmented_schedule(q, k, v, do, boundaries)
    for got, want in ((o2, o), (lse2, lse), (dq2, dq), (dk2, dk), (dv2, dv)):
        np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-13)
    for i in range(len(boundaries) - 1):
        a, b = boundaries[i], boundaries[i + 1]
        np.testing.assert_allclose(trace[i][0][:, a:b], dk[:, a:b], rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(trace[i][1][:, a:b], dv[:, a:b], rtol=1e-12, atol=1e-13)
        if a > 0 and i > 0:   # earlier rows still miss the contributions of segments before i
            assert np.abs(trace[i][1][:, :a] - dv[:, :a]).max() > 1e-6


def test_rows_oracle_matches_dense_oracle_on_bf16_inputs():
    hq, hkv, n, d = 4, 2, 200, 80
    q, k, v, do = _rand(hq, hkv, n, d, seed=13, dtype="bf16")
    o, lse = A.full_forward(q, k, v)
    dq, dk, dv = A.full_backward(do, q, k, v)
    o2, lse2 = R.forward_rows(q, k, v, 3, 50, 200)
    np.testing.assert_allclose(o2, o[3, 50:], rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(lse2, lse[3, 50:], rtol=1e-13)
    np.testing.assert_allclose(R.dq_rows(q, k, v, do, 1, 0, 120), dq[1, :120], rtol=1e-11, atol=1e-12)
    dk2, dv2 = R.dkdv_keys(q, k, v, do, 1, 100, 200)
    np.testing.assert_allclose(dk2, dk[1, 100:], rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(dv2, dv[1, 100:], rtol=1e-11, atol=1e-12)
