"""Pins for the oracle's primitives: closed forms, brute force, and independent library routines."""
import os

import math

import numpy as np
import pytest
import torch

from oracle import primitives as P
from oracle.hourglass import shorten, upsample

GOLD = os.path.join(os.path.dirname(__file__), "golden")
rng = np.random.default_rng(7)


def test_bf16_round_format_cases():
    for line in open(os.path.join(GOLD, "bf16_cases.txt")):
        if line.startswith("#") or not line.strip():
            continue
        a, b = line.split()
        x = np.array([int(a, 16)], np.uint32).view(np.float32)
        assert P.bf16_round(x).view(np.uint32)[0] == int(b, 16), line


def test_bf16_round_matches_torch_cast():
    x = rng.standard_normal(20000).astype(np.float32) * np.float32(10.0) ** rng.integers(-6, 6, 20000).astype(np.float32)
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(P.bf16_round(x), want)
    x64 = x.astype(np.float64)
    assert P.bf16_round(x64).dtype == np.float64 and np.array_equal(P.bf16_round(x64), want.astype(np.float64))


def test_rmsnorm_closed_form():
    x = np.array([[3.0, -4.0, 0.0, 0.0]])
    g = np.array([1.0, 2.0, 3.0, 4.0])
    # mean square = 25/4, so x / 2.5 * g when eps = 0
    assert np.allclose(P.rmsnorm(x, g, 0.0), [[1.2, -3.2, 0.0, 0.0]], rtol=0, atol=1e-15)
    y = P.rmsnorm(rng.standard_normal((5, 64)), np.ones(64), 0.0)
    assert np.allclose(np.mean(y * y, axis=-1), 1.0)
    xt = torch.randn(6, 32, dtype=torch.float64)
    gt = torch.randn(32, dtype=torch.float64)
    want = torch.nn.functional.rms_norm(xt, (32,), gt, eps=1e-6).numpy()
    assert np.allclose(P.rmsnorm(xt.numpy(), gt.numpy(), 1e-6), want, rtol=1e-12, atol=1e-12)


def test_gelu_and_softmax_match_library():
    x = torch.linspace(-6, 6, 401, dtype=torch.float64)
    want = torch.nn.functional.gelu(x, approximate="tanh").numpy()
    assert np.allclose(P.gelu_tanh(x.numpy()), want, rtol=1e-12, atol=1e-14)
    s = rng.standard_normal((4, 9)) * 5
    assert np.allclose(P.softmax(s), torch.softmax(torch.from_numpy(s), -1).numpy(), atol=1e-15)
    assert np.allclose(P.softmax(s).sum(-1), 1.0)


def test_rope_rotation_properties():
    q = rng.standard_normal((1, 2, 64))
    k = rng.standard_normal((1, 2, 64))
    # position 0 is the identity
    assert np.allclose(P.rope(q, [0], 10000.0), q, atol=0)
    # pairwise norms are preserved (pair = (i, i+32))
    r = P.rope(q, [37], 10000.0)
    assert np.allclose(q[..., :32] ** 2 + q[..., 32:] ** 2, r[..., :32] ** 2 + r[..., 32:] ** 2)
    # the inner product depends only on the position difference
    a = np.sum(P.rope(q, [11], 10000.0) * P.rope(k, [4], 10000.0), -1)
    b = np.sum(P.rope(q, [107], 10000.0) * P.rope(k, [100], 10000.0), -1)
    assert np.allclose(a, b, atol=1e-10)
    # pair 0 turns by exactly pos radians, pair 31 by pos * base**(-31/32)
    e = np.zeros((1, 1, 64))
    e[0, 0, 0] = 1.0
    e[0, 0, 31] = 1.0
    r = P.rope(e, [2], 10000.0)[0, 0]
    assert np.allclose([r[0], r[32]], [np.cos(2.0), np.sin(2.0)])
    th = 2.0 * 10000.0 ** (-31 / 32)
    assert np.allclose([r[31], r[63]], [np.cos(th), np.sin(th)])


def _attend_loops(q, K, V, limit):
    rows, H, D = q.shape
    out = np.zeros_like(q)
    for r in range(rows):
        for h in range(H):
            sc = []
            for j in range(limit[r] + 1):
                acc = 0.0
                for d in range(D):
                    acc += q[r, h, d] * K[j, h, d]
                sc.append(acc / 8.0)
            mx = max(sc)
            w = [np.exp(v - mx) for v in sc]
            z = sum(w)
            for d in range(D):
                out[r, h, d] = sum(w[j] * V[j, h, d] for j in range(len(w))) / z
    return out


def test_attend_matches_triple_loop():
    q = rng.standard_normal((4, 2, 64))
    K = rng.standard_normal((9, 2, 64))
    V = rng.standard_normal((9, 2, 64))
    lim = [0, 5, 8, 3]
    assert np.allclose(P.attend(q, K, V, lim), _attend_loops(q, K, V, lim), atol=1e-12)
    # same limit for every row takes the batched path
    assert np.allclose(P.attend(q, K, V, [6] * 4), _attend_loops(q, K, V, [6] * 4), atol=1e-12)
    # block-causal form
    got = P.attend_causal(q, K, V, 5)
    assert np.allclose(got, _attend_loops(q, K, V, [5, 6, 7, 8]), atol=1e-12)


def test_windowed_attention_closed_forms_and_brute_force():
    """Sliding window (Sec. 5.1 "window size"): a row with limit p sees the W keys [p - W + 1, p]."""
    q = rng.standard_normal((4, 2, 64))
    K = rng.standard_normal((12, 2, 64))
    V = rng.standard_normal((12, 2, 64))
    lim = [0, 5, 11, 3]
    # W = 1: softmax over a single key, the result is that key's value row
    got = P.attend(q, K, V, lim, window=1)
    for r, p_ in enumerate(lim):
        assert np.allclose(got[r], V[p_], atol=1e-13)
    assert np.allclose(P.attend_causal(q, K, V, 8, window=1), V[8:12], atol=1e-13)
    # identical keys: uniform weights, the result is the mean of exactly the visible values
    Kc = np.broadcast_to(K[:1], K.shape)
    for W in (2, 3, 5):
        got = P.attend(q, Kc, V, lim, window=W)
        for r, p_ in enumerate(lim):
            assert np.allclose(got[r], V[max(0, p_ - W + 1):p_ + 1].mean(axis=0), atol=1e-12), (W, r)
        got = P.attend_causal(q, Kc, V, 8, window=W)
        for r in range(4):
            assert np.allclose(got[r], V[8 + r - W + 1:8 + r + 1].mean(axis=0), atol=1e-12), (W, r)
    # brute force: plain attention over the slice of visible keys
    for W in (1, 4, 7, 50):
        got = P.attend(q, K, V, lim, window=W)
        for r, p_ in enumerate(lim):
            a = max(0, p_ - W + 1)
            want = _attend_loops(q[r:r + 1], K[a:p_ + 1], V[a:p_ + 1], [p_ - a])
            assert np.allclose(got[r], want[0], atol=1e-12), (W, r)
        assert np.allclose(P.attend_causal(q, K, V, 8, window=W), P.attend(q, K, V, [8, 9, 10, 11], window=W), atol=1e-12)
        assert np.allclose(P.attend(q, K, V, [9] * 4, window=W), _attend_loops(q, K[max(0, 10 - W):10], V[max(0, 10 - W):10], [min(W, 10) - 1] * 4), atol=1e-12)
    # a window that covers everything changes nothing
    assert np.array_equal(P.attend(q, K, V, lim, window=12), P.attend(q, K, V, lim))
    assert np.array_equal(P.attend_causal(q, K, V, 8, window=12), P.attend_causal(q, K, V, 8))


def test_attend_matches_torch_sdpa():
    q = torch.randn(5, 3, 64, dtype=torch.float64)
    K = torch.randn(5, 3, 64, dtype=torch.float64)
    V = torch.randn(5, 3, 64, dtype=torch.float64)
    want = torch.nn.functional.scaled_dot_product_attention(
        q.permute(1, 0, 2)[None], K.permute(1, 0, 2)[None], V.permute(1, 0, 2)[None], is_causal=True)[0].permute(1, 0, 2)
    got = P.attend_causal(q.numpy(), K.numpy(), V.numpy(), 0)
    assert np.allclose(got, want.numpy(), atol=1e-12)


@pytest.mark.parametrize("T", [1, 2, 3, 4, 9, 10, 28, 30])
def test_shorten_upsample_brute_force(T):
    d = 4
    h = rng.standard_normal((T, d))
    W = rng.standard_normal((d, d))
    got = shorten(h, W)
    n = (T - 1) // 3 + 1
    assert got.shape == (n, d)
    for j in range(n):
        acc = np.zeros(d)
        for i in (3 * j - 2, 3 * j - 1, 3 * j):
            if 0 <= i < T:
                acc += h[i]
        acc /= 3.0                      # always three slots, also for the zero-padded first group
        want = np.array([sum(W[o, i] * acc[i] for i in range(d)) for o in range(d)])
        assert np.allclose(got[j], want, atol=1e-12)
    y = rng.standard_normal((n, d))
    up = upsample(h, y)
    for i in range(T):
        assert np.allclose(up[i], h[i] + y[i // 3])
    # causality of the pair: coarse row floor(i/3) only pools fine rows <= i
    for i in range(T):
        assert 3 * (i // 3) <= i


@pytest.mark.parametrize("hd", [64, 96, 128])
def test_rope_and_attention_take_the_head_width_from_their_operands(hd):
    """Head widths of the paper's own models (Sec. 5.1: 96 and 128): pair i of a head turns by pos * base^(-i / (hd/2)),
    scores are scaled by 1/sqrt(hd)."""
    rng = np.random.default_rng(hd)
    x = rng.standard_normal((3, 2, hd))
    pos = np.array([0, 5, 1234])
    y = P.rope(x, pos, 10000.0)
    assert np.allclose(y[0], x[0])                                         # position 0: identity
    for i in (0, 1, hd // 2 - 1):
        ang = pos[2] * 10000.0 ** (-i / (hd / 2))
        a, b = x[2, 1, i], x[2, 1, i + hd // 2]
        assert abs(y[2, 1, i] - (a * math.cos(ang) - b * math.sin(ang))) < 1e-9
        assert abs(y[2, 1, i + hd // 2] - (b * math.cos(ang) + a * math.sin(ang))) < 1e-9
    assert np.allclose(np.linalg.norm(y, axis=-1), np.linalg.norm(x, axis=-1))
    q, K, V = rng.standard_normal((2, 2, hd)), rng.standard_normal((7, 2, hd)), rng.standard_normal((7, 2, hd))
    out = P.attend(q, K, V, [3, 6])
    for r, lim in enumerate((3, 6)):
        for h in range(2):
            sc = np.array([q[r, h] @ K[j, h] for j in range(lim + 1)]) / math.sqrt(hd)
            w = np.exp(sc - sc.max())
            w /= w.sum()
            assert np.allclose(out[r, h], sum(w[j] * V[j, h] for j in range(lim + 1)))
    assert np.allclose(P.attend_causal(q, K, V, 5), P.attend(q, K, V, [5, 6]))
