"""TEST INFRASTRUCTURE ONLY - slow, plain CPU definitions of the primitives.

Only tests, the smoke check and the benchmark's cpu_baseline leg may use
anything in this package; the product path never does.

Every function here is the textbook definition written out with NumPy, in the
floating-point type of its inputs (float64 unless a test asks otherwise).
The paper (Sec. 3.1, "Speculative Prediction Block") only says that a block is
self-attention, cross-attention to the condition c and a feed-forward network;
the concrete choices (RMSNorm, rotary positions, tanh-GELU) come from the
benchmark configuration list and are listed as readings in the design notes.
"""
from __future__ import annotations

import numpy as np

HEAD_DIM = 64      # head width of the five benchmark configurations; every function below takes the width from its operands


def bf16_round(x):
    """Nearest-even rounding to bfloat16, via float32 (the device rounds float32 values)."""
    x32 = np.ascontiguousarray(x, dtype=np.float32)
    u = x32.view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    y = ((u + r) & np.uint32(0xFFFF0000)).astype(np.uint32).view(np.float32).reshape(x32.shape)
    return y.astype(np.asarray(x).dtype, copy=False)


def rmsnorm(x, g, eps):
    """x * g / sqrt(mean(x^2) + eps) over the last axis."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * g


def gelu_tanh(x):
    return 0.5 * x * (1.0 + np.tanh(np.sqrt(2.0 / np.pi) * (x + 0.044715 * x ** 3)))


def softmax(x):
    z = x - np.max(x, axis=-1, keepdims=True)
    e = np.exp(z)
    return e / np.sum(e, axis=-1, keepdims=True)


def rope(x, pos, base):
    """Rotary position embedding on [rows, heads, hd] with half-split pairing (i, i + hd/2).

    Pair i is rotated by the angle pos * base**(-i/(hd/2)); hd = 64 in the benchmark configurations, 96 / 128 in the
    paper's own model shapes (Sec. 5.1)."""
    half = x.shape[-1] // 2
    pos = np.asarray(pos, dtype=np.float64)
    inv = base ** (-np.arange(half, dtype=np.float64) / half)
    ang = pos[:, None] * inv[None, :]                     # [rows, 32], always float64
    c = np.cos(ang).astype(x.dtype)[:, None, :]
    s = np.sin(ang).astype(x.dtype)[:, None, :]
    a, b = x[..., :half], x[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def attend(q, K, V, limit, window=0):
    """Scaled dot-product attention, one query row at a time over keys [first, limit[row]].

    q [rows, H, hd]; K, V [L, H, hd]; limit[row] is the last visible key (inclusive).
    window = 0: first = 0.  window = W > 0 (sliding window, Sec. 5.1 "window size"): a row sees the
    W keys that end at its limit, first = max(0, limit[row] - W + 1).
    Scores are scaled by 1/sqrt(hd); softmax in the working precision."""
    rows, H, hd = q.shape
    out = np.zeros_like(q)
    scale = 1.0 / np.sqrt(hd)
    lim = np.asarray(limit)
    if rows and np.all(lim == lim[0]):
        # all rows see the same keys: one batched product per head
        n = int(lim[0]) + 1
        a = max(0, n - window) if window > 0 else 0
        s = np.matmul(q.transpose(1, 0, 2), K[a:n].transpose(1, 2, 0)) * scale    # [H, rows, n - a]
        return np.matmul(softmax(s), V[a:n].transpose(1, 0, 2)).transpose(1, 0, 2)
    for r in range(rows):
        n = int(lim[r]) + 1
        a = max(0, n - window) if window > 0 else 0
        s = np.einsum("hd,khd->hk", q[r], K[a:n]) * scale
        out[r] = np.einsum("hk,khd->hd", softmax(s), V[a:n])
    return out


def attend_causal(q, K, V, first_pos, window=0):
    """Block-causal attention: row r (absolute position p = first_pos + r) sees keys [0, p], or with a
    window W > 0 the keys [max(0, p - W + 1), p].

    Same result as attend(q, K, V, first_pos + arange(rows), window) but with one masked
    matrix product per head, for long teacher-forced blocks."""
    rows, H, hd = q.shape
    n = first_pos + rows
    scale = 1.0 / np.sqrt(hd)
    s = np.matmul(q.transpose(1, 0, 2), K[:n].transpose(1, 2, 0)) * scale        # [H, rows, n]
    kk = np.arange(n)[None, :]
    rr = (first_pos + np.arange(rows))[:, None]
    seen = kk <= rr
    if window > 0:
        seen = seen & (kk > rr - window)
    s = np.where(seen[None, :, :], s, -np.inf)
    return np.matmul(softmax(s), V[:n].transpose(1, 0, 2)).transpose(1, 0, 2)
