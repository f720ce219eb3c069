"""Pins of the oracle's transformer block, output head and level averaging against definitions written out with
plain loops (no oracle routine is called on the reference side).

Sec. 3.1 ("Speculative Prediction Block") fixes the block as self-attention, cross-attention to the condition c, and a
feed-forward network, each with a residual; the supplement ("Integrating the three levels") averages the predicted
distributions of the levels that cover a position.  A swapped gain, a dropped residual, a transposed weight or a
cross-attention / feed-forward order swap changes the loop result by far more than the tolerance used here, and the
planted-mistake cases at the end of each test show it.
"""
import math

import numpy as np

import synth_inputs as si
from oracle import primitives as P
from oracle import speculative as sp
from oracle.hourglass import Model, SeqState, forward_block

HD = 64


def _matvec(W, x):
    """y[o] = sum_i W[o][i] x[i], one scalar product at a time."""
    return [math.fsum(W[o][i] * x[i] for i in range(len(x))) for o in range(len(W))]


def _rms(x, g, eps):
    ms = math.fsum(v * v for v in x) / len(x)
    r = 1.0 / math.sqrt(ms + eps)
    return [x[i] * r * g[i] for i in range(len(x))]


def _rot(x, pos, base):
    """Rotary position on one head vector of 64 values: pair (i, i + 32) turned by pos * base^(-i/32)."""
    y = list(x)
    for i in range(HD // 2):
        ang = pos * base ** (-i / (HD / 2))
        c, s = math.cos(ang), math.sin(ang)
        a, b = x[i], x[i + HD // 2]
        y[i], y[i + HD // 2] = a * c - b * s, b * c + a * s
    return y


def _soft(z):
    m = max(z)
    e = [math.exp(v - m) for v in z]
    t = math.fsum(e)
    return [v / t for v in e]


def _attn_row(q, keys, vals):
    """One head, one query: softmax(q.k / sqrt(64)) weighted sum of the values."""
    p = _soft([math.fsum(q[i] * k[i] for i in range(HD)) / math.sqrt(HD) for k in keys])
    return [math.fsum(p[j] * vals[j][i] for j in range(len(vals))) for i in range(HD)]


def _gelu(u):
    return 0.5 * u * (1.0 + math.tanh(math.sqrt(2.0 / math.pi) * (u + 0.044715 * u ** 3)))


def _block_by_loops(w, pfx, h, pos, mem, cfg):
    """One transformer block on rows h (positions pos, each row seeing the rows up to itself) with the condition memory."""
    d, H, eps, base = cfg.d_model, cfg.n_heads, cfg.rms_eps, cfg.rope_base
    W = {k: w[pfx + k].astype(np.float64).tolist() for k in ("wq", "wk", "wv", "wo", "cq", "ck", "cv", "co", "w1", "w2")}
    g = {k: w[pfx + k].astype(np.float64).tolist() for k in ("g1", "g2", "g3")}
    rows = len(h)
    # self-attention sub-layer
    q, k, v = [], [], []
    for r in range(rows):
        x = _rms(h[r], g["g1"], eps)
        qr, kr, vr = _matvec(W["wq"], x), _matvec(W["wk"], x), _matvec(W["wv"], x)
        q.append([_rot(qr[a * HD:(a + 1) * HD], pos[r], base) for a in range(H)])
        k.append([_rot(kr[a * HD:(a + 1) * HD], pos[r], base) for a in range(H)])
        v.append([vr[a * HD:(a + 1) * HD] for a in range(H)])
    h1 = []
    for r in range(rows):
        o = []
        for a in range(H):
            o += _attn_row(q[r][a], [k[j][a] for j in range(r + 1)], [v[j][a] for j in range(r + 1)])
        y = _matvec(W["wo"], o)
        h1.append([h[r][i] + y[i] for i in range(d)])
    # cross-attention sub-layer: keys / values straight from the memory rows (no norm, no rotary on that side)
    km = [_matvec(W["ck"], m) for m in mem]
    vm = [_matvec(W["cv"], m) for m in mem]
    h2 = []
    for r in range(rows):
        q2 = _matvec(W["cq"], _rms(h1[r], g["g2"], eps))
        o = []
        for a in range(H):
            o += _attn_row(q2[a * HD:(a + 1) * HD], [m[a * HD:(a + 1) * HD] for m in km], [m[a * HD:(a + 1) * HD] for m in vm])
        y = _matvec(W["co"], o)
        h2.append([h1[r][i] + y[i] for i in range(d)])
    # feed-forward sub-layer
    out = []
    for r in range(rows):
        u = _matvec(W["w1"], _rms(h2[r], g["g3"], eps))
        y = _matvec(W["w2"], [_gelu(t) for t in u])
        out.append([h2[r][i] + y[i] for i in range(d)])
    return np.array(out)


def _block_by_oracle(model, pfx, h, pos, mem):
    q, k, v = model.qkv(pfx, h, pos)
    o = P.attend(q, k, v, np.arange(len(pos)))
    return model.after_self_attention(pfx, h, o, *model.mem_kv(pfx, mem))


def _setup(jitter=0.3):
    cfg = si.TEST_CONFIGS["t_f32_99"]
    w = si.make_weights(cfg, 0, jitter)
    mem = si.make_memory(cfg, 0)[:7].astype(np.float64)
    rng = np.random.default_rng(21)
    h = rng.standard_normal((4, cfg.d_model))
    pos = np.array([5, 6, 7, 8])
    return cfg, w, mem, h, pos


def test_one_block_matches_plain_loops():
    cfg, w, mem, h, pos = _setup()
    pfx = "vpost.1."
    want = _block_by_loops(w, pfx, h.tolist(), pos.tolist(), mem.tolist(), cfg)
    got = _block_by_oracle(Model(cfg, w), pfx, h, pos, mem)
    assert np.abs(got - want).max() < 1e-10
    # planted mistakes in the oracle's inputs: each must move the result far beyond the tolerance
    def mutated(**swap):
        w2 = dict(w)
        for a, b in swap.items():
            w2[pfx + a] = w[pfx + b]
        return _block_by_oracle(Model(cfg, w2), pfx, h, pos, mem)
    assert np.abs(mutated(g2="g3", g3="g2") - want).max() > 1e-3          # gains of the two later norms swapped
    assert np.abs(mutated(g1="g2", g2="g1") - want).max() > 1e-3
    assert np.abs(mutated(cq="co", co="cq") - want).max() > 1e-3          # cross-attention projections swapped
    assert np.abs(mutated(ck="cv", cv="ck") - want).max() > 1e-3
    w0 = dict(w)
    w0[pfx + "co"] = np.zeros_like(w[pfx + "co"])                          # cross-attention sub-layer dropped
    assert np.abs(_block_by_oracle(Model(cfg, w0), pfx, h, pos, mem) - want).max() > 1e-3
    wt = dict(w)
    wt[pfx + "cq"] = np.ascontiguousarray(w[pfx + "cq"].T)                 # a transposed operand
    assert np.abs(_block_by_oracle(Model(cfg, wt), pfx, h, pos, mem) - want).max() > 1e-3


def test_block_sublayer_order_is_self_cross_feedforward():
    """Cross-attention before the feed-forward network (Sec. 3.1): the loop block with the two later sub-layers
    exchanged is a different function, and the oracle agrees with the stated order only."""
    cfg, w, mem, h, pos = _setup()
    pfx = "cpre.0."
    want = _block_by_loops(w, pfx, h.tolist(), pos.tolist(), mem.tolist(), cfg)
    got = _block_by_oracle(Model(cfg, w), pfx, h, pos, mem)
    assert np.abs(got - want).max() < 1e-10
    # feed-forward first, then cross-attention, written with the same loops
    d, eps = cfg.d_model, cfg.rms_eps
    m = Model(cfg, w)
    q, k, v = m.qkv(pfx, h, pos)
    o = P.attend(q, k, v, np.arange(len(pos))).reshape(len(pos), d)
    W = {n: w[pfx + n].astype(np.float64) for n in ("wo", "cq", "ck", "cv", "co", "w1", "w2", "g2", "g3")}
    h1 = h + o @ W["wo"].T
    swapped = []
    for r in range(len(pos)):
        u = _matvec(W["w1"].tolist(), _rms(h1[r].tolist(), W["g3"].tolist(), eps))
        hf = h1[r] + np.array(_matvec(W["w2"].tolist(), [_gelu(t) for t in u]))
        q2 = _matvec(W["cq"].tolist(), _rms(hf.tolist(), W["g2"].tolist(), eps))
        km = [_matvec(W["ck"].tolist(), x) for x in mem.tolist()]
        vm = [_matvec(W["cv"].tolist(), x) for x in mem.tolist()]
        oo = []
        for a in range(cfg.n_heads):
            oo += _attn_row(q2[a * HD:(a + 1) * HD], [x[a * HD:(a + 1) * HD] for x in km], [x[a * HD:(a + 1) * HD] for x in vm])
        swapped.append(hf + np.array(_matvec(W["co"].tolist(), oo)))
    assert np.abs(np.array(swapped) - got).max() > 1e-3


def test_condition_memory_keys_values_match_plain_loops():
    cfg, w, mem, _, _ = _setup()
    pfx = "face.1."
    K, V = Model(cfg, w).mem_kv(pfx, mem)
    ck, cv = w[pfx + "ck"].astype(np.float64).tolist(), w[pfx + "cv"].astype(np.float64).tolist()
    for j, row in enumerate(mem.tolist()):
        kj, vj = _matvec(ck, row), _matvec(cv, row)
        for a in range(cfg.n_heads):
            assert np.abs(K[j, a] - np.array(kj[a * HD:(a + 1) * HD])).max() < 1e-12
            assert np.abs(V[j, a] - np.array(vj[a * HD:(a + 1) * HD])).max() < 1e-12


def test_output_head_matches_plain_loops():
    """logits = W_lm RMSNorm(h; g_f): one scalar product per vocabulary entry."""
    cfg, w, _, h, _ = _setup()
    got = Model(cfg, w).logits(h)
    gf, lm = w["gf"].astype(np.float64).tolist(), w["lm"].astype(np.float64).tolist()
    for r in range(h.shape[0]):
        want = _matvec(lm, _rms(h[r].tolist(), gf, cfg.rms_eps))
        assert np.abs(got[r] - np.array(want)).max() < 1e-11
    assert got.shape == (h.shape[0], cfg.vocab)
    # planted mistake: the final gain left out
    w1 = dict(w)
    w1["gf"] = np.ones_like(w["gf"])
    assert np.abs(Model(cfg, w1).logits(h) - got).max() > 1e-3


def test_merged_draft_row_is_the_arithmetic_mean_of_the_levels():
    """Supplement, "Integrating the three levels": a position covered by several levels gets the mean of their
    distributions and the draft token is its arg max.  Rows of the point and face levels are set by hand (kept from an
    earlier firing); the coordinate level's rows are whatever its heads produce in this call."""
    cfg = si.TEST_CONFIGS["t_f32_99"]                       # Dc = 2, m = n = 9
    model = Model(cfg, si.make_weights(cfg, 0, 0.1))
    mem = si.make_memory(cfg, 0)
    st = SeqState(model, mem, 90)
    toks = [cfg.bos] + [int(t) for t in np.random.default_rng(2).integers(0, cfg.n_bins, 10)]
    forward_block(model, st, toks)
    st.P, st.main = len(toks), 4                            # s = 10: neither a vertex nor a face split node fires below
    s = st.P - 1
    st.fired_v, st.fired_f = s // 3, s // 9
    V = cfg.vocab

    def row(peaks):
        r = np.full(V, 0.0)
        for i, p in peaks.items():
            r[i] = p
        r[V - 1] = 1.0 - r.sum()                            # the rest of the mass on a special token (never chosen)
        return r
    A, B, C = row({3: 0.50, 7: 0.40}), row({5: 0.50, 7: 0.45}), row({9: 0.9})
    A2, B2 = row({3: 0.50, 7: 0.40}), row({5: 0.50, 7: 0.45})
    st.rows["v"] = {s + 2: A, s + 4: A2}
    st.rows["f"] = {s + 2: B, s + 3: C, s + 4: B2}
    merged = []
    block = sp.draft(model, st, 90, merged)
    c2, c3 = st.rows["c"][s + 2], st.rows["c"][s + 3]      # the coordinate level covers x_{s+2}, x_{s+3} only
    assert sorted(st.rows["c"]) == [s + 2, s + 3]
    assert len(block) == 4 and block[0] == 4
    assert np.abs(merged[0] - (c2 + A + B) / 3.0).max() < 1e-15
    assert np.abs(merged[1] - (c3 + C) / 2.0).max() < 1e-15
    assert np.abs(merged[2] - (A2 + B2) / 2.0).max() < 1e-15
    # the mean decides, not either level alone: 7 wins with 0.425 against 0.25 for the two single-level favourites
    assert block[3] == 7 and int(np.argmax(A2[:cfg.n_bins])) == 3 and int(np.argmax(B2[:cfg.n_bins])) == 5
    for i in (1, 2):
        assert block[i] == int(np.argmax(merged[i - 1][:cfg.n_bins]))
