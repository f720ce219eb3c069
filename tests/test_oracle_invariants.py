"""Invariants that pin the oracle's backbone and decode loop without any other implementation."""
import os

import numpy as np
import pytest

import synth_inputs as si
from oracle import primitives as P
from oracle import correct as oc
from oracle import sampling as smp
from oracle import speculative as sp
from oracle.hourglass import Model, SeqState, forward_block, forward_full

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _model(name, jitter=0.1, **kw):
    cfg = si.TEST_CONFIGS[name]
    if kw:
        cfg = cfg.replace(**kw)
    return cfg, Model(cfg, si.make_weights(cfg, 0, jitter)), si.make_memory(cfg, 0)


def _tokens(cfg, n, seed=3):
    r = np.random.default_rng(seed)
    return [cfg.bos] + [int(t) for t in r.integers(0, cfg.n_bins, n - 1)]


# -- T1: incremental decoding equals full-sequence recompute ------------------------------
@pytest.mark.parametrize("name", ["t_f32_99", "t_bf16_99", "t_f32_hd96", "t_f32_hd128"])
def test_incremental_equals_full(name):
    cfg, m, mem = _model(name)
    T = 64
    toks = _tokens(cfg, T)
    taps = {}
    full = forward_full(m, toks, mem, taps)
    tol = 1e-9 if cfg.dtype == "f32" else 2e-2
    r = np.random.default_rng(5)
    for trial in range(6):
        st = SeqState(m, mem, T)
        i = 0
        while i < T:
            B = int(r.integers(1, 20)) if trial else 1
            B = min(B, T - i)
            lg = forward_block(m, st, toks[i:i + B], long_block=bool(trial % 2))
            assert np.abs(lg - full[i:i + B]).max() < tol, (trial, i, B)
            i += B
            st.P = i
            assert SeqState.level_lengths(i) == (i, (i - 1) // 3 + 1, (i - 1) // 9 + 1)
        if cfg.dtype == "f32":
            assert np.abs(st.tap["c"][:T] - taps["tap_c"]).max() < 1e-9
            nv, nf = (T - 1) // 3 + 1, (T - 1) // 9 + 1
            assert np.abs(st.tap["v"][:nv] - taps["tap_v"]).max() < 1e-9
            assert np.abs(st.tap["f"][:nf] - taps["tap_f"]).max() < 1e-9
            assert np.abs(st.y_f[:nf] - taps["y_f"]).max() < 1e-9


@pytest.mark.parametrize("window", [9, 18, 27])
def test_incremental_equals_full_with_sliding_window(window):
    """With a window shorter than the sequence the cached block forward still equals the full recompute,
    and the logits differ from the unwindowed model once the window has started to drop keys."""
    cfg, m, mem = _model("t_f32_99", window=window)
    _, m_all, _ = _model("t_f32_99")
    T = 64
    toks = _tokens(cfg, T)
    full = forward_full(m, toks, mem)
    full_all = forward_full(m_all, toks, mem)
    # the face level sees window/9 faces: position p is unaffected while p < window/9 * 9 - 8 at least
    assert np.abs(full[:window // 9] - full_all[:window // 9]).max() < 1e-12
    assert np.abs(full[window + 9:] - full_all[window + 9:]).max() > 1e-6
    r = np.random.default_rng(11)
    for trial in range(4):
        st = SeqState(m, mem, T)
        i = 0
        while i < T:
            B = min(int(r.integers(1, 20)) if trial else 1, T - i)
            lg = forward_block(m, st, toks[i:i + B], long_block=bool(trial % 2))
            assert np.abs(lg - full[i:i + B]).max() < 1e-9, (trial, i, B)
            i += B
            st.P = i


def test_sliding_window_forgets_old_tokens():
    """Changing a token that has left the window of every level cannot change a later logit row; changing one
    inside the window does (the window is measured in the level's own positions: W, W/3, W/9)."""
    cfg, m, mem = _model("t_f32_99", window=9)
    T = 118
    toks = _tokens(cfg, T)
    base = forward_full(m, toks, mem)
    # Information from position 3 travels at most one window per layer and level; the chain is finite, so far
    # enough downstream the logits are untouched.  Windows 9 / 3 / 1: per coordinate layer 8 positions (3 layers),
    # per vertex layer 2 vertices = 6 positions (3 layers), the face layers see their own face only; the two
    # poolings and upsamplings add at most 2 + 8 + 8 positions: under 70 in all.
    other = list(toks)
    other[3] = (other[3] + 1) % cfg.n_bins
    alt = forward_full(m, other, mem)
    assert np.abs(alt[4] - base[4]).max() > 1e-9
    _, m_all, _ = _model("t_f32_99")
    reach_all = np.abs(forward_full(m_all, other, mem) - forward_full(m_all, toks, mem)).max(axis=1)
    reach = np.abs(alt - base).max(axis=1)
    assert reach_all[-1] > 1e-9            # without a window the change is visible to the end
    last = np.nonzero(reach > 0)[0].max()
    assert last < 3 + 70 and reach[-1] == 0.0, last


def test_speculative_equals_sequential_with_sliding_window():
    cfg, m, mem = _model("t_f32_99", window=18, faces=8)
    seq, _ = sp.generate(m, mem, cfg.faces, speculative=False)
    spec, _ = sp.generate(m, mem, cfg.faces, speculative=True)
    assert seq == spec and len(seq) == 9 * cfg.faces
    _, m_all, _ = _model("t_f32_99", faces=8)
    seq_all, _ = sp.generate(m_all, mem, cfg.faces, speculative=False)
    assert seq_all[:18] == seq[:18]


def test_every_block_length_and_phase():
    """All block lengths 1..19 from every start phase mod 9, re-verified after a partial commit."""
    cfg, m, mem = _model("t_f32_c")
    T = 48
    toks = _tokens(cfg, T)
    full = forward_full(m, toks, mem)
    for P0 in range(0, 9):
        st = SeqState(m, mem, T)
        if P0:
            forward_block(m, st, toks[:P0])
            st.P = P0
        for B in range(1, 20):
            # a wrong block first (rejected drafts must leave no trace) ...
            junk = toks[P0:P0 + 1] + [(t + 1) % cfg.n_bins for t in toks[P0 + 1:P0 + B]]
            forward_block(m, st, junk)
            # ... then the right one
            lg = forward_block(m, st, toks[P0:P0 + B])
            assert np.abs(lg - full[P0:P0 + B]).max() < 1e-9, (P0, B)


# -- T3: causality ----------------------------------------------------------------------------
def test_causality_probe():
    cfg, m, mem = _model("t_f32_99")
    T = 30
    toks = _tokens(cfg, T)
    base = forward_full(m, toks, mem)
    for qpos in (1, 3, 8, 9, 10, 17, 18, 26):
        t2 = list(toks)
        t2[qpos] = (t2[qpos] + 5) % cfg.n_bins
        out = forward_full(m, t2, mem)
        assert np.array_equal(out[:qpos], base[:qpos]), qpos
        assert not np.allclose(out[qpos], base[qpos])


def test_hourglass_collapses_when_shortening_is_zero():
    """With W_s(coord->vertex) = 0 and the coarse levels' cross-attention outputs zeroed, every coarse
    feature is exactly zero (RMSNorm(0) = 0, no biases), so the model must equal the flat stack
    cpre -> cpost: pins that upsample adds nothing else."""
    cfg, m, mem = _model("t_f32_99")
    m.w["short_cv"] = np.zeros_like(m.w["short_cv"])
    for k in list(m.w):
        if k.split(".")[0] in ("vpre", "face", "vpost") and k.endswith(".co"):
            m.w[k] = np.zeros_like(m.w[k])
    T = 20
    toks = _tokens(cfg, T)
    got = forward_full(m, toks, mem)
    h = m.embed(toks)
    pos = np.arange(T)
    for stack in ("cpre", "cpost"):
        for i in range(m.layers[stack]):
            pfx = f"{stack}.{i}."
            q, k, v = m.qkv(pfx, h, pos)
            o = P.attend(q, k, v, pos)
            h = m.after_self_attention(pfx, h, o, *m.mem_kv(pfx, mem))
    assert np.abs(got - m.logits(h)).max() < 1e-10


def test_single_block_is_textbook_attention():
    """One block with the cross-attention and FFN outputs zeroed is h + Wo * softmax(QK^T/8) V."""
    cfg, m, mem = _model("t_f32_c", jitter=0.0)
    pfx = "cpre.0."
    m.w[pfx + "co"] = np.zeros_like(m.w[pfx + "co"])
    m.w[pfx + "w2"] = np.zeros_like(m.w[pfx + "w2"])
    T = 7
    h = np.random.default_rng(1).standard_normal((T, cfg.d_model))
    q, k, v = m.qkv(pfx, h, np.zeros(T))          # position 0 everywhere: rotary is the identity
    out = m.after_self_attention(pfx, h, P.attend_causal(q, k, v, 0), *m.mem_kv(pfx, mem))
    x = h / np.sqrt(np.mean(h * h, -1, keepdims=True) + cfg.rms_eps)
    want = h.copy()
    for r in range(T):
        for hd in range(cfg.n_heads):
            sl = slice(64 * hd, 64 * hd + 64)
            qq = m.w[pfx + "wq"][sl] @ x[r]
            sc = np.array([qq @ (m.w[pfx + "wk"][sl] @ x[j]) / 8.0 for j in range(r + 1)])
            wgt = np.exp(sc - sc.max())
            wgt /= wgt.sum()
            o = sum(wgt[j] * (m.w[pfx + "wv"][sl] @ x[j]) for j in range(r + 1))
            want[r] += m.w[pfx + "wo"][:, sl] @ o
    assert np.abs(out - want).max() < 1e-10


# -- T4: speculative greedy == sequential greedy -------------------------------------------------
@pytest.mark.parametrize("name", ["t_f32_c", "t_f32_99", "t_f32_1815", "t_bf16_99", "t_f32_hd96"])
def test_speculative_equals_sequential_native_heads(name):
    cfg, m, mem = _model(name)
    seq, st0 = sp.generate(m, mem, cfg.faces, speculative=False)
    trace = []
    spec, st1 = sp.generate(m, mem, cfg.faces, speculative=True, trace=trace)
    assert seq == spec and len(seq) == 9 * cfg.faces
    assert st0.P == st1.P == 9 * cfg.faces
    assert sum(a for _, _, a in trace) == 9 * cfg.faces
    assert all(1 <= a <= len(b) <= cfg.block_max for _, b, a in trace)


def test_speculative_equals_sequential_adversarial_drafts():
    cfg, m, mem = _model("t_f32_99")
    faces = 5
    truth, _ = sp.generate(m, mem, faces, speculative=False)
    x = [cfg.bos] + truth                      # x[p] = token index p
    wrong = lambda t: (t + 1) % cfg.n_bins
    r = np.random.default_rng(11)

    def source(kind, k=None):
        def fn(st, budget):
            B = min(cfg.block_max, budget - st.P)
            true = [x[st.P + i] for i in range(B)]
            if kind == "correct":
                return true
            if kind == "wrong":
                return [true[0]] + [wrong(t) for t in true[1:]]
            if kind == "random":
                return [true[0]] + [int(t) for t in r.integers(0, cfg.n_bins, B - 1)]
            blk = list(true)                   # corrupted at index k
            if k < B:
                blk[k] = wrong(blk[k])
            return blk
        return fn

    for kind in ("correct", "wrong", "random"):
        trace = []
        out, _ = sp.generate(m, mem, faces, draft_fn=source(kind), trace=trace)
        assert out == truth, kind
        if kind == "correct":
            assert all(a == len(b) for _, b, a in trace)
        if kind == "wrong":
            assert all(a == 1 for _, _, a in trace)
    for k in range(1, cfg.block_max):
        trace = []
        out, _ = sp.generate(m, mem, faces, draft_fn=source("corrupt", k), trace=trace)
        assert out == truth
        for _, b, a in trace:
            assert a == min(k, len(b)), (k, len(b), a)


def test_accept_truth_table():
    """Brute force over every match pattern for D = 1..5 drafts (Sec. 3.3: main accepted outright,
    then the longest run of drafts that equal the backbone's own predictions)."""
    for D in range(1, 6):
        for pattern in range(1 << D):
            y = list(range(100, 100 + D + 1))
            block = [7] + [y[i] if (pattern >> i) & 1 else -1 for i in range(D)]
            lead = 0
            while lead < D and (pattern >> lead) & 1:
                lead += 1
            assert sp.accept_length(block, y) == 1 + lead


def test_eos_stops_generation():
    cfg, m, mem = _model("t_f32_99", ban_specials=0)
    # bias the LM head so that EOS wins everywhere: the first predicted token ends the mesh
    m.w["lm"][cfg.eos] = 50.0 * m.w["lm"][cfg.eos] + 0.0
    m.w["gf"] = np.ones_like(m.w["gf"])
    out, st = sp.generate(m, mem, 3, speculative=True)
    assert out[-1] == cfg.eos or len(out) == 27
    if out[-1] == cfg.eos:
        assert st.finished and cfg.eos not in out[:-1]


# -- T5: schedule against the paper's worked example -----------------------------------------------
def _walk(cfg, m, mem, n_pos):
    """Commit one true token at a time and record what each level covers at every position s."""
    st = SeqState(m, mem, 9 * cfg.faces)
    rec = {}
    while st.P < n_pos:
        block = sp.draft(m, st, 9 * cfg.faces)
        s = st.P - 1
        if s >= 0:
            rec[s] = {l: sorted(st.rows[l]) for l in "cvf"} | {"len": len(block)}
        _, y, _ = sp.verify(m, st, [st.main])
        sp.commit(m, st, [st.main], y, 1)
    return rec


def test_schedule_9_9_worked_example():
    gold = {}
    for line in open(os.path.join(GOLD, "schedule_9_9.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, main, c, p, total, dbl = line.split()
        gold[name] = ([int(v) for v in c.split(",")], [int(v) for v in p.split(",")], int(total),
                      [] if dbl == "none" else [int(v) for v in dbl.split(",")])
    # the example shows the point and coordinate levels only: switch the face level off
    cfg, m, mem = _model("t_f32_99", draft_face=0, faces=4)
    rec = _walk(cfg, m, mem, 18)
    for s in (3, 6, 12, 15):                      # point split nodes that are not face nodes
        for name, ss in (("at_point_node", s), ("one_position_later", s + 1)):
            if ss not in rec:
                continue
            c, p, total, dbl = gold[name]
            main = ss + 1
            assert [t - main for t in rec[ss]["c"]] == c
            assert [t - main for t in rec[ss]["v"]] == p
            assert rec[ss]["len"] == total
            assert sorted(set(rec[ss]["c"]) & set(rec[ss]["v"])) == [main + v for v in dbl]
        assert rec[s]["f"] == []


def test_step_totals_and_rules():
    for line in open(os.path.join(GOLD, "step_totals.txt")):
        if line.startswith("#") or not line.strip():
            continue
        n, mm, dc, at_face, at_point = (int(v) for v in line.split())
        name = "t_f32_1815" if n == 18 else "t_f32_99"
        cfg, m, mem = _model(name, faces=8)
        assert (cfg.draft_face, cfg.draft_point, cfg.draft_coord) == (n, mm, dc)
        rec = _walk(cfg, m, mem, 40)
        fired_v_at = []
        for s in sorted(rec):
            main = s + 1
            if s % 9 == 0:
                # rule (B): the face level leaves the first three future tokens to the coordinate level
                assert rec[s]["f"] == list(range(main + 3, main + n))
                assert rec[s]["len"] == at_face
                # rule (A): no fresh point-level rows at a face node (fresh rows would end at main+mm-1)
                assert main + mm - 1 not in rec[s]["v"]
            elif s % 3 == 0:
                assert rec[s]["v"] == list(range(main + 3, main + mm))
                assert rec[s]["len"] == at_point
                fired_v_at.append(s)
            assert rec[s]["c"] == [main + 1, main + 2]
        assert fired_v_at == [s for s in sorted(rec) if s % 3 == 0 and s % 9 != 0]


def test_rule_a_switched_off_lets_the_point_level_fire_at_face_nodes():
    """Supplement "Optimizations": rule (A) drops the point-level prediction where a face-level one fires.  With the
    rule off both fire at a face split node and cover the same positions; everything else is unchanged, and the
    emitted stream is the backbone's either way."""
    cfg, m, mem = _model("t_f32_99", faces=8, rule_a=0)
    rec = _walk(cfg, m, mem, 40)
    n, mm = cfg.draft_face, cfg.draft_point
    for s in sorted(rec):
        main = s + 1
        if s % 3 == 0:
            assert rec[s]["v"] == list(range(main + 3, main + mm))           # also where s % 9 == 0
        if s % 9 == 0:
            assert rec[s]["f"] == list(range(main + 3, main + n))
            assert sorted(set(rec[s]["v"]) & set(rec[s]["f"])) == list(range(main + 3, main + min(n, mm)))
        assert rec[s]["c"] == [main + 1, main + 2]
    cfg_on, m_on, _ = _model("t_f32_99", faces=8)
    rec_on = _walk(cfg_on, m_on, mem, 40)
    assert all(rec_on[s]["len"] == rec[s]["len"] for s in rec)                # the face level already covered the block
    a, _ = sp.generate(m, mem, 4, speculative=True)
    b, _ = sp.generate(m_on, mem, 4, speculative=False)
    assert a == b


def test_rule_b_switched_off_keeps_the_first_three_tokens_of_the_upper_levels():
    """Supplement "Optimizations": rule (B) drops the first three tokens of a point- or face-level prediction because the
    coordinate level predicts them anyway.  With the rule off the upper levels keep them (offset 0 is the main token's
    own slot and is never asked for), so the two coordinate-level positions are covered twice and the block length stays."""
    cfg, m, mem = _model("t_f32_99", draft_face=0, faces=4, rule_b=0)
    rec = _walk(cfg, m, mem, 18)
    for s in (3, 6, 12, 15):                                   # point split nodes (face level off, as in the 9-9 example)
        main = s + 1
        assert rec[s]["v"] == list(range(main, main + cfg.draft_point))
        assert rec[s]["c"] == [main + 1, main + 2] and rec[s]["len"] == 9
        assert sorted(set(rec[s]["c"]) & set(rec[s]["v"])) == [main + 1, main + 2]
        if s + 1 in rec:                                       # one position later: one token shorter, both fresh rows doubled
            assert rec[s + 1]["len"] == 8
            assert sorted(set(rec[s + 1]["c"]) & set(rec[s + 1]["v"])) == [main + 2, main + 3]
    cfg, m, mem = _model("t_f32_1815", faces=6, rule_a=0, rule_b=0)
    rec = _walk(cfg, m, mem, 30)
    for s in sorted(rec):
        main = s + 1
        if s % 9 == 0:
            assert rec[s]["f"] == list(range(main, main + cfg.draft_face)) and rec[s]["len"] == 18
        if s % 3 == 0:
            assert rec[s]["v"] == list(range(main, main + cfg.draft_point))
    a, _ = sp.generate(m, mem, 4, speculative=True)
    b, _ = sp.generate(m, mem, 4, speculative=False)
    assert a == b
    assert sp.point_targets(2, 9, rule_b=False) == list(range(7, 16)) and sp.point_targets(2, 9) == list(range(10, 16))
    assert sp.face_targets(1, 9, rule_b=False) == list(range(10, 19)) and sp.face_targets(1, 9) == list(range(13, 19))


# -- T7: residual wiring of the draft heads ------------------------------------------------------
def test_sp_and_hf_residual_wiring():
    cfg, m, mem = _model("t_f32_99", faces=3)
    for k, v in m.w.items():
        if k.startswith("sp.") and k.endswith(".lin"):
            m.w[k] = np.zeros_like(v)
        if k.startswith("hf.") and k.endswith(".w2"):
            m.w[k] = np.zeros_like(v)
    st = SeqState(m, mem, 27)
    toks = _tokens(cfg, 14)
    forward_block(m, st, toks[:13])
    st.P = 13
    st.main = toks[13]
    sp.draft(m, st, 27)
    s = 12
    # Eq. 1 with Linear = 0 leaves h_s: every coordinate head predicts from the tapped feature itself
    want = P.softmax(m.logits(st.tap["c"][s][None]))[0]
    for tgt in (s + 2, s + 3):
        assert np.allclose(st.rows["c"][tgt], want, atol=1e-12)
    # Eq. 6 with FFN = 0 is the identity on the upsampled feature; Eq. 1 then gives the vertex tap
    v = s // 3
    want_v = P.softmax(m.logits(st.tap["v"][v][None]))[0]
    assert sorted(st.rows["v"]) == list(range(3 * v + 4, 3 * v + 10))
    for tgt in st.rows["v"]:
        assert np.allclose(st.rows["v"][tgt], want_v, atol=1e-12)
    # face level (fired at s = 9): with n = 9 there is no face SP head; the face output repeats down
    f = 1
    want_f = P.softmax(m.logits(st.y_f[f][None]))[0]
    assert st.fired_f == f and sorted(st.rows["f"]) == list(range(9 * f + 4, 9 * f + 10))
    for tgt in st.rows["f"]:
        assert np.allclose(st.rows["f"][tgt], want_f, atol=1e-12)


def test_sp_and_hf_closed_form_with_uniform_self_attention():
    """With a zero query projection every visible key gets the same weight, so the self-attention of an SP head
    (Eq. 1) or HF block (Eq. 3-6) is the mean of the cached values; the rest of the chain is then written out here
    step by step with plain loops (cross-attention scores, softmax, tanh-GELU) and must match."""
    cfg, m, mem = _model("t_f32_99", faces=3)
    st = SeqState(m, mem, 27)
    toks = _tokens(cfg, 14)
    forward_block(m, st, toks[:13])
    st.P = 13
    s, d, H = 12, cfg.d_model, cfg.n_heads
    r = np.random.default_rng(4)
    pfx = "cpost.%d." % (cfg.l_cpost - 1)                    # the last layer of the coordinate level
    # --- SP head 1 of the coordinate level
    m.w["sp.c.1.wq"] = np.zeros((d, d))
    h_s = r.standard_normal(d)
    got = sp.sp_head(m, st, "c", 1, h_s, s)
    vmean = st.V[pfx][:s + 1].mean(axis=0).reshape(d)        # uniform weights over keys 0..s, heads side by side
    a = m.w["sp.c.1.wo"] @ vmean
    q2 = (m.w["sp.c.1.cq"] @ a).reshape(H, 64)
    Km, Vm = st.Kmem[pfx], st.Vmem[pfx]                       # [M, H, 64]
    c = np.zeros((H, 64))
    for h in range(H):
        sc = np.array([np.dot(q2[h], Km[j, h]) / 8.0 for j in range(Km.shape[0])])
        w = np.exp(sc - sc.max())
        w /= w.sum()
        for j in range(Km.shape[0]):
            c[h] += w[j] * Vm[j, h]
    want = m.w["sp.c.1.lin"] @ (m.w["sp.c.1.co"] @ c.reshape(d)) + h_s
    assert np.allclose(got, want, atol=1e-10)
    # --- HF block of coordinate offset t = 3: keys 0..limit, FFN with tanh-GELU, residual on the upsampled feature
    m.w["hf.c.3.wq"] = np.zeros((d, d))
    h_up = r.standard_normal(d)
    limit = 9
    got = sp.hf_block(m, st, "c", 3, h_up, limit + 3, limit)
    vmean = st.V[pfx][:limit + 1].mean(axis=0).reshape(d)
    z = m.w["hf.c.3.w1"] @ vmean
    gelu = 0.5 * z * (1.0 + np.tanh(np.sqrt(2.0 / np.pi) * (z + 0.044715 * z ** 3)))
    want = h_up + m.w["hf.c.3.w2"] @ gelu
    assert np.allclose(got, want, atol=1e-10)
    # the visible range matters: one key fewer changes the result
    assert not np.allclose(sp.hf_block(m, st, "c", 3, h_up, limit + 3, limit - 1), want, atol=1e-6)


def test_sp_and_hf_query_side_by_rotary_retrieval():
    """The query side of the heads (norm gain, W_q, rotary position of the query).  Keys are set to one vector rotated
    to their positions; a query that is a large multiple of the same vector rotated to position q scores
    big * sum_i |u_i|^2 cos((q - j) theta_i) against key j, so the softmax collapses onto one key that the test can
    name: j = s for an SP head (its query stands at s), and for an HF block with all the energy in the first rotary
    pair (theta = 1) and q = limit + 3 the key at distance 6 (cos 6 = 0.96 beats distances 3, 4, 5, 7 ... 12), which is
    not the key a query standing at `limit` would pick."""
    cfg, m, mem = _model("t_f32_99", faces=3)
    st = SeqState(m, mem, 27)
    toks = _tokens(cfg, 14)
    forward_block(m, st, toks[:13])
    st.P = 13
    s, d, H = 12, cfg.d_model, cfg.n_heads
    r = np.random.default_rng(8)
    pfx = "cpost.%d." % (cfg.l_cpost - 1)

    def rest_of_sp(a_heads, h_s):
        a = m.w["sp.c.1.wo"] @ a_heads.reshape(d)
        q2 = (m.w["sp.c.1.cq"] @ a).reshape(H, 64)
        Km, Vm = st.Kmem[pfx], st.Vmem[pfx]
        c = np.zeros((H, 64))
        for h in range(H):
            sc = np.array([np.dot(q2[h], Km[j, h]) / 8.0 for j in range(Km.shape[0])])
            w = np.exp(sc - sc.max())
            c[h] = (w[:, None] * Vm[:, h]).sum(axis=0) / w.sum()
        return m.w["sp.c.1.lin"] @ (m.w["sp.c.1.co"] @ c.reshape(d)) + h_s

    # --- SP head: the query stands at s, so it retrieves the value cached at s
    u = r.standard_normal((H, 64))
    for j in range(s + 1):
        st.K[pfx][j] = P.rope(u[None], [j], cfg.rope_base)[0]
    h_s = r.standard_normal(d)
    g = 1.0 + 0.3 * r.standard_normal(d)
    m.w["sp.c.1.g"] = g
    n = P.rmsnorm(h_s[None], g, cfg.rms_eps)[0]
    m.w["sp.c.1.wq"] = 60.0 * np.outer(u.reshape(d), n) / np.dot(n, n)         # W_q n = 60 u
    got = sp.sp_head(m, st, "c", 1, h_s, s)
    assert np.allclose(got, rest_of_sp(st.V[pfx][s], h_s), atol=1e-9)
    assert not np.allclose(got, rest_of_sp(st.V[pfx][s - 1], h_s), atol=1e-6)
    # --- HF block: the query stands at the slot it predicts for (limit + 3), not at the last visible key
    u1 = np.zeros((H, 64))
    u1[:, 0] = 1.0
    limit, pos = 9, 12
    for j in range(limit + 1):
        st.K[pfx][j] = P.rope(u1[None], [j], cfg.rope_base)[0]
    h_up = r.standard_normal(d)
    g = 1.0 + 0.3 * r.standard_normal(d)
    m.w["hf.c.3.g"] = g
    n = P.rmsnorm(h_up[None], g, cfg.rms_eps)[0]
    m.w["hf.c.3.wq"] = 16000.0 * np.outer(u1.reshape(d), n) / np.dot(n, n)
    got = sp.hf_block(m, st, "c", 3, h_up, pos, limit)

    def rest_of_hf(v_heads):
        z = m.w["hf.c.3.w1"] @ v_heads.reshape(d)
        return h_up + m.w["hf.c.3.w2"] @ (0.5 * z * (1.0 + np.tanh(np.sqrt(2.0 / np.pi) * (z + 0.044715 * z ** 3))))

    assert np.allclose(got, rest_of_hf(st.V[pfx][pos - 6]), atol=1e-9)
    assert not np.allclose(got, rest_of_hf(st.V[pfx][limit]), atol=1e-6)


# -- correct stage (Sec. 3.2) ---------------------------------------------------------------
def _correct_cases():
    for line in open(os.path.join(GOLD, "correct_cases.txt")):
        if line.startswith("#") or not line.strip():
            continue
        f = [x.strip() for x in line.split("|")]
        labels = {int(a): int(b) for a, b in (kv.split(":") for kv in f[3].split())}
        yield int(f[0]), [int(t) for t in f[1].split()], [int(t) for t in f[2].split()], labels, int(f[4]), [int(t) for t in f[5].split()]


def test_correct_stage_worked_examples():
    cfg = si.TEST_CONFIGS["t_f32_99"]
    n = 0
    for Pc, known, block, labels, hv, want in _correct_cases():
        assert len(known) == Pc + 1 and known[-1] == block[0]
        assert oc.correct_block(cfg, Pc, block, labels, known, hv) == want, (Pc, block)
        n += 1
    assert n == 6


def test_correct_stage_properties_random_blocks():
    """Random blocks and labels: the main token and every token outside the block's own points never change;
    points labelled new only move within their face; whole draft faces come out sorted; all-new labels on
    sorted faces change nothing; the nearest rule agrees with a brute-force search."""
    cfg = si.TEST_CONFIGS["t_f32_99"]
    r = np.random.default_rng(12)
    for trial in range(300):
        Pc = int(r.integers(0, 40))
        B = int(r.integers(1, 28))
        known = [cfg.bos] + [int(t) for t in r.integers(0, 6, Pc)]
        block = [known[-1]] + [int(t) for t in r.integers(0, 6, B - 1)]
        if trial % 7 == 0 and B > 3:
            block[int(r.integers(1, B))] = cfg.eos
        u0, u1 = oc.draft_vertex_range(Pc, B)
        labels = {u: int(r.integers(0, 3)) for u in range(u0, u1 + 1) if r.random() < 0.8}
        hv = int(r.integers(0, 8))
        out = oc.correct_block(cfg, Pc, block, labels, known, hv)
        assert len(out) == B and out[0] == block[0]
        lo, hi = 3 * u0 + 1 - Pc, 3 * u1 + 4 - Pc      # block indices of the complete draft vertices
        for i in range(B):
            if not (lo <= i < hi):
                assert out[i] == block[i], (trial, i)
        tri = lambda b, u: tuple(b[3 * u + 1 - Pc:3 * u + 4 - Pc])
        ok = lambda c: all(t < cfg.n_bins for t in c)
        for f in range((u0 + 2) // 3, (u1 + 1) // 3):
            vs = [3 * f, 3 * f + 1, 3 * f + 2]
            if all(ok(tri(out, u)) for u in vs):
                assert [tri(out, u) for u in vs] == sorted(tri(out, u) for u in vs)
        # brute force of the two move rules on the first point that qualifies, before any other move can interfere
        pts = [u for u in range(u0, u1 + 1) if ok(tri(block, u))]
        hist = [(h, tuple(known[3 * h + 1:3 * h + 4])) for h in range(max(0, Pc // 3 - hv), Pc // 3)]
        if pts:
            u = pts[0]
            c = np.array(tri(block, u))
            moved = None
            if labels.get(u, oc.NEW) == oc.HIST and hist and all(tuple(c) != hc for _, hc in hist):
                dd = np.array([((c - np.array(hc)) ** 2).sum() for _, hc in hist])
                moved = hist[int(np.argmin(dd))][1]
            if labels.get(u, oc.NEW) == oc.INTRA and all(tri(block, w) != tuple(c) for w in pts[1:]):
                cand = [w for w in pts[1:] if labels.get(w, oc.NEW) == oc.NEW and w // 3 != u // 3]
                if cand:
                    dd = np.array([((c - np.array(tri(block, w))) ** 2).sum() for w in cand])
                    moved = tri(block, cand[int(np.argmin(dd))])
            if moved is not None:
                # the point now holds `moved` (possibly at another slot of its face after the re-sort)
                f = u // 3
                face = [tri(out, w) for w in range(max(3 * f, u0), min(3 * f + 2, u1) + 1)]
                assert tuple(moved) in face, (trial, u, moved, face)
        # all-new labels: only the sort acts
        out2 = oc.correct_block(cfg, Pc, out, {}, known, hv)
        out3 = oc.correct_block(cfg, Pc, out2, {}, known, hv)
        assert out2 == out3


def test_correct_stage_keeps_the_stream():
    """The correct stage edits drafts only, so the emitted stream is still plain greedy decoding (Sec. 3.2, 3.3),
    while the blocks that are verified do change."""
    cfg, m, mem = _model("t_f32_1815")
    seq, _ = sp.generate(m, mem, cfg.faces, speculative=False)
    t0, t1 = [], []
    plain, _ = sp.generate(m, mem, cfg.faces, speculative=True, trace=t0)
    fixed, _ = sp.generate(m, mem, cfg.faces, speculative=True, trace=t1, correct_hist=6)
    assert seq == plain == fixed
    assert [b for _, b, _ in t0] != [b for _, b, _ in t1]
    assert all(b0[0] == b1[0] for (_, b0, _), (_, b1, _) in zip(t0[:3], t1[:3]))


def test_label_rows_are_softmax_of_the_linear_head():
    cfg, m, mem = _model("t_f32_99")
    f = np.random.default_rng(2).standard_normal(cfg.d_model)
    row = oc.label_row(m, f)
    z = np.array([float(np.dot(m.w["label"][i], f)) for i in range(3)])
    assert np.allclose(row, np.exp(z) / np.exp(z).sum(), atol=1e-14) and abs(row.sum() - 1.0) < 1e-14


# -- non-greedy verification (oracle.sampling) ----------------------------------------------------
def test_inverse_cdf_closed_forms():
    w = np.array([0.0, 2.0, 0.0, 1.0, 1.0])
    assert smp.inverse_cdf(w, 0.0) == 1                       # first index with weight
    assert [smp.inverse_cdf(w, u) for u in (0.49, 0.5, 0.74, 0.75, 0.999999)] == [1, 3, 3, 4, 4]
    assert smp.inverse_cdf(np.ones(8), 0.37) == 2             # uniform weights: floor(8 u)
    assert smp.inverse_cdf(np.ones(8) * 1e-30, 0.999) == 7
    r = np.random.default_rng(0)
    w = r.random(50)
    for u in r.random(200):
        i = smp.inverse_cdf(w, u)
        assert w[:i].sum() <= u * w.sum() < w[:i + 1].sum() + 1e-12


def test_target_row_is_tempered_softmax_and_tends_to_greedy():
    z = np.array([0.3, -1.0, 2.0, 1.9, 7.0, 0.0])
    p = smp.target_row(z, 4, 0.5)                               # only the first four tokens are admissible
    want = np.exp(z[:4] / 0.5)
    assert np.allclose(p, want / want.sum(), atol=1e-15) and len(p) == 4
    assert np.argmax(smp.target_row(z, 4, 1e-3)) == 2 and smp.target_row(z, 4, 1e-3)[2] > 1 - 1e-12


def test_rejection_rule_special_cases():
    p = np.array([0.5, 0.3, 0.2, 0.0])
    # proposal equal to the target: every draft is accepted
    assert all(smp.accept_draft(p, p, x, u) for x in range(3) for u in (0.0, 0.5, 0.999999))
    # a draft the target gives no mass is always rejected and the replacement comes from the target itself
    q = np.array([0.0, 0.0, 0.0, 1.0])
    assert not smp.accept_draft(p, q, 3, 0.0)
    assert np.allclose(smp.residual(p, q, 3), p)
    # general case: acceptance probability min(1, p/q), residual max(p - q, 0)
    q = np.array([0.1, 0.6, 0.3, 0.0])
    assert smp.accept_draft(p, q, 0, 0.999999)                                   # p/q = 5
    assert smp.accept_draft(p, q, 1, 0.49) and not smp.accept_draft(p, q, 1, 0.51)   # p/q = 1/2
    assert np.allclose(smp.residual(p, q, 1), [0.4, 0.0, 0.0, 0.0])
    # point-mass proposal: accepted with probability p(x), replacement from p without x
    assert smp.accept_draft(p, None, 1, 0.29) and not smp.accept_draft(p, None, 1, 0.31)
    assert np.allclose(smp.residual(p, None, 1), [0.5, 0.0, 0.2, 0.0])
    # a draft outside the admissible tokens is rejected
    assert not smp.accept_draft(p, None, 7, 0.0)


def test_speculative_sampling_reproduces_the_target_distribution():
    """The defining property: draw a draft from q, apply the rejection test, and the token that comes out is
    distributed as the target p, whatever q is (chi-square against p over many draws, two positions deep)."""
    r = np.random.default_rng(3)
    V, N = 6, 60000
    for trial in range(3):
        p0, p1 = r.dirichlet(np.ones(V)), r.dirichlet(np.ones(V) * 0.5)
        q0, q1 = r.dirichlet(np.ones(V) * 2.0), r.dirichlet(np.ones(V))
        if trial == 2:
            q0 = None                                      # point-mass proposals (a replayed draft)
        first = np.zeros(V)
        second_given_accept = np.zeros(V)
        n_acc = 0
        for _ in range(N):
            u = r.random(6)
            x1 = smp.inverse_cdf(q0, u[0]) if q0 is not None else int(r.integers(0, V))
            x2 = smp.inverse_cdf(q1, u[1])
            a, tok = smp.verify_rows([p0, p1, p0], [q0, q1, None], [0, x1, x2], u[2:5], [u[5], r.random(), r.random()])
            emitted = [x1, x2][:a - 1] + [tok]
            first[emitted[0]] += 1
            if a >= 2:
                n_acc += 1
                second_given_accept[emitted[1]] += 1
        chi = ((first - N * p0) ** 2 / (N * p0)).sum()
        assert chi < 25.0, (trial, chi)                    # 5 degrees of freedom: P(chi2 > 25) ~ 1e-4
        chi2 = ((second_given_accept - n_acc * p1) ** 2 / (n_acc * p1)).sum()
        assert chi2 < 25.0, (trial, chi2)


def test_sampled_generation_is_keyed_and_tends_to_greedy():
    cfg, m, mem = _model("t_f32_99")
    a, _ = sp.generate(m, mem, cfg.faces, True, sampling=(1.0, 5))
    b, _ = sp.generate(m, mem, cfg.faces, True, sampling=(1.0, 5))
    c, _ = sp.generate(m, mem, cfg.faces, True, sampling=(1.0, 6))
    assert a == b and a != c and len(a) == 9 * cfg.faces
    greedy, _ = sp.generate(m, mem, cfg.faces, True)
    cold, _ = sp.generate(m, mem, cfg.faces, True, sampling=(1e-4, 5))
    assert cold == greedy
    cold_seq, _ = sp.generate(m, mem, cfg.faces, False, sampling=(1e-4, 9))
    assert cold_seq == greedy
