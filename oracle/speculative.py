"""TEST INFRASTRUCTURE ONLY - plain CPU predict / verify / commit loop.

Follows Sec. 3.1 (SP-Block Eq. 1, draft upsample Eq. 2, HF-Block Eq. 3-6), the
supplement's "Three-Level Speculative Decoding", "Integrating the three levels"
and optimisation rules (A)/(B), and the verify mechanism of Sec. 3.3.  Greedy
only.  Where the paper is silent the reading taken is stated at the function.

Pins of the SP/HF draft heads (the paper prints no worked numbers for them): wiring special
cases (zeroed projections), a closed form of the whole chain under uniform self-attention
(zero query projection), the query side (norm gain, W_q, rotary position of the query) by
rotary retrieval of one key, and the model-free schedule against the supplement's 9-9 example.
"""
from __future__ import annotations

import numpy as np

from . import primitives as P
from .correct import correct_block, draft_vertex_range, label_row, point_labels
from .hourglass import Model, SeqState, forward_block
from . import sampling as smp


# ---------------------------------------------------------------------------------------
# Model-free schedule (supplement, "Optimizations" and its 9-9 worked example)
# ---------------------------------------------------------------------------------------
def coord_targets(s: int, Dc: int):
    """Token indices the coordinate-level SP heads predict from position s: x_{s+2} .. x_{s+1+Dc}."""
    return [s + 1 + d for d in range(1, Dc + 1)]


def point_fires(s: int, fired_v: int, m: int, rule_a: bool = True) -> bool:
    """Point level fires once per vertex token v = floor(s/3), except where the face level does (rule A; with the
    rule switched off it fires there as well and both levels cover the same positions)."""
    v = s // 3
    return m > 0 and s >= 0 and (v % 3 != 0 or not rule_a) and fired_v != v


def face_fires(s: int, fired_f: int, n: int) -> bool:
    f = s // 9
    return n > 0 and s >= 0 and fired_f != f


def point_targets(v: int, m: int, rule_b: bool = True):
    """Offsets t = 3 .. m-1 from the split node 3v predict x_{3v+t+1} (rule B drops t = 0..2; with the rule off they stay)."""
    return [3 * v + t + 1 for t in range(3 if rule_b else 0, m)]


def face_targets(f: int, n: int, rule_b: bool = True):
    return [9 * f + t + 1 for t in range(3 if rule_b else 0, n)]


# ---------------------------------------------------------------------------------------
# Draft heads
# ---------------------------------------------------------------------------------------
_LAST = {"c": "cpost", "v": "vpost", "f": "face"}


def _last_prefix(model: Model, lvl: str) -> str:
    stack = _LAST[lvl]
    return f"{stack}.{model.layers[stack] - 1}."


def sp_head(model: Model, st: SeqState, lvl: str, k: int, h_s, s_l: int):
    """Eq. 1: Linear(CA(SA(h_s), c)) + h_s for head k of level lvl.

    Reading: the head owns a norm gain, the query/output projections of both
    attentions and the final linear; keys/values (self and condition memory) are
    those the backbone cached for the LAST layer of the same level, rows [0, s_l]."""
    m, rnd, cfg = model, model.rnd, model.cfg
    p = f"sp.{lvl}.{k}."
    pfx = _last_prefix(m, lvl)
    x = rnd(P.rmsnorm(h_s[None, :], m.w[p + "g"], cfg.rms_eps))
    q = rnd(P.rope(m.heads(m.lin(x, p + "wq")), [s_l], cfg.rope_base))
    a = P.attend(q, st.K[pfx], st.V[pfx], [s_l], cfg.level_window(lvl)).reshape(1, m.d)
    a = m.lin(rnd(a), p + "wo")
    q2 = rnd(m.heads(m.lin(rnd(a), p + "cq")))
    c = P.attend(q2, st.Kmem[pfx], st.Vmem[pfx], [st.Kmem[pfx].shape[0] - 1]).reshape(1, m.d)
    c = m.lin(rnd(c), p + "co")
    return (m.lin(rnd(c), p + "lin") + h_s[None, :])[0]


def hf_block(model: Model, st: SeqState, lvl: str, t: int, h_up, pos: int, limit: int):
    """Eq. 3-6: h' + FFN_t(Attn(W_q^t h', K, V)) against the backbone's last-layer cache of level lvl.

    Reading: the query carries the rotary position of the slot it stands for (pos);
    visible keys are the committed rows up to and including the split node (limit)."""
    m, rnd, cfg = model, model.rnd, model.cfg
    p = f"hf.{lvl}.{t}."
    pfx = _last_prefix(m, lvl)
    x = rnd(P.rmsnorm(h_up[None, :], m.w[p + "g"], cfg.rms_eps))
    q = rnd(P.rope(m.heads(m.lin(x, p + "wq")), [pos], cfg.rope_base))
    a = P.attend(q, st.K[pfx], st.V[pfx], [limit], cfg.level_window(lvl)).reshape(1, m.d)
    z = rnd(P.gelu_tanh(m.lin(rnd(a), p + "w1")))
    return (h_up[None, :] + m.lin(z, p + "w2"))[0]


def _dist(model: Model, h):
    return P.softmax(model.logits(h[None, :]))[0]


def draft(model: Model, st: SeqState, budget_tokens: int, merged=None, sampling=None, seq=0):
    """Build the next verify block [main, drafts...] from the state left by the last commit.

    If `merged` is a list it receives the averaged distribution behind every draft token.
    sampling = (temperature, seed): the draft tokens are drawn from the averaged distributions
    (oracle.sampling) instead of their arg max."""
    m, cfg = model, model.cfg
    if st.finished:
        return []
    s = st.P - 1
    if s < 0:
        return [st.main]
    Dc, mm, nn = cfg.draft_coord, cfg.draft_point, cfg.draft_face
    rule_b = bool(getattr(cfg, "rule_b", 1))

    # coordinate level: every position (supplement, "Coordinate-level speculative decoding")
    rows = {}
    for k, tgt in zip(range(1, Dc + 1), coord_targets(s, Dc)):
        rows[tgt] = _dist(m, sp_head(m, st, "c", k, st.tap["c"][s], s))
    st.rows["c"] = rows

    # point level: SP heads on the vertex feature, repeat x3 (Eq. 2, no skip exists for a future
    # token), one coordinate-level HF block per offset
    if point_fires(s, st.fired_v, mm, bool(getattr(cfg, "rule_a", 1))):
        v = s // 3
        rows = {}
        labels = {}
        for k in range(1 if rule_b else 0, mm // 3):
            # k = 0 (rule (B) off): the current vertex, whose feature is the tapped one itself
            u = sp_head(m, st, "v", k, st.tap["v"][v], v) if k else st.tap["v"][v]
            if k:
                labels[v + k] = label_row(m, u)      # point-level feature of vertex v + k (Sec. 3.2)
            for t in (3 * k, 3 * k + 1, 3 * k + 2):
                rows[3 * v + t + 1] = _dist(m, hf_block(m, st, "c", t, u, 3 * v + t, 3 * v))
        st.rows["v"] = rows
        st.labels["v"] = labels
        st.fired_v = v

    # face level: the current face feature plus SP heads for later faces, repeat x3 to vertex
    # slots, vertex-level HF, repeat x3 to coordinate slots, coordinate-level HF
    if face_fires(s, st.fired_f, nn):
        f = s // 9
        g = [st.y_f[f]] + [sp_head(m, st, "f", k, st.tap["f"][f], f) for k in range(1, nn // 9)]
        rows = {}
        labels = {}
        for j in range(1 if rule_b else 0, nn // 3):
            hv = hf_block(m, st, "v", j, g[j // 3], 3 * f + j, 3 * f)
            labels[3 * f + j] = label_row(m, hv)     # point-level feature of vertex 3f + j
            for t in (3 * j, 3 * j + 1, 3 * j + 2):
                rows[9 * f + t + 1] = _dist(m, hf_block(m, st, "c", t, hv, 9 * f + t, 9 * f))
        st.rows["f"] = rows
        st.labels["f"] = labels
        st.fired_f = f

    # merge: mean of the distributions that cover a position; stop at the first gap
    block = [st.main]
    p = s + 2
    while len(block) < cfg.block_max and p < budget_tokens:
        have = [st.rows[l][p] for l in ("c", "v", "f") if p in st.rows[l]]
        if not have:
            break
        dist = sum(have) / float(len(have))
        if merged is not None:
            merged.append(dist)
        if sampling is None:
            block.append(pick(dist, cfg))
        else:
            n = cfg.n_bins if cfg.ban_specials else cfg.vocab
            block.append(smp.inverse_cdf(dist[:n], smp.uniform(sampling[1], seq, p, smp.DRAFT)))
        p += 1
    return block


def pick(scores, cfg) -> int:
    """Greedy choice: lowest index among exact ties; special tokens excluded when banned."""
    n = cfg.n_bins if cfg.ban_specials else cfg.vocab
    return int(np.argmax(scores[:n]))


# ---------------------------------------------------------------------------------------
# Verify / commit (Sec. 3.3)
# ---------------------------------------------------------------------------------------
def accept_length(block, y) -> int:
    """block[0] is the main token (accepted outright); draft i is accepted while it equals y[i-1]."""
    a = 1
    while a < len(block) and block[a] == y[a - 1]:
        a += 1
    return a


def verify(model: Model, st: SeqState, block):
    logits = forward_block(model, st, block)
    y = [pick(logits[i], model.cfg) for i in range(len(block))]
    return logits, y, accept_length(block, y)


def verify_sampled(model: Model, st: SeqState, block, proposals, sampling, seq=0):
    """Non-greedy verification (oracle.sampling).  proposals[i] is the averaged distribution block[i + 1] was drawn
    from, or None for a draft that did not come from it.  Returns (logits, y, a) in the shape verify() uses:
    only y[a - 1], the token emitted after the accepted prefix, is meaningful."""
    cfg = model.cfg
    T, seed = sampling
    n = cfg.n_bins if cfg.ban_specials else cfg.vocab
    logits = forward_block(model, st, block)
    B = len(block)
    ps = [smp.target_row(logits[i], n, T) for i in range(B)]
    qs = [None if proposals[i] is None else smp.proposal_row(proposals[i], n) for i in range(B - 1)] + [None]
    us_acc = [smp.uniform(seed, seq, st.P + i + 1, smp.ACCEPT) for i in range(B)]
    us_res = [smp.uniform(seed, seq, st.P + i + 1, smp.RESAMPLE) for i in range(B)]
    a, tok = smp.verify_rows(ps, qs, block, us_acc, us_res)
    y = [-1] * B
    y[a - 1] = tok
    return logits, y, a


def commit(model: Model, st: SeqState, block, y, a: int):
    """Accept block[:a]; the backbone's prediction after the last accepted token is the next main token.

    An accepted end-of-sequence draft is not fed as input: acceptance stops before it, so it
    becomes the pending main token and ends the sequence."""
    cfg = model.cfg
    for i in range(1, a):
        if block[i] == cfg.eos:
            a = i
            break
    st.tokens += list(block[:a])
    st.P += a
    st.main = y[a - 1]
    if st.main == cfg.eos:
        st.finished = True
    return a


def corrected(model: Model, st: SeqState, block, hist_vertices: int):
    """The draft block after the correct stage (Sec. 3.2), from the label rows the draft left in the state."""
    if len(block) < 4:
        return list(block)
    u0, u1 = draft_vertex_range(st.P, len(block))
    labels = {u: lab for u, (lab, _) in point_labels(st, u0, u1).items()}
    return correct_block(model.cfg, st.P, block, labels, st.tokens + [st.main], hist_vertices)


def generate(model: Model, mem, faces: int, speculative=True, draft_fn=None, trace=None, correct_hist=0, sampling=None,
             seq=0):
    """Greedy generation of up to `faces` faces.  Returns (x_1 .., final state); BOS excluded, the pending main token included.

    speculative=False is plain one-token-at-a-time decoding of the same backbone.
    draft_fn(st, budget) overrides the draft source (tests feed adversarial drafts).
    correct_hist > 0 runs the correct stage on every draft block with that many historical vertices.
    sampling = (temperature, seed) switches from greedy decoding to sampled decoding with non-greedy verification."""
    budget = 9 * faces
    st = SeqState(model, mem, budget)
    while not st.finished and st.P < budget:
        if not speculative:
            block, merged = [st.main], []
        elif draft_fn is not None:
            block = draft_fn(st, budget)
            merged = [None] * (len(block) - 1)
        else:
            merged = []
            block = draft(model, st, budget, merged, sampling, seq)
        if speculative and correct_hist > 0:
            fixed = corrected(model, st, block, correct_hist)
            merged = [m if fixed[i + 1] == block[i + 1] else None for i, m in enumerate(merged)]
            block = fixed
        if sampling is None:
            _, y, a = verify(model, st, block)
        else:
            _, y, a = verify_sampled(model, st, block, merged, sampling, seq)
        a = commit(model, st, block, y, a)
        if trace is not None:
            trace.append((st.P - a, list(block), a))
    return st.tokens[1:] + [st.main], st
