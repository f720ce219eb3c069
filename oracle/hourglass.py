"""TEST INFRASTRUCTURE ONLY - plain CPU hourglass transformer over mesh coordinate tokens.

Two definitions of the backbone forward (Supp. "Hourglass Transformer"; block
structure from Sec. 3.1 "Speculative Prediction Block"):

* forward_full   - the whole token sequence at once, written level by level with
                   no cache: the plain definition.
* forward_block  - a block of B new positions against per-layer K/V caches at
                   all three levels (what one verify pass computes, Sec. 3.3).

Alignment (a reading; the paper gives prose only): the sequence is x_0 = BOS
followed by 9 coordinate tokens per face.  Input position n predicts x_{n+1}.
Vertex token j is W_s * mean(h[3j-2], h[3j-1], h[3j]) (missing rows are zero,
always divided by 3) and is upsampled onto input positions 3j, 3j+1, 3j+2; face
token f pools vertex tokens 3f-2..3f and is upsampled onto vertex tokens
3f..3f+2.  Upsampling is repeat plus the skip connection from before the
shortening.  Everything is causal.

Sliding window (Sec. 5.1 names a window size of 18K / 36K tokens and nothing
else; a reading): with cfg.window = W > 0 a self-attention row at position p of
the coordinate level sees keys [p - W + 1, p]; the vertex and face levels use
W/3 and W/9 of their own positions, i.e. the same span of the mesh.  Rotary
positions stay absolute; cross-attention to the condition is not windowed.
The oracle keeps every key and masks, which is the definition; a ring buffer is
an implementation of it.

bf16 configurations: the weights arrive already rounded to bf16 values and all
arithmetic on them is done in the working precision (float64 by default) with
no further rounding: the oracle is the exact forward function of the
bf16-valued parameters.  `act_round=True` additionally rounds every GEMM
input, q/k/v and the condition memory to bf16, which is only used to study how
reduced-precision activations perturb the logits.
"""
from __future__ import annotations

import numpy as np

from . import primitives as P

STACKS = ("cpre", "vpre", "face", "vpost", "cpost")
LEVEL_OF = {"cpre": "c", "cpost": "c", "vpre": "v", "vpost": "v", "face": "f"}


class Model:
    """Holds the parameters (cast to the working precision) and the hyper-parameters."""

    def __init__(self, cfg, weights: dict, work=np.float64, act_round=False):
        self.cfg = cfg
        self.work = work
        self.w = {k: np.asarray(v, dtype=work) for k, v in weights.items()}
        self.d = cfg.d_model
        self.H = cfg.n_heads
        self.layers = {"cpre": cfg.l_cpre, "vpre": cfg.l_vpre, "face": cfg.l_face,
                       "vpost": cfg.l_vpost, "cpost": cfg.l_cpost}
        if cfg.dtype == "bf16" and act_round:
            self.rnd = P.bf16_round
        else:
            self.rnd = lambda x: x

    # -- pieces of one transformer block ------------------------------------------------
    def lin(self, x, name):
        return x @ self.w[name].T

    def heads(self, x):
        return x.reshape(x.shape[0], self.H, self.d // self.H)

    def qkv(self, pfx, h, pos):
        """Pre-norm, projections and rotary position for self-attention."""
        cfg, rnd = self.cfg, self.rnd
        x = rnd(P.rmsnorm(h, self.w[pfx + "g1"], cfg.rms_eps))
        q = rnd(P.rope(self.heads(self.lin(x, pfx + "wq")), pos, cfg.rope_base))
        k = rnd(P.rope(self.heads(self.lin(x, pfx + "wk")), pos, cfg.rope_base))
        v = rnd(self.heads(self.lin(x, pfx + "wv")))
        return q, k, v

    def mem_kv(self, pfx, mem):
        """Keys/values of the condition memory for one layer (no norm, no rotary on the memory side)."""
        m = self.rnd(np.asarray(mem, dtype=self.work))
        return self.rnd(self.heads(self.lin(m, pfx + "ck"))), self.rnd(self.heads(self.lin(m, pfx + "cv")))

    def after_self_attention(self, pfx, h, o, Kmem, Vmem):
        """Output projection + residual, cross-attention sub-layer, feed-forward sub-layer."""
        cfg, rnd = self.cfg, self.rnd
        rows = h.shape[0]
        h = h + self.lin(rnd(o.reshape(rows, self.d)), pfx + "wo")
        x = rnd(P.rmsnorm(h, self.w[pfx + "g2"], cfg.rms_eps))
        q = rnd(self.heads(self.lin(x, pfx + "cq")))
        o = P.attend(q, Kmem, Vmem, np.full(rows, Kmem.shape[0] - 1))
        h = h + self.lin(rnd(o.reshape(rows, self.d)), pfx + "co")
        x = rnd(P.rmsnorm(h, self.w[pfx + "g3"], cfg.rms_eps))
        h = h + self.lin(rnd(P.gelu_tanh(self.lin(x, pfx + "w1"))), pfx + "w2")
        return h

    def logits(self, h):
        x = self.rnd(P.rmsnorm(h, self.w["gf"], self.cfg.rms_eps))
        return self.lin(x, "lm")

    def embed(self, tokens):
        return self.w["emb"][np.asarray(tokens, dtype=np.int64)]


# ---------------------------------------------------------------------------------------
# Plain definition: the whole sequence at once
# ---------------------------------------------------------------------------------------
def shorten(h, W, rnd=lambda x: x):
    """Coarse token j = W * mean(h[3j-2], h[3j-1], h[3j]); rows before the start count as zero."""
    T = h.shape[0]
    n = (T - 1) // 3 + 1 if T else 0
    hp = np.concatenate([np.zeros((2, h.shape[1]), h.dtype), h], axis=0)  # hp[i + 2] = h[i]
    pooled = np.stack([(hp[3 * j] + hp[3 * j + 1] + hp[3 * j + 2]) / 3.0 for j in range(n)]) if n else h[:0]
    return rnd(pooled) @ W.T


def upsample(h_skip, y_coarse):
    """Fine row i = skip row i + coarse row floor(i/3)."""
    idx = np.arange(h_skip.shape[0]) // 3
    return h_skip + y_coarse[idx]


def forward_full(model: Model, tokens, mem, taps=None):
    """Logits for every position of `tokens` (x_0 = BOS first), no cache.

    If `taps` is a dict it receives the inputs of the last layer of the coordinate
    post stack, vertex post stack and face stack, and the level outputs."""
    m = model
    mem_cache = {}

    def run_stack(st, h):
        pos = np.arange(h.shape[0])
        for i in range(m.layers[st]):
            pfx = f"{st}.{i}."
            if taps is not None and i == m.layers[st] - 1 and st in ("cpost", "vpost", "face"):
                taps["tap_" + LEVEL_OF[st]] = h.copy()
            q, k, v = m.qkv(pfx, h, pos)
            o = P.attend_causal(q, k, v, 0, m.cfg.level_window(LEVEL_OF[st]))
            if pfx not in mem_cache:
                mem_cache[pfx] = m.mem_kv(pfx, mem)
            h = m.after_self_attention(pfx, h, o, *mem_cache[pfx])
        return h

    h_c = run_stack("cpre", m.embed(tokens))
    h_v = run_stack("vpre", shorten(h_c, m.w["short_cv"], m.rnd))
    y_f = run_stack("face", shorten(h_v, m.w["short_vf"], m.rnd))
    y_v = run_stack("vpost", upsample(h_v, y_f))
    y_c = run_stack("cpost", upsample(h_c, y_v))
    if taps is not None:
        taps.update(y_f=y_f, y_v=y_v, y_c=y_c, h_c=h_c, h_v=h_v)
    return m.logits(y_c)


# ---------------------------------------------------------------------------------------
# Incremental definition: a block of new positions against the caches
# ---------------------------------------------------------------------------------------
class SeqState:
    """Everything one sequence carries between verify passes.

    P positions are committed.  Arrays are indexed by absolute level-local position and
    hold valid data below the committed lengths (Lc = P, Lv = ceil(P/3), Lf = ceil(P/9));
    rows at or above them are scratch that the next pass overwrites."""

    def __init__(self, model: Model, mem, cap_tokens: int):
        m = model
        self.cap = cap_c = cap_tokens
        cap_v = (cap_c + 2) // 3 + 1
        cap_f = (cap_c + 8) // 9 + 1
        self.caps = {"c": cap_c, "v": cap_v, "f": cap_f}
        self.P = 0
        self.main = m.cfg.bos                 # pending main token x_P (x_0 = BOS)
        self.tokens = []                      # committed x_0 .. x_{P-1}
        self.finished = False
        z = lambda n, *s: np.zeros((n,) + s, m.work)
        self.K, self.V, self.Kmem, self.Vmem = {}, {}, {}, {}
        for st in STACKS:
            cap = self.caps[LEVEL_OF[st]]
            for i in range(m.layers[st]):
                pfx = f"{st}.{i}."
                self.K[pfx] = z(cap, m.H, m.d // m.H)
                self.V[pfx] = z(cap, m.H, m.d // m.H)
                self.Kmem[pfx], self.Vmem[pfx] = m.mem_kv(pfx, mem)
        self.h_c = z(cap_c, m.d)   # coordinate pre-stack outputs (pool input, skip)
        self.h_v = z(cap_v, m.d)   # vertex pre-stack outputs
        self.y_f = z(cap_f, m.d)   # face-level outputs
        self.y_v = z(cap_v, m.d)   # vertex-level outputs
        self.tap = {"c": z(cap_c, m.d), "v": z(cap_v, m.d), "f": z(cap_f, m.d)}
        # draft bookkeeping (used by oracle.speculative)
        self.rows = {"c": {}, "v": {}, "f": {}}
        self.labels = {"v": {}, "f": {}}      # label distributions per vertex (oracle.correct)
        self.fired_v = -1
        self.fired_f = -1

    @staticmethod
    def level_lengths(Pc: int):
        """Committed lengths at the three levels for Pc committed coordinate positions."""
        return Pc, (Pc + 2) // 3, (Pc + 8) // 9


def forward_block(model: Model, st: SeqState, tokens, long_block=False):
    """Logits [B, V] for tokens placed at positions P .. P+B-1; writes (does not commit) the caches."""
    m = model
    Pc = st.P
    B = len(tokens)
    assert B >= 1 and Pc + B <= st.cap

    def run_stack(stack, h, first):
        lvl = LEVEL_OF[stack]
        rows = h.shape[0]
        pos = first + np.arange(rows)
        for i in range(m.layers[stack]):
            pfx = f"{stack}.{i}."
            if i == m.layers[stack] - 1 and stack in ("cpost", "vpost", "face"):
                st.tap[lvl][pos] = h
            q, k, v = m.qkv(pfx, h, pos)
            st.K[pfx][pos] = k
            st.V[pfx][pos] = v
            win = m.cfg.level_window(lvl)
            if long_block:
                o = P.attend_causal(q, st.K[pfx], st.V[pfx], first, win)
            else:
                o = P.attend(q, st.K[pfx], st.V[pfx], pos, win)
            h = m.after_self_attention(pfx, h, o, st.Kmem[pfx], st.Vmem[pfx])
        return h

    def pool(src, first_new, n_new, W):
        """Coarse rows first_new .. first_new+n_new-1 from fine rows held in `src`."""
        out = np.zeros((n_new, m.d), m.work)
        for r in range(n_new):
            j = first_new + r
            acc = np.zeros(m.d, m.work)
            for i in (3 * j - 2, 3 * j - 1, 3 * j):
                if i >= 0:
                    acc = acc + src[i]
            out[r] = acc / 3.0
        return m.rnd(out) @ W.T

    pos_c = Pc + np.arange(B)
    h = run_stack("cpre", m.embed(tokens), Pc)
    st.h_c[pos_c] = h

    # vertex rows: one per block position that is a multiple of 3
    v0 = (Pc + 2) // 3
    nv = (Pc + B - 1) // 3 + 1 - v0
    f0 = (v0 + 2) // 3
    nf = (v0 + nv - 1) // 3 + 1 - f0 if nv > 0 else 0
    if nv > 0:
        hv = run_stack("vpre", pool(st.h_c, v0, nv, m.w["short_cv"]), v0)
        st.h_v[v0:v0 + nv] = hv
        if nf > 0:
            st.y_f[f0:f0 + nf] = run_stack("face", pool(st.h_v, f0, nf, m.w["short_vf"]), f0)
        vidx = v0 + np.arange(nv)
        st.y_v[vidx] = run_stack("vpost", st.h_v[vidx] + st.y_f[vidx // 3], v0)
    y_c = run_stack("cpost", st.h_c[pos_c] + st.y_v[pos_c // 3], Pc)
    return m.logits(y_c)
