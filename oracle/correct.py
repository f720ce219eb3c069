"""TEST INFRASTRUCTURE ONLY - the correct stage of the predict-correct-verify step (Sec. 3.2,
"Correction Mechanism"), plain Python over integer bin coordinates.

The paper gives prose and one figure: a label head (a linear layer) on each point-level
feature sorts every generated point into historical / new / intra-batch; an intra-batch point
that overlaps no other vertex of the batch takes the coordinates of the nearest new point
outside its own triangle; the figure's second example moves a point onto a vertex of the
earlier faces; vertices are then re-sorted z-y-x; only draft tokens are touched.
Everything below that sentence level is a reading and is listed in the design notes:

* batch = the draft block of one step; its points = the vertices whose three coordinate
  tokens (order z, y, x) are all drafts of the block and all coordinate bins.  Vertex u owns
  the tokens x_{3u+1}, x_{3u+2}, x_{3u+3}; its face is u // 3.
* historical vertices = the last `hist_vertices` vertices whose tokens are all known
  (x_0 .. x_P, the main token included).
* label of a point = arg max (lowest index on ties) of the mean of the label distributions
  the point and face pipelines hold for it; a point that no pipeline covers counts as new.
* historical point: left alone if it equals a historical vertex, else moved onto the nearest
  one.  intra-batch point: left alone if it equals another point of the batch, else moved
  onto the nearest point labelled new in another face of the batch.  Nearest = smallest
  squared Euclidean distance in bins, lowest vertex index on ties; no candidate: left alone.
  Points are visited in ascending order and later points see earlier moves.
* re-sort: a face all of whose nine tokens are drafts has its three vertices put in
  ascending (z, y, x) order.
"""
from __future__ import annotations

import numpy as np

from . import primitives as P

HIST, NEW, INTRA = 0, 1, 2


def label_row(model, feature):
    """Label distribution of one point-level feature: softmax of the linear label head."""
    return P.softmax((model.w["label"] @ feature)[None, :])[0]


def point_labels(st, first_vertex: int, last_vertex: int):
    """Labels of the vertices first..last from the rows the point ("v") and face ("f") pipelines left in the state.

    Returns {vertex: (label, mean distribution or None)}."""
    out = {}
    for u in range(first_vertex, last_vertex + 1):
        rows = [st.labels[l][u] for l in ("v", "f") if u in st.labels[l]]
        if not rows:
            out[u] = (NEW, None)
            continue
        dist = sum(rows) / float(len(rows))
        out[u] = (int(np.argmax(dist)), dist)
    return out


def draft_vertex_range(Pc: int, block_len: int):
    """First and last vertex whose three tokens are all drafts of a block [x_P, x_{P+1}, ...] (last < first: none)."""
    return (Pc + 2) // 3, (Pc + block_len - 4) // 3


def _dist2(a, b) -> int:
    return sum((int(x) - int(y)) ** 2 for x, y in zip(a, b))


def correct_block(cfg, Pc: int, block, labels: dict, known, hist_vertices: int):
    """The corrected block.  block[0] = x_P (main), block[i] = draft of x_{P+i}; labels {vertex: HIST|NEW|INTRA};
    known = [x_0, ..., x_P]."""
    toks = [int(t) for t in block]
    u0, u1 = draft_vertex_range(Pc, len(toks))

    def get(u):
        i = 3 * u + 1 - Pc
        return tuple(toks[i:i + 3])

    def put(u, c):
        i = 3 * u + 1 - Pc
        toks[i:i + 3] = list(c)

    def is_point(c):
        return all(0 <= t < cfg.n_bins for t in c)

    n_known_vertices = Pc // 3
    hist = []
    for h in range(max(0, n_known_vertices - hist_vertices), n_known_vertices):
        c = tuple(int(t) for t in known[3 * h + 1:3 * h + 4])
        if is_point(c):
            hist.append((h, c))
    pts = [u for u in range(u0, u1 + 1) if is_point(get(u))]
    for u in pts:
        lab = labels.get(u, NEW)
        c = get(u)
        if lab == HIST:
            if hist and all(c != hc for _, hc in hist):
                put(u, min(hist, key=lambda e: (_dist2(c, e[1]), e[0]))[1])
        elif lab == INTRA:
            others = [w for w in pts if w != u]
            if all(get(w) != c for w in others):
                cand = [w for w in others if labels.get(w, NEW) == NEW and w // 3 != u // 3]
                if cand:
                    put(u, get(min(cand, key=lambda w: (_dist2(c, get(w)), w))))
    for f in range((u0 + 2) // 3, (u1 + 1) // 3):
        vs = [3 * f, 3 * f + 1, 3 * f + 2]
        if all(is_point(get(u)) for u in vs):
            for u, c in zip(vs, sorted(get(u) for u in vs)):
                put(u, c)
    return toks
