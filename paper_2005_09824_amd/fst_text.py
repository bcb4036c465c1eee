"""Reader of graphs in the OpenFst text format, into the arc-list dictionaries the
binding takes (Section 3.3: a graph is its transitions (from, to, pdf, weight)
plus initial and final probabilities).

Host-side parsing only; nothing of the method's arithmetic lives here.

Format, one item per line, fields separated by blanks:
    src dst ilabel [olabel] [cost]     an arc (cost = -log weight, default 0)
    state [cost]                       a final state
The start state is the source of the first arc line, as OpenFst defines it.
"""
from __future__ import annotations

import math

import numpy as np


def read_fst_text(lines, num_pdfs=None, label_offset=1, acceptor=False):
    """lines: an iterable of text lines (an open file works).

    ilabel - label_offset is the arc's pdf-id (Kaldi's graphs number pdfs from 1 and
    keep 0 for epsilon, which a chain graph must not contain). With acceptor=True a
    line `src dst label cost` has no olabel column. num_pdfs defaults to the largest
    pdf-id + 1. Returns a dict with num_states, num_pdfs, src, dst, pdf, logw,
    init_prob (one-hot at the start state), final_prob (exp(-cost), 0 if not final).
    Raises ValueError on malformed lines, epsilon labels or infinite arc costs."""
    src, dst, pdf, logw = [], [], [], []
    finals = {}
    start = None
    for n, raw in enumerate(lines, 1):
        f = raw.split()
        if not f:
            continue
        try:
            if len(f) <= 2:  # final state
                s = int(f[0])
                cost = float(f[1]) if len(f) == 2 else 0.0
                if s < 0:
                    raise ValueError("negative state id")
                finals[s] = cost
                continue
            arc_cols = 3 if acceptor else 4
            if len(f) not in (arc_cols, arc_cols + 1):
                raise ValueError("expected %d or %d fields" % (arc_cols, arc_cols + 1))
            s, d, lab = int(f[0]), int(f[1]), int(f[2])
            if not acceptor:
                int(f[3])  # olabel: parsed for validity, unused
            cost = float(f[arc_cols]) if len(f) == arc_cols + 1 else 0.0
        except ValueError as e:
            raise ValueError("line %d: %s: %r" % (n, e, raw.rstrip("\n")))
        if s < 0 or d < 0:
            raise ValueError("line %d: negative state id" % n)
        if lab - label_offset < 0:
            raise ValueError("line %d: label %d is below the first pdf label %d (epsilon arcs "
                             "are not allowed)" % (n, lab, label_offset))
        if not math.isfinite(cost):
            raise ValueError("line %d: arc cost is not finite (leave the arc out)" % n)
        if start is None:
            start = s
        src.append(s); dst.append(d); pdf.append(lab - label_offset); logw.append(-cost)
    if start is None:
        raise ValueError("no arcs")
    S = max(max(src), max(dst), max(finals) if finals else 0) + 1
    P = max(pdf) + 1
    if num_pdfs is not None:
        if P > num_pdfs:
            raise ValueError("pdf-id %d does not fit num_pdfs = %d" % (P - 1, num_pdfs))
        P = int(num_pdfs)
    init = np.zeros(S, dtype=np.float32)
    init[start] = 1.0
    fin = np.zeros(S, dtype=np.float32)
    for s, cost in finals.items():
        fin[s] = math.exp(-cost) if math.isfinite(cost) else 0.0
    return {
        "num_states": S, "num_pdfs": P,
        "src": np.asarray(src, dtype=np.int32), "dst": np.asarray(dst, dtype=np.int32),
        "pdf": np.asarray(pdf, dtype=np.int32), "logw": np.asarray(logw, dtype=np.float32),
        "init_prob": init, "final_prob": fin,
    }


def write_fst_text(graph, label_offset=1):
    """The inverse, for graphs with a one-hot init_prob: a list of text lines."""
    init = np.asarray(graph["init_prob"])
    starts = np.flatnonzero(init > 0)
    if len(starts) != 1:
        raise ValueError("the text format has one start state")
    start = int(starts[0])
    order = sorted(range(len(graph["src"])), key=lambda a: (graph["src"][a] != start, a))
    if not order or graph["src"][order[0]] != start:
        raise ValueError("the start state has no outgoing arc")
    out = []
    for a in order:
        lab = int(graph["pdf"][a]) + label_offset
        out.append("%d %d %d %d %.9g" % (graph["src"][a], graph["dst"][a], lab, lab,
                                         -float(graph["logw"][a])))
    for s, p in enumerate(np.asarray(graph["final_prob"])):
        if p > 0:
            out.append("%d %.9g" % (s, -math.log(float(p))))
    return out
