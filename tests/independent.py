"""Independent little programs the oracle is pinned against.  None of them
uses Eq. 3-7: they are path enumeration, the transducer forward recursion and a
frame-by-frame beam search, written directly from their definitions."""

from __future__ import annotations

import math
from collections import defaultdict

import numpy as np


def softmax_np(v):
    v = np.asarray(v, dtype=np.float64)
    e = np.exp(v - v.max())
    return e / e.sum()


class Lattice:
    """J(t, tokens) of a toy transducer given by logits_fn(frame, tokens)."""

    def __init__(self, logits_fn, vocab, blank=0):
        self.fn, self.V, self.blank = logits_fn, vocab, blank
        self.cache = {}

    def J(self, t, y):
        key = (t, y)
        if key not in self.cache:
            self.cache[key] = softmax_np(self.fn(t, y))
        return self.cache[key]


def enumerate_paths(lat: Lattice, T: int, S: int, max_emit_per_segment: int):
    """Sum of alignment probabilities per token tuple, by walking every path of
    the transducer lattice: at (t, y) a blank moves to (t+1, y), a token k stays
    at t with y+k.  A path may emit at most max_emit_per_segment tokens inside
    any one segment of S frames.  Returns {tokens: probability}."""
    out = defaultdict(float)

    def walk(t, y, prob, emitted):
        if t == T:
            out[y] += prob
            return
        j = lat.J(t, y)
        nxt = t + 1
        walk(nxt, y, prob * j[lat.blank], 0 if nxt % S == 0 else emitted)
        if emitted < max_emit_per_segment:
            for k in range(lat.V):
                if k != lat.blank:
                    walk(t, y + (k,), prob * j[k], emitted + 1)

    walk(0, (), 1.0, 0)
    return dict(out)


def last_emission_profile(lat: Lattice, S: int, max_emit: int):
    """Within the first segment of S frames: for every non-empty token tuple
    y, the probability of the paths that emit exactly y with the last token in
    frame t (0-based), not counting any blank after it.  Returns {y: [S]}."""
    out = defaultdict(lambda: np.zeros(S))

    def walk(t, y, prob):
        if t == S:
            return
        j = lat.J(t, y)
        walk(t + 1, y, prob * j[lat.blank])
        if len(y) < max_emit:
            for k in range(lat.V):
                if k != lat.blank:
                    y2 = y + (k,)
                    out[y2][t] += prob * j[k]
                    walk(t, y2, prob * j[k])

    walk(0, (), 1.0)
    return {k: v for k, v in out.items()}


def forward_probability(lat: Lattice, T: int, y: tuple) -> float:
    """Textbook transducer forward recursion (Graves 2012):
    alpha(t,u) = alpha(t-1,u) J(t-1,u,blank) + alpha(t,u-1) J(t,u-1,y_u);
    p(y|x) = alpha(T-1,U) J(T-1,U,blank) with 0-based frames."""
    U = len(y)
    alpha = np.zeros((T, U + 1))
    alpha[0, 0] = 1.0
    for t in range(T):
        for u in range(U + 1):
            if t == 0 and u == 0:
                continue
            a = 0.0
            if t > 0:
                a += alpha[t - 1, u] * lat.J(t - 1, y[:u])[lat.blank]
            if u > 0:
                a += alpha[t, u - 1] * lat.J(t, y[:u - 1])[y[u - 1]]
            alpha[t, u] = a
    return alpha[T - 1, U] * lat.J(T - 1, y)[lat.blank]


def framewise_beam_search(lat: Lattice, T: int, N: int):
    """Breadth-first frame-by-frame transducer beam search (Eq. 1 and the
    paragraph after it): per frame, hypotheses are extended by blank (done with
    the frame, merged by token sequence) or by a token (stay in the frame); the
    N best token extensions survive if the finished list is still short of N
    or they beat its N-th score.  Probabilities kept as plain floats."""
    done = [((), 1.0)]
    for t in range(T):
        done.sort(key=lambda h: -h[1])
        active = done[:N]
        done = []
        while active:
            ext = []
            for hi, (y, p) in enumerate(active):
                j = lat.J(t, y)
                pb = p * j[lat.blank]
                for i, (y2, p2) in enumerate(done):
                    if y2 == y:
                        done[i] = (y2, p2 + pb)
                        break
                else:
                    done.append((y, pb))
                for k in range(lat.V):
                    if k != lat.blank:
                        ext.append((p * j[k], hi, k))
            ext.sort(key=lambda e: (-e[0], e[1], e[2]))
            nth = sorted((p for _, p in done), reverse=True)[N - 1] if len(done) >= N else None
            nxt = []
            for p, hi, k in ext[:N]:
                if nth is None or p > nth:
                    nxt.append((active[hi][0] + (k,), p))
            active = nxt
    done.sort(key=lambda h: -h[1])
    return done[:N]


def alpha_scan(b, d_old):
    """Forward variable over one segment for one hypothesis:
    alpha[0] = d_old[0]; alpha[t] = alpha[t-1]*b[t-1] + d_old[t].
    Returns (alpha [S], delta_blank)."""
    S = len(b)
    alpha = np.zeros(S)
    alpha[0] = d_old[0]
    for t in range(1, S):
        alpha[t] = alpha[t - 1] * b[t - 1] + d_old[t]
    return alpha, alpha[S - 1] * b[S - 1]
