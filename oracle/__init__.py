"""ctypes binding of the C oracle (oracle/tbs_oracle.c).

TEST INFRASTRUCTURE: a plain fp64 CPU implementation of token-wise RNN-T beam
search written from the paper.  Only tests/, the smoke check and the
benchmark's cpu_baseline leg may import this package; the HIP library and its
Python binding never do, and this package imports nothing of theirs.
"""

from __future__ import annotations

import ctypes as C
import math
import os
from dataclasses import dataclass, field

import numpy as np

from .build import build as _build, LIB as _LIB

_dp = C.POINTER(C.c_double)
_ip = C.POINTER(C.c_int)

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build(force=False)
        L = C.CDLL(path)
        L.orc_softmax.argtypes = [_dp, C.c_int, C.c_int, _dp]
        L.orc_blank_product.argtypes = [_dp, C.c_int, C.c_int, C.c_int, C.c_int, _dp]
        L.orc_nonblank_expansion_t.argtypes = [_dp, _dp, _dp, C.c_int, C.c_int, C.c_int, C.c_int, _dp]
        L.orc_nonblank_expansion.argtypes = [_dp, C.c_int, C.c_int, C.c_int, _dp]
        L.orc_blank_expansion.argtypes = [_dp, _dp, C.c_int, C.c_int, _dp]
        L.orc_round_bf16.argtypes = [C.c_double]
        L.orc_round_bf16.restype = C.c_double
        L.orc_set_mutant.argtypes = [C.c_int]
        L.orc_lstm_create.argtypes = [C.POINTER(_LstmWeightsC), _dp, C.c_int]
        L.orc_lstm_create.restype = C.c_void_p
        L.orc_lstm_destroy.argtypes = [C.c_void_p]
        L.orc_lstm_as_model.argtypes = [C.c_void_p, C.POINTER(_ModelC)]
        L.orc_lstm_init_state.argtypes = [C.c_void_p]
        L.orc_lstm_update_state.argtypes = [C.c_void_p, C.c_int, C.c_int]
        L.orc_lstm_joiner.argtypes = [C.c_void_p, C.c_int, C.c_int, _dp]
        L.orc_lstm_get_state.argtypes = [C.c_void_p, C.c_int, _dp, _dp, _dp]
        L.orc_lstm_joiner_vec.argtypes = [C.POINTER(_LstmWeightsC), _dp, _dp, _dp]
        L.orc_decode.argtypes = [C.POINTER(_ModelC), C.c_int, C.POINTER(_OptsC)]
        L.orc_decode.restype = C.c_void_p
        L.orc_result_free.argtypes = [C.c_void_p]
        L.orc_result_count.argtypes = [C.c_void_p]
        L.orc_result_len.argtypes = [C.c_void_p, C.c_int]
        L.orc_result_tokens.argtypes = [C.c_void_p, C.c_int]
        L.orc_result_tokens.restype = _ip
        L.orc_result_logscore.argtypes = [C.c_void_p, C.c_int]
        L.orc_result_logscore.restype = C.c_double
        L.orc_result_counters.argtypes = [C.c_void_p, C.POINTER(C.c_long), C.POINTER(C.c_long), C.POINTER(C.c_long)]
        L.orc_result_min_gap.argtypes = [C.c_void_p]
        L.orc_result_min_gap.restype = C.c_double
        L.orc_result_final_gap.argtypes = [C.c_void_p]
        L.orc_result_final_gap.restype = C.c_double
        L.orc_result_trace.argtypes = [C.c_void_p, C.POINTER(_ip), C.POINTER(C.c_long), C.POINTER(_dp), C.POINTER(C.c_long)]
        L.orc_result_trace.restype = C.c_long
        L.orc_decode_lstm_batch.argtypes = [C.POINTER(_LstmWeightsC), _dp, _ip, C.c_int, C.POINTER(_OptsC),
                                            C.c_int, C.POINTER(C.c_void_p)]
        L.orc_max_threads.restype = C.c_int
        _lib = L
    return _lib


_INIT = C.CFUNCTYPE(C.c_int, C.c_void_p)
_UPDATE = C.CFUNCTYPE(C.c_int, C.c_void_p, C.c_int, C.c_int)
_JOINER = C.CFUNCTYPE(None, C.c_void_p, C.c_int, C.c_int, _dp)


class _ModelC(C.Structure):
    _fields_ = [("user", C.c_void_p), ("vocab", C.c_int), ("blank_id", C.c_int),
                ("init_state", _INIT), ("update_state", _UPDATE), ("joiner", _JOINER)]


class _LstmWeightsC(C.Structure):
    _fields_ = [("d_joint", C.c_int), ("vocab", C.c_int), ("blank_id", C.c_int),
                ("embed_dim", C.c_int), ("hidden", C.c_int), ("layers", C.c_int),
                ("act", C.c_int), ("quant_bf16", C.c_int),
                ("w_out", _dp), ("b_out", _dp), ("embed", _dp),
                ("w_ih", _dp * 8), ("w_hh", _dp * 8), ("b", _dp * 8),
                ("w_proj", _dp), ("b_proj", _dp), ("pred_init", _dp)]


class _OptsC(C.Structure):
    _fields_ = [("beam_n", C.c_int), ("seg_s", C.c_int), ("max_rounds", C.c_int),
                ("raw_prob", C.c_int), ("trace", C.c_int)]


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _ptr(a):
    return a.ctypes.data_as(_dp)


# ---------------------------------------------------------------- algebra

def softmax(logits):
    l = _f64(logits)
    V = l.shape[-1]
    out = np.empty_like(l)
    lib().orc_softmax(_ptr(l), l.size // V, V, _ptr(out))
    return out


def blank_product(J, blank):
    J = _f64(J)
    H, S, V = J.shape
    Bl = np.empty((H, S + 1, S + 1))
    lib().orc_blank_product(_ptr(J), H, S, V, blank, _ptr(Bl))
    return Bl


def nonblank_expansion_t(J, Bl, d_old, blank):
    J, Bl, d_old = _f64(J), _f64(Bl), _f64(d_old)
    H, S, V = J.shape
    d = np.empty((H, V, S))
    lib().orc_nonblank_expansion_t(_ptr(J), _ptr(Bl), _ptr(d_old), H, S, V, blank, _ptr(d))
    return d


def nonblank_expansion(d):
    d = _f64(d)
    H, V, S = d.shape
    out = np.empty((H, V))
    lib().orc_nonblank_expansion(_ptr(d), H, S, V, _ptr(out))
    return out


def blank_expansion(Bl, d_old):
    Bl, d_old = _f64(Bl), _f64(d_old)
    H, S = d_old.shape
    out = np.empty(H)
    lib().orc_blank_expansion(_ptr(Bl), _ptr(d_old), H, S, _ptr(out))
    return out


def expansion_scores(logits, d_old, blank):
    """Softmax then Eq. 3-7 in the paper's order for logits [H,S,V], d_old [H,S].
    Returns (J, Bl, d, delta_nb, delta_blank)."""
    J = softmax(logits)
    Bl = blank_product(J, blank)
    d = nonblank_expansion_t(J, Bl, d_old, blank)
    return J, Bl, d, nonblank_expansion(d), blank_expansion(Bl, d_old)


def round_bf16(x):
    f = np.vectorize(lambda v: lib().orc_round_bf16(float(v)), otypes=[np.float64])
    return f(np.asarray(x, dtype=np.float64))


def set_mutant(m: int):
    lib().orc_set_mutant(int(m))


# ---------------------------------------------------------------- models

class TableModel:
    """A transducer given as a Python function logits_fn(frame, tokens) -> [V]."""

    def __init__(self, logits_fn, vocab, blank_id=0):
        self.logits_fn = logits_fn
        self.vocab = vocab
        self.blank_id = blank_id
        self.states = []
        self._init = _INIT(self._init_state)
        self._update = _UPDATE(self._update_state)
        self._joiner = _JOINER(self._joiner_fn)
        self.c = _ModelC(None, vocab, blank_id, self._init, self._update, self._joiner)

    def _init_state(self, _u):
        self.states.append(())
        return len(self.states) - 1

    def _update_state(self, _u, parent, tok):
        self.states.append(self.states[parent] + (int(tok),))
        return len(self.states) - 1

    def _joiner_fn(self, _u, frame, state, out):
        v = np.asarray(self.logits_fn(int(frame), self.states[state]), dtype=np.float64)
        for k in range(self.vocab):
            out[k] = v[k]


class LstmWeights:
    """float64 copies of a tbs_inputs model dict in the oracle's layout."""

    def __init__(self, model: dict, blank_id: int, act: str = "tanh", quant_bf16: bool = False):
        self.keep = []
        w = _LstmWeightsC()
        V, Dj = model["w_out"].shape
        w.d_joint, w.vocab, w.blank_id = Dj, V, blank_id
        w.embed_dim = model["embed"].shape[1]
        w.hidden = model["w_proj"].shape[1]
        w.layers = len(model["lstm"])
        w.act = {"tanh": 0, "relu": 1}[act]
        w.quant_bf16 = 1 if quant_bf16 else 0

        def put(a):
            a = _f64(a)
            self.keep.append(a)
            return _ptr(a)

        w.w_out, w.b_out, w.embed = put(model["w_out"]), put(model["b_out"]), put(model["embed"])
        for l, (wi, wh, b) in enumerate(model["lstm"]):
            w.w_ih[l], w.w_hh[l], w.b[l] = put(wi), put(wh), put(b)
        w.w_proj, w.b_proj, w.pred_init = put(model["w_proj"]), put(model["b_proj"]), put(model["pred_init"])
        self.c = w
        self.d_joint, self.vocab, self.hidden, self.layers = Dj, V, w.hidden, w.layers

    def joiner_vec(self, e, p):
        e, p = _f64(e), _f64(p)
        out = np.empty(self.vocab)
        lib().orc_lstm_joiner_vec(C.byref(self.c), _ptr(e), _ptr(p), _ptr(out))
        return out


class LstmModel:
    def __init__(self, weights: LstmWeights, enc):
        self.weights = weights
        self.enc = _f64(enc)
        self.T = self.enc.shape[0]
        self.h = lib().orc_lstm_create(C.byref(weights.c), _ptr(self.enc), self.T)
        self.c = _ModelC()
        lib().orc_lstm_as_model(self.h, C.byref(self.c))

    def __del__(self):
        if getattr(self, "h", None):
            lib().orc_lstm_destroy(self.h)
            self.h = None

    def init_state(self):
        return lib().orc_lstm_init_state(self.h)

    def update_state(self, parent, tok):
        return lib().orc_lstm_update_state(self.h, parent, tok)

    def joiner(self, frame, state):
        out = np.empty(self.weights.vocab)
        lib().orc_lstm_joiner(self.h, frame, state, _ptr(out))
        return out

    def get_state(self, state):
        w = self.weights
        p = np.empty(w.d_joint)
        h = np.empty((w.layers, w.hidden))
        c = np.empty((w.layers, w.hidden))
        lib().orc_lstm_get_state(self.h, state, _ptr(p), _ptr(h), _ptr(c))
        return p, h, c


# ---------------------------------------------------------------- decode

@dataclass
class Round:
    seg: int
    round: int
    S: int
    a_tokens: list          # incoming hypotheses
    a_scores: list
    delta_blank: list
    d_old: list
    b_tokens: list          # B after the merges
    b_scores: list
    threshold: float
    new_pairs: list         # (parent h, token)
    new_scores: list
    new_d: list
    head_gap: float = math.inf   # gap of the ChooseNBest(B) that opened the segment of this round
    gap: float = math.inf        # smallest gap of this round's own decisions


@dataclass
class Decoded:
    nbest: list             # [(tokens tuple, log score)]
    joiner_calls: int
    joined_frames: int
    frames: int
    min_gap: float
    final_gap: float = math.inf
    rounds: list = field(default_factory=list)

    def first_ambiguous_segment(self, tol: float):
        """Index of the first segment in which a decision (the ChooseNBest that opens it, or a
        round's top-N cut or threshold test) had a gap of at most tol; None if there is none.
        Needs a decode with trace=True."""
        for r in self.rounds:
            if r.head_gap <= tol or r.gap <= tol:
                return r.seg
        return None


def _collect(res_ptr, want_trace) -> Decoded:
    L = lib()
    n = L.orc_result_count(res_ptr)
    nbest = []
    for i in range(n):
        ln = L.orc_result_len(res_ptr, i)
        tp = L.orc_result_tokens(res_ptr, i)
        nbest.append((tuple(int(tp[j]) for j in range(ln)), float(L.orc_result_logscore(res_ptr, i))))
    a, b, c = C.c_long(), C.c_long(), C.c_long()
    L.orc_result_counters(res_ptr, C.byref(a), C.byref(b), C.byref(c))
    out = Decoded(nbest, a.value, b.value, c.value, float(L.orc_result_min_gap(res_ptr)),
                  float(L.orc_result_final_gap(res_ptr)))
    if want_trace:
        ip, dp_ = _ip(), _dp()
        ni, nd = C.c_long(), C.c_long()
        L.orc_result_trace(res_ptr, C.byref(ip), C.byref(ni), C.byref(dp_), C.byref(nd))
        it = np.ctypeslib.as_array(ip, shape=(ni.value,)).copy() if ni.value else np.zeros(0, np.int32)
        dt = np.ctypeslib.as_array(dp_, shape=(nd.value,)).copy() if nd.value else np.zeros(0)
        out.rounds = _parse_trace(it, dt)
    L.orc_result_free(res_ptr)
    return out


def _parse_trace(it, dt):
    rounds = []
    i = d = 0

    def toks():
        nonlocal i
        ln = int(it[i]); i += 1
        t = tuple(int(x) for x in it[i:i + ln]); i += ln
        return t

    while i < len(it):
        assert it[i] == -1
        seg, rnd, Sp, H, nB, nA = (int(x) for x in it[i + 1:i + 7])
        i += 7
        a_tokens = [toks() for _ in range(H)]
        b_tokens = [toks() for _ in range(nB)]
        pairs = [(int(it[i + 2 * j]), int(it[i + 2 * j + 1])) for j in range(nA)]
        i += 2 * nA
        a_scores, dphi, d_old = [], [], []
        for _ in range(H):
            a_scores.append(float(dt[d])); dphi.append(float(dt[d + 1]))
            d_old.append(dt[d + 2:d + 2 + Sp].copy()); d += 2 + Sp
        thr = float(dt[d]); d += 1
        b_scores = [float(x) for x in dt[d:d + nB]]; d += nB
        new_scores, new_d = [], []
        for _ in range(nA):
            new_scores.append(float(dt[d])); new_d.append(dt[d + 1:d + 1 + Sp].copy()); d += 1 + Sp
        head_gap, gap = float(dt[d]), float(dt[d + 1]); d += 2
        rounds.append(Round(seg, rnd, Sp, a_tokens, a_scores, dphi, d_old, b_tokens, b_scores, thr,
                            pairs, new_scores, new_d, head_gap, gap))
    assert d == len(dt)
    return rounds


def decode(model, T, N, S, max_rounds=0, raw_prob=False, trace=False) -> Decoded:
    """Algorithm 1 on one utterance of T frames.  model: TableModel or LstmModel."""
    o = _OptsC(N, S, max_rounds, 1 if raw_prob else 0, 1 if trace else 0)
    res = lib().orc_decode(C.byref(model.c), T, C.byref(o))
    return _collect(res, trace)


def decode_lstm_batch(weights: LstmWeights, enc, offsets, N, S, threads=1, max_rounds=0, trace=False):
    """Algorithm 1 on every utterance of a ragged batch; returns ([Decoded], threads used)."""
    enc = _f64(enc)
    offsets = np.ascontiguousarray(offsets, dtype=np.int32)
    U = len(offsets) - 1
    o = _OptsC(N, S, max_rounds, 0, 1 if trace else 0)
    res = (C.c_void_p * U)()
    used = lib().orc_decode_lstm_batch(C.byref(weights.c), _ptr(enc), offsets.ctypes.data_as(_ip), U,
                                       C.byref(o), int(threads), res)
    return [_collect(res[u], trace) for u in range(U)], used


def max_threads() -> int:
    return int(lib().orc_max_threads())
