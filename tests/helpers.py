"""Shared set-up for the GPU parity tests: seeded inputs, the oracle on them and
the HIP context on them.  The two sides meet only here, through tbs_inputs."""

from __future__ import annotations

import numpy as np

import oracle
from tbs_inputs import TbsShape, SHAPES, make_model, make_utterances


def small_bf16_shape(n_utts=3, vocab=96, d=64, hidden=64, layers=1, name="small"):
    return TbsShape(name, 7, n_utts, 5, 23, d, d, vocab, 0, layers, hidden, hidden, "bf16")


def build_case(shape: TbsShape, n_utts=None, lengths=None):
    model = make_model(shape)
    offsets, enc = make_utterances(shape, model, n_utts=n_utts, lengths=lengths)
    return model, offsets, enc


def oracle_weights(shape: TbsShape, model):
    return oracle.LstmWeights(model, shape.blank_id, act=shape.act, quant_bf16=(shape.dtype == "bf16"))


def make_tbs(shape: TbsShape, model, offsets, N, S, **kw):
    from paper_2302_14357_amd import Tbs
    U = len(offsets) - 1
    return Tbs(model, blank_id=shape.blank_id, beam_n=N, seg_s=S, max_utts=kw.pop("max_utts", U),
               max_frames_total=kw.pop("max_frames_total", int(offsets[-1])), dtype=shape.dtype, act=shape.act,
               **kw)


def compare_nbest(gpu, ref, score_tol=2e-3, gap_tol=1e-3):
    """Per-utterance comparison under the gap rule: where every decision of
    the oracle had a score gap above gap_tol the token sequences and their order
    must be identical and total log scores within score_tol (absolute; the
    total is a sum of hundreds of per-round terms each good to ~1e-6); elsewhere a mismatch is counted,
    not failed.  Returns (identical, ambiguous_mismatch, total)."""
    same = amb = 0
    for u, (g, r) in enumerate(zip(gpu, ref)):
        gt = [y for y, _ in g]
        rt = [y for y, _ in r.nbest]
        if gt == rt:
            gs = np.array([s for _, s in g])
            rs = np.array([s for _, s in r.nbest])
            assert np.all(np.abs(gs - rs) <= score_tol), (u, gs, rs)
            same += 1
        else:
            assert r.min_gap <= gap_tol, f"utterance {u}: N-best differ although the smallest gap is {r.min_gap}"
            amb += 1
    return same, amb, len(ref)
