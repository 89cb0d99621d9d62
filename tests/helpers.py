"""Shared set-up for the GPU parity tests: seeded inputs, the oracle on them and
the HIP context on them.  The two sides meet only here, through tbs_inputs.

How two decodes are compared.  Token-wise beam search is a pruned search: where two scores lie
closer than the arithmetic can tell apart, either outcome of a ranking or of the threshold test
is a correct run of Algorithm 1, and the two runs may then differ in everything that follows.
The oracle records the gap |log a - log b| of every such decision (the N-th against the (N+1)-th
entry wherever a list is cut to N, every expansion score against its threshold).  An utterance
whose smallest gap exceeds the tolerance has ONE correct N-best list and the HIP path must return
it; an utterance with a closer decision is decoded again on both sides up to the segment of its
first close decision, and there the results must again be identical.
"""

from __future__ import annotations

import math

import numpy as np

import oracle
from tbs_inputs import TbsShape, SHAPES, make_model, make_utterances


def small_bf16_shape(n_utts=3, vocab=96, d=64, hidden=64, layers=1, name="small", **kw):
    return TbsShape(name, 7, n_utts, 5, 23, d, d, vocab, 0, layers, hidden, hidden, "bf16", **kw)


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


def tolerance(shape: TbsShape, model: dict):
    """(gap and expansion-score tolerance, tolerance on a final log score).

    The stated bar is 1e-3 on scores relative to the hypothesis score for the bf16 joiner (1e-4 is
    used for fp32 models).  What differs between the two sides acts on the logits.  fp32
    accumulation order is ~1e-6 relative to the size of a logit.  For bf16 models the larger
    term is an activation that lands on the other side of a bf16 rounding boundary because its
    fp32 argument (a predictor output accumulated in fp32) differs in the last bits: that moves
    one activation by at most 2^-8 and so one logit by at most 2^-8 * max|W_out|, which is 2.4e-4
    for the benchmark models, inside the stated bar, and more for a test model whose output
    matrix is scaled up to make its distributions peaked.  The tolerance is therefore the stated
    bar or that bound (with a quarter added for the accumulation term), whichever is larger; fp32
    models scale the bar with logit_scale.  A final score is a sum of per-round terms: twice that."""
    if shape.dtype == "bf16":
        tol = max(1e-3, 1.25 * 2.0 ** -8 * float(np.abs(model["w_out"]).max()))
    else:
        tol = 1e-4 * max(1.0, shape.logit_scale)
    return tol, 2.0 * tol


def nbest_agrees(g, r, score_tol, gap_tol):
    """One utterance: the HIP N-best g = [(tokens, log score)] against the oracle's Decoded r.
    Unique content must be equal: the same set of token sequences (except entries that tie with the
    N-th place within gap_tol when the final cut itself was that close), scores within score_tol,
    and the HIP list in descending score order.  Returns None, or a string saying what differs."""
    gt = {y: s for y, s in g}
    rt = {y: s for y, s in r.nbest}
    if len(gt) != len(g):
        return "duplicate token sequences in the HIP result"
    gs = [s for _, s in g]
    if any(gs[i] < gs[i + 1] - 1e-12 for i in range(len(gs) - 1)):
        return f"HIP result not in descending score order: {gs}"
    if len(g) != len(r.nbest):
        return f"{len(g)} hypotheses, oracle has {len(r.nbest)}"
    s_last = r.nbest[-1][1] if r.nbest else 0.0
    close_cut = r.final_gap <= gap_tol
    for y, s in rt.items():
        if y in gt:
            if abs(gt[y] - s) > score_tol:
                return f"score of {y}: {gt[y]} vs oracle {s}"
        elif not (close_cut and s <= s_last + gap_tol):
            return f"oracle hypothesis {y} ({s}) missing"
    for y, s in gt.items():
        if y not in rt and not (close_cut and abs(s - s_last) <= 2 * gap_tol + score_tol):
            return f"HIP hypothesis {y} ({s}) not in the oracle's list"
    # order among common entries follows from equal scores and both lists being sorted, except for
    # entries closer than the tolerance, whose order is not unique
    return None


def compare_nbest(gpu, ref, score_tol=2e-3, gap_tol=1e-3):
    """All utterances of a batch.  Where every decision of the oracle had a gap above gap_tol
    (final cut aside, which nbest_agrees handles) the results must agree; elsewhere a difference
    is counted, not failed: strict_prefixes() then checks those up to their first close decision.
    Returns (identical, ambiguous_mismatch, total)."""
    same = amb = 0
    for u, (g, r) in enumerate(zip(gpu, ref)):
        why = nbest_agrees(g, r, score_tol, gap_tol)
        if why is None:
            same += 1
            continue
        inner_gap = min([min(x.head_gap, x.gap) for x in r.rounds], default=math.inf) if r.rounds else r.min_gap
        assert inner_gap <= gap_tol, f"utterance {u}: {why} (smallest decision gap {inner_gap:.3g} > {gap_tol:.3g})"
        amb += 1
    return same, amb, len(ref)


def strict_prefixes(ref, offsets, enc, S, gap_tol):
    """For a batch decoded by the oracle with trace=True: every utterance cut back to the whole
    segments before its first decision closer than gap_tol (utterances without one stay whole).
    Returns (offsets, enc, kept_frames [U]) of the shortened batch: decoded again, every decision
    is clear, so the two sides must agree on every utterance."""
    U = len(offsets) - 1
    keep = np.zeros(U, dtype=np.int64)
    for u in range(U):
        T = int(offsets[u + 1] - offsets[u])
        seg = ref[u].first_ambiguous_segment(gap_tol)
        keep[u] = T if seg is None else min(T, seg * S)
    off2 = np.concatenate([[0], np.cumsum(keep)]).astype(np.int32)
    parts = [enc[offsets[u]: offsets[u] + keep[u]] for u in range(U)]
    enc2 = np.concatenate(parts) if keep.sum() else np.zeros((0, enc.shape[1]), np.float32)
    return off2, enc2, keep


def assert_all_agree(gpu, ref, score_tol, gap_tol):
    """Every utterance must agree (used on batches whose decisions are all clear)."""
    for u, (g, r) in enumerate(zip(gpu, ref)):
        why = nbest_agrees(g, r, score_tol, gap_tol)
        assert why is None, f"utterance {u}: {why}"
