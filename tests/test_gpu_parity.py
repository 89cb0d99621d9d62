"""GPU parity: the HIP path through the C ABI against the CPU oracle, element
by element, on the same seeded inputs.

Tolerances.  Expansion scores: relative 1e-3 on scores
relative to the hypothesis score, i.e. |log gpu - log oracle| <= 1e-3, for
entries above 1e-30.  For bf16 models the oracle rounds act(e+p) and the
recurrent inputs to bf16 at the same points as the kernels; what remains is
fp32 accumulation order and exp/log/tanh rounding (~1e-6), plus rare bf16
rounding flips.  fp32 models: the same checks at 1e-4.  Integer results
(tokens, candidate sets, list sizes) must match exactly wherever the oracle's
own decision margin exceeds the tolerance.
"""

import math

import numpy as np
import pytest

import oracle
from tbs_inputs import SHAPES, TbsShape, make_model, make_utterances
from helpers import (build_case, oracle_weights, make_tbs, compare_nbest, small_bf16_shape, tolerance,
                     strict_prefixes, assert_all_agree, nbest_agrees)

pytestmark = pytest.mark.gpu


def _bf16_values(rng, shape, scale=1.0):
    import torch
    x = (rng.standard_normal(shape) * scale).astype(np.float32)
    return torch.from_numpy(x).to(torch.bfloat16)


# ------------------------------------------------------------------ the MFMA GEMM on its own

@pytest.mark.parametrize("kernel", [0, 1, 2, 3, 4])
@pytest.mark.parametrize("M,N,K", [(64, 64, 64), (200, 192, 128), (37, 100, 72), (1000, 1024, 512), (300, 2560, 640),
                                   (4100, 4096, 1024), (513, 257, 256)])
def test_gemm_bf16_tiles(M, N, K, kernel):
    """Every GEMM kernel (0 = the one the decode would pick; 64x64, 128x128, 256x256 tiles of the
    persistent kernel; the multi-stage kernel for small problems) on shapes with ragged edges."""
    import torch
    from paper_2302_14357_amd import gemm_bf16
    if kernel == 4 and K % 128:
        pytest.skip("the multi-stage kernel takes K in multiples of 128")
    rng = np.random.default_rng(M + N + K)
    a, b = _bf16_values(rng, (M, K)), _bf16_values(rng, (N, K), 0.1)
    bias = torch.from_numpy(rng.standard_normal(N).astype(np.float32))
    got = gemm_bf16(a.cuda(), b.cuda(), bias.cuda(), kernel=kernel).cpu().numpy()
    want = a.to(torch.float64).numpy() @ b.to(torch.float64).numpy().T + bias.numpy().astype(np.float64)
    np.testing.assert_allclose(got, want, rtol=1e-4, atol=1e-4 * math.sqrt(K))


# ------------------------------------------------------------------ joiner + expansion on chosen inputs

def _teacher_forced_state(rng, U, N, S, Dj):
    counts = rng.integers(0, N + 1, size=U).astype(np.int32)
    counts[0] = N
    if U > 1:
        counts[1] = 1
    pred = (rng.standard_normal((U, N, Dj)) * 0.5).astype(np.float32)
    dhat = rng.random((U, N, S)).astype(np.float32)
    dhat[rng.random((U, N, S)) < 0.35] = 0.0
    dhat[:, :, 0] += 0.05
    logs = -rng.random((U, N)) * 50.0
    return counts, pred, dhat, logs


_EXPAND_DEBUG = {"auto": 1, "generic": 3}   # tbs_config.debug: statistics kept + kernel choice


def _check_joiner_expand(shape, U, N, S, seg, sample_pairs=None, tol=1e-3, kernel="auto", flat=False, **kw):
    model, offsets, enc = build_case(shape, n_utts=U)
    if flat:   # every logit equal: every expansion ties, the smallest tokens must win
        model["w_out"] = np.zeros_like(model["w_out"])
        model["b_out"] = np.zeros_like(model["b_out"])
    W = oracle_weights(shape, model)
    tbs = make_tbs(shape, model, offsets, N, S, debug=_EXPAND_DEBUG[kernel], **kw)
    enc_dev = tbs.upload_frames(enc)
    rng = np.random.default_rng(11)
    counts, pred, dhat, logs = _teacher_forced_state(rng, U, N, S, shape.d_joint)
    tbs.begin(enc_dev, offsets)
    from paper_2302_14357_amd import BUF
    tbs.debug_write(BUF.A_COUNT, counts)
    tbs.debug_write(BUF.A_LOGS, logs)
    tbs.debug_write(BUF.A_PRED, pred)
    tbs.debug_write(BUF.A_DHAT, dhat)
    rows = tbs.debug_rebuild(seg)
    lens = np.diff(offsets)
    sp = np.clip(lens - seg * S, 0, S)
    assert rows == int(np.sum(np.where(sp > 0, counts, 0) * sp))
    np.testing.assert_array_equal(tbs.debug_read(BUF.A_PRED)[0, :N], pred[0, :N])
    tbs.joiner_segment()
    tbs.expand()
    pu, ph = tbs.debug_read(BUF.PAIR_UTT), tbs.debug_read(BUF.PAIR_HYP)
    row0, plen = tbs.debug_read(BUF.PAIR_ROW0), tbs.debug_read(BUF.PAIR_LEN)
    logits = tbs.debug_read(BUF.LOGITS)
    stats = tbs.debug_read(BUF.ROW_STATS)
    dphi = tbs.debug_read(BUF.DELTA_BLANK)
    dnb = tbs.debug_read(BUF.DELTA_NB)
    cs, ct = tbs.debug_read(BUF.CAND_SCORE), tbs.debug_read(BUF.CAND_TOKEN)
    pairs = len(pu)
    # pair list: utterances in order, hypotheses in order, finished utterances absent
    want_pairs = [(u, h) for u in range(U) if sp[u] > 0 for h in range(counts[u])]
    assert list(zip(pu.tolist(), ph.tolist())) == want_pairs
    which = range(pairs) if sample_pairs is None else rng.choice(pairs, size=min(sample_pairs, pairs), replace=False)
    worst = 0.0
    for j in which:
        u, h, r0, L = int(pu[j]), int(ph[j]), int(row0[j]), int(plen[j])
        assert L == sp[u]
        ref_logits = np.stack([W.joiner_vec(enc[offsets[u] + seg * S + t], pred[u, h]) for t in range(L)])
        np.testing.assert_allclose(logits[r0:r0 + L], ref_logits, rtol=0, atol=tol)
        d_old = dhat[u, h, :L].astype(np.float64)
        J, Bl, d, ref_nb, ref_phi = oracle.expansion_scores(ref_logits[None], d_old[None], shape.blank_id)
        np.testing.assert_allclose(stats[r0:r0 + L, 2], J[0, :, shape.blank_id], rtol=tol)
        assert abs(dphi[j] - math.log(ref_phi[0])) <= tol   # the kernel hands on log delta_blank
        ref_nb = ref_nb[0]
        big = ref_nb > 1e-30
        err = np.abs(np.log(dnb[j][big]) - np.log(ref_nb[big]))
        worst = max(worst, float(err.max()))
        assert err.max() <= tol
        assert dnb[j][shape.blank_id] == 0.0
        # the N best expansions of this hypothesis: same set wherever the margin is clear
        order = np.argsort(-ref_nb, kind="stable")
        n_take = min(N, shape.vocab - 1)
        margin = math.log(ref_nb[order[n_take - 1]]) - math.log(ref_nb[order[n_take]]) if n_take < shape.vocab - 1 else 1.0
        if margin > 2 * tol:
            assert set(ct[j][:n_take].tolist()) == set(order[:n_take].tolist())
        if flat:
            assert ct[j][:n_take].tolist() == list(range(1, n_take + 1))
        got_sorted = cs[j][:n_take]
        assert np.all(np.diff(got_sorted) <= 0)
        np.testing.assert_allclose(got_sorted, np.log(ref_nb[ct[j][:n_take]]), rtol=0, atol=tol)
    tbs.close()
    return worst


def test_joiner_expand_tiny_fp32():
    _check_joiner_expand(SHAPES["tiny"], U=1, N=2, S=3, seg=2, tol=1e-4)
    _check_joiner_expand(SHAPES["tiny"], U=1, N=2, S=3, seg=16, tol=1e-4)  # ragged last segment (2 frames)


@pytest.mark.parametrize("kernel", ["auto", "generic"])
@pytest.mark.parametrize("N,S", [(5, 3), (2, 1), (10, 5), (3, 50), (4, 12), (32, 2)])
def test_joiner_expand_small_bf16(N, S, kernel):
    """Both expansion kernels (the one that holds a hypothesis' logits in registers, which gives
    way to the other where S is beyond its range, and the two-pass kernel for any shape)."""
    shape = small_bf16_shape(n_utts=5, vocab=200, d=128, hidden=64)
    _check_joiner_expand(shape, U=5, N=N, S=S, seg=1 if S < 20 else 0, kernel=kernel)


@pytest.mark.parametrize("V,N,S", [(2048, 8, 7), (1028, 3, 2), (4096, 10, 5), (3000, 4, 3), (2000, 6, 5), (4096, 20, 3),
                                   (1024, 16, 4), (4096, 32, 2), (16000, 3, 2), (5001, 4, 3)])
def test_joiner_expand_wide_vocab(V, N, S):
    """Vocabulary widths that exercise every register-kernel instantiation and a ragged last column block."""
    shape = small_bf16_shape(n_utts=4, vocab=V, d=64, hidden=64)
    _check_joiner_expand(shape, U=4, N=N, S=S, seg=1, sample_pairs=6)


@pytest.mark.parametrize("kernel", ["auto", "generic"])
def test_expand_all_scores_equal(kernel):
    """Degenerate input: every expansion of a hypothesis has the same score (exercises the
    tie order and the selection path taken when too many candidates reach the threshold)."""
    shape = small_bf16_shape(n_utts=3, vocab=1024, d=64, hidden=64)
    _check_joiner_expand(shape, U=3, N=6, S=3, seg=0, kernel=kernel, flat=True)


def test_joiner_expand_odd_vocab():
    shape = small_bf16_shape(n_utts=3, vocab=77, d=64, hidden=64)
    _check_joiner_expand(shape, U=3, N=4, S=3, seg=0)


def test_joiner_expand_librispeech_full_size_sampled():
    """Headline configuration at full size (64 utterances, V=1024, Dj=512,
    N=5, S=3): sampled hypotheses against the oracle."""
    _check_joiner_expand(SHAPES["librispeech"], U=64, N=5, S=3, seg=10, sample_pairs=12)


def test_joiner_expand_assistant_full_width_sampled():
    """Large-assistant widths (V=4096, Dj=1024, N=10, S=3) with a multi-tile row count."""
    _check_joiner_expand(SHAPES["assistant"].with_utts(48), U=48, N=10, S=3, seg=5, sample_pairs=6)
    _check_joiner_expand(SHAPES["assistant"].with_utts(48), U=48, N=10, S=3, seg=5, sample_pairs=4, kernel="generic")


@pytest.mark.parametrize("kernel", ["auto", "generic"])
@pytest.mark.parametrize("N,S,chunk", [(5, 3, 16), (10, 5, 37), (3, 50, 60), (4, 12, 1), (6, 2, 7)])
def test_joiner_expand_in_pieces(N, S, chunk, kernel):
    """A joiner call run in pieces (input rows, GEMM and expansion of some hypotheses, then of the
    next): piece sizes that are no multiple of the segment size, ragged last segments, a piece of a
    single hypothesis, finished utterances in the batch."""
    shape = small_bf16_shape(n_utts=5, vocab=200, d=128, hidden=64)
    _check_joiner_expand(shape, U=5, N=N, S=S, seg=1 if S < 20 else 0, kernel=kernel, joiner_chunk_rows=chunk)


def test_joiner_expand_throughput_shape_in_pieces():
    """The largest configuration's widths with ~8000 rows in two pieces of 6144 rows at most: each
    piece runs on the 256x256-tile persistent GEMM over a row range read from device memory."""
    import dataclasses
    shape = dataclasses.replace(SHAPES["throughput"], n_utts=320, len_lo=25, len_hi=25)
    _check_joiner_expand(shape, U=320, N=10, S=5, seg=3, sample_pairs=10, joiner_chunk_rows=6144)


def test_joiner_expand_throughput_shape_sampled():
    """The largest configuration's widths (Dj=1024, V=4096, N=10, S=5) with enough rows (320
    utterances, ~8000 rows) that the joiner runs on the 256x256-tile persistent GEMM and the
    expansion on the 80-logits-per-thread kernel: the two kernels the at-scale roofline figures
    are measured on, sampled hypotheses against the oracle."""
    import dataclasses
    shape = dataclasses.replace(SHAPES["throughput"], n_utts=320, len_lo=25, len_hi=25)
    _check_joiner_expand(shape, U=320, N=10, S=5, seg=3, sample_pairs=8)


# ------------------------------------------------------------------ whole decode

def _oracle_decode(shape, model, offsets, enc, N, S, threads=16, **kw):
    W = oracle_weights(shape, model)
    kw.setdefault("trace", True)   # the per-round decision gaps decide how strictly results are compared
    res, _ = oracle.decode_lstm_batch(W, enc, offsets, N, S, threads=min(threads, oracle.max_threads()), **kw)
    return res


def _gpu_decode(shape, model, offsets, enc, N, S, **kw):
    tbs = make_tbs(shape, model, offsets, N, S, **kw)
    out = tbs.decode(tbs.upload_frames(enc), offsets)
    st = tbs.stats()
    st["path"] = tbs.path()
    tbs.close()
    return out, st


def _check_decode(shape, model, offsets, enc, N, S, max_rounds=0, report=None, **kw):
    """tbs_decode against the oracle under the gap rule, in two steps.  (1) The whole batch:
    utterances all of whose decisions were clear must agree.  (2) Every utterance cut back to the
    whole segments before its first close decision, decoded again by both sides: now every
    decision is clear, so every utterance must agree and the joiner-call counters must be equal.
    Returns a dict of what was seen (for assertions on coverage, e.g. hypothesis lengths)."""
    tol, score_tol = tolerance(shape, model)
    okw = dict(max_rounds=max_rounds) if max_rounds else {}
    gkw = dict(kw)
    if max_rounds:
        gkw["max_rounds_per_segment"] = max_rounds
    ref = _oracle_decode(shape, model, offsets, enc, N, S, **okw)
    U = len(offsets) - 1
    tbs = make_tbs(shape, model, offsets, N, S, **gkw)
    got = tbs.decode(tbs.upload_frames(enc), offsets)
    st = tbs.stats()
    same, amb, tot = compare_nbest(got, ref, score_tol=score_tol, gap_tol=tol)
    clear = [u for u in range(U) if ref[u].first_ambiguous_segment(tol) is None]
    info = {"same": same, "amb": amb, "tot": tot, "clear": len(clear),
            "max_len_checked": max([len(y) for u in clear for y, _ in ref[u].nbest], default=0)}
    if len(clear) == U:
        assert same == tot
        assert st["joiner_calls"] == sum(r.joiner_calls for r in ref)
        assert st["joined_frames"] == sum(r.joined_frames for r in ref)
    else:
        off2, enc2, keep = strict_prefixes(ref, offsets, enc, S, tol)
        ref2 = _oracle_decode(shape, model, off2, enc2, N, S, **okw)
        got2 = tbs.decode(tbs.upload_frames(enc2), off2)
        st2 = tbs.stats()
        assert_all_agree(got2, ref2, score_tol, tol)
        assert st2["joiner_calls"] == sum(r.joiner_calls for r in ref2)
        assert st2["joined_frames"] == sum(r.joined_frames for r in ref2)
        info["prefix_frames"] = int(keep.sum())
        info["max_len_checked"] = max(info["max_len_checked"],
                                      max([len(y) for r in ref2 for y, _ in r.nbest], default=0))
    tbs.close()
    if report:
        print(f"{report}: identical {same}/{tot}, differing after a close decision {amb}, "
              f"utterances with every decision clear {len(clear)}, "
              f"frames checked strictly {info.get('prefix_frames', int(offsets[-1]))}/{int(offsets[-1])}, "
              f"longest hypothesis checked {info['max_len_checked']}")
    return info


def test_decode_tiny_reference_config():
    shape = SHAPES["tiny"]
    model, offsets, enc = build_case(shape)
    info = _check_decode(shape, model, offsets, enc, 2, 3, report="tiny")
    assert info["tot"] == 1


@pytest.mark.parametrize("N,S", [(1, 1), (2, 2), (5, 3), (3, 7), (4, 30)])
def test_decode_small_bf16_and_edges(N, S):
    """Ragged batch with an empty utterance, one shorter than a segment and
    lengths that leave ragged last segments."""
    shape = small_bf16_shape(n_utts=6, vocab=64, d=64, hidden=64, layers=2)
    lengths = np.array([0, 1, 2, 7, 12, 23])
    model, offsets, enc = build_case(shape, n_utts=6, lengths=lengths)
    got, _ = _gpu_decode(shape, model, offsets, enc, N, S)
    assert got[0] == [((), 0.0)]
    _check_decode(shape, model, offsets, enc, N, S)


# ------------------------------------------------------------------ peaked models: long hypotheses

def _peaked(shape, scale, blank_bias):
    """A model with peaked output distributions (the output matrix scaled up, the blank bias with it):
    hypotheses then grow to many tokens, which the benchmark models' flat distributions never
    produce.  Such a model keeps emitting within a frame, so these runs cap the rounds of a
    segment on both sides (Section 3.2 mentions such a cap)."""
    import dataclasses
    return dataclasses.replace(shape, logit_scale=scale, blank_bias=blank_bias)


@pytest.mark.parametrize("dtype,N,S,cap,bb,min_len", [("f32", 5, 3, 8, 8.0, 5), ("bf16", 5, 3, 8, 8.0, 4),
                                                     ("bf16", 4, 2, 6, 12.0, 5), ("f32", 8, 5, 8, 12.0, 5),
                                                     ("bf16", 3, 1, 5, 10.0, 4)])
def test_decode_peaked_model_long_hypotheses(dtype, N, S, cap, bb, min_len):
    """Whole decodes whose N-best lists hold sequences of five and more tokens: deep walks of the
    token trie in AddAndMerge, hash-and-walk matches between long sequences, token read-out.
    (The list kernels are the same for both storage types; the fp32 models, whose tolerance is
    ten times tighter, are the ones that stay comparable over whole utterances; bf16 models meet a
    close decision sooner and are compared strictly on shorter prefixes.)"""
    import dataclasses
    shape = _peaked(dataclasses.replace(small_bf16_shape(n_utts=8, vocab=96, d=64, hidden=64), dtype=dtype), 8.0, bb)
    lengths = np.array([23, 17, 30, 9, 41, 26, 12, 35])
    model, offsets, enc = build_case(shape, n_utts=8, lengths=lengths)
    info = _check_decode(shape, model, offsets, enc, N, S, max_rounds=cap, report=f"peaked {dtype} N={N} S={S}")
    assert info["max_len_checked"] >= min_len, info


def test_decode_peaked_model_librispeech_widths():
    """The same at the headline widths (Dj=512, V=1024, LSTM 640, N=5, S=3)."""
    import dataclasses
    shape = _peaked(dataclasses.replace(SHAPES["librispeech"], n_utts=6), 16.0, 20.0)
    lengths = np.array([60, 90, 45, 33, 75, 52])
    model, offsets, enc = build_case(shape, n_utts=6, lengths=lengths)
    info = _check_decode(shape, model, offsets, enc, 5, 3, max_rounds=4, report="peaked, Librispeech widths")
    assert info["max_len_checked"] >= 5, info


def test_decode_truncation_and_capacity_codes():
    """Results longer than max_len come back truncated to their first max_len tokens, with their
    true lengths, and the call says TBS_EOVERFLOW; a list B or a token trie too small for the run
    is reported as the same code, not as a crash or a wrong result."""
    from paper_2302_14357_amd import TbsError
    shape = _peaked(small_bf16_shape(n_utts=3, vocab=96, d=64, hidden=64), 8.0, 8.0)
    lengths = np.array([23, 17, 30])
    model, offsets, enc = build_case(shape, n_utts=3, lengths=lengths)
    N, S, cap = 5, 3, 8
    tol, score_tol = tolerance(shape, model)
    ref = _oracle_decode(shape, model, offsets, enc, N, S, max_rounds=cap)
    longest = max(len(y) for r in ref for y, _ in r.nbest)
    assert longest >= 5
    tbs = make_tbs(shape, model, offsets, N, S, max_rounds_per_segment=cap)
    enc_dev = tbs.upload_frames(enc)
    full = tbs.decode(enc_dev, offsets)
    cut = 3
    tok = np.full((3, N, cut), -7, np.int32)
    lens = np.zeros((3, N), np.int32)
    logs = np.zeros((3, N), np.float64)
    cnt = np.zeros(3, np.int32)
    rc = tbs.decode_raw(enc_dev, offsets, tok, lens, logs, cnt, cut)
    assert rc == -5
    for u in range(3):
        assert cnt[u] == len(full[u])
        for i, (y, sc) in enumerate(full[u]):
            assert lens[u, i] == len(y) and logs[u, i] == sc
            assert tok[u, i, :min(cut, len(y))].tolist() == list(y[:cut])
            assert (tok[u, i, len(y):] == -1).all()
    with pytest.raises(TbsError) as e:
        tbs.result(max_len=257)          # beyond the configuration's max_result_len (256)
    assert e.value.code == -1
    tbs.close()
    # a trie with room for a handful of sequences only
    tbs = make_tbs(shape, model, offsets, N, S, max_rounds_per_segment=cap, max_nodes=40)
    with pytest.raises(TbsError) as e:
        tbs.decode(tbs.upload_frames(enc), offsets)
    assert e.value.code == -5
    tbs.close()
    # the same where every utterance takes nodes from a range of its own (width 128: the layout with
    # every hypothesis in a fixed place)
    shape128 = _peaked(small_bf16_shape(n_utts=3, vocab=96, d=128, hidden=128), 8.0, 8.0)
    model128, off128, enc128 = build_case(shape128, n_utts=3, lengths=lengths)
    tbs = make_tbs(shape128, model128, off128, N, S, max_rounds_per_segment=cap, max_nodes=40)
    with pytest.raises(TbsError) as e:
        tbs.decode(tbs.upload_frames(enc128), off128)
    assert e.value.code == -5
    tbs.close()
    # a list B smaller than a segment's blank expansions: the rounds of a segment are not capped,
    # the workspaces are sized for two
    tbs = make_tbs(shape, model, offsets, N, S, rounds_capacity=2)
    with pytest.raises(TbsError) as e:
        tbs.decode(tbs.upload_frames(enc), offsets)
    assert e.value.code == -5
    tbs.close()


def test_longest_list_b():
    """N * rounds capacity = 2048 entries of B per utterance, the most the library accepts."""
    shape = small_bf16_shape(n_utts=2, vocab=48, d=64, hidden=64)
    model, offsets, enc = build_case(shape, n_utts=2, lengths=np.array([9, 14]))
    _check_decode(shape, model, offsets, enc, 4, 3, rounds_capacity=512)
    from paper_2302_14357_amd import TbsError
    with pytest.raises(TbsError) as e:
        make_tbs(shape, model, offsets, 4, 3, rounds_capacity=513)
    assert e.value.code == -1


@pytest.mark.parametrize("debug", [0, 8, 32, 64, 8 + 16 + 32])
def test_decode_cell_update_inside_and_outside_the_gate_gemm(debug):
    """Two LSTM layers of 128 units: both layers fit the gate GEMM whose epilogue updates the cell
    (debug=0); debug=8 keeps the cell update a kernel of its own, 32 the gather of the first layer's
    input rows (otherwise part of the row list kernel), 64 the predictor step behind the host's wait
    for the counts (otherwise enqueued ahead of it), 56 every step that has a fused form.  All
    against the oracle."""
    shape = small_bf16_shape(n_utts=5, vocab=96, d=128, hidden=128, layers=2)
    lengths = np.array([4, 9, 15, 22, 31])
    model, offsets, enc = build_case(shape, n_utts=5, lengths=lengths)
    _check_decode(shape, model, offsets, enc, 4, 3, debug=debug)


@pytest.mark.parametrize("d,hidden,N,S", [(128, 128, 4, 3), (144, 128, 5, 7), (80, 256, 8, 2)])
def test_decode_joiner_rows_from_the_projection_epilogue(d, hidden, N, S):
    """Where the predictor projection is a small GEMM its epilogue also forms the joiner input rows
    of the coming round; debug=16 keeps them a kernel of their own.  Widths that leave a ragged
    column tile, segments longer than the epilogue's chunk of four frames, more pairs than one
    row tile.  The two variants do the same arithmetic: identical results, and both against the
    oracle."""
    shape = small_bf16_shape(n_utts=14, vocab=96, d=d, hidden=hidden, layers=1)
    lengths = np.array([0, 1, 3, 5, 8, 9, 11, 14, 15, 17, 20, 23, 26, 29])
    model, offsets, enc = build_case(shape, n_utts=14, lengths=lengths)
    got, st = _gpu_decode(shape, model, offsets, enc, N, S)
    own, st2 = _gpu_decode(shape, model, offsets, enc, N, S, debug=16)
    for a, b in zip(got, own):
        assert [h[0] for h in a] == [h[0] for h in b]
        np.testing.assert_allclose([h[1] for h in a], [h[1] for h in b], rtol=1e-6, atol=1e-6)
    assert st["joiner_calls"] == st2["joiner_calls"]
    _check_decode(shape, model, offsets, enc, N, S)
    _check_decode(shape, model, offsets, enc, N, S, debug=16)


@pytest.mark.parametrize("base,N,S", [("tiny", 2, 3), ("small64", 4, 3), ("small128", 5, 4)])
def test_decode_relu_joiner(base, N, S):
    """The joiner with a ReLU in place of tanh (the activation of the paper's Librispeech model,
    Section 4): fp32 model, bf16 model with the input rows from their own kernel (width 64) and
    from the projection's epilogue (width 128)."""
    import dataclasses
    if base == "tiny":
        shape, kw = dataclasses.replace(SHAPES["tiny"], act="relu"), {}
    else:
        w = int(base[5:])
        shape = dataclasses.replace(small_bf16_shape(n_utts=6, vocab=80, d=w, hidden=w), act="relu")
        kw = dict(n_utts=6, lengths=np.array([2, 5, 9, 14, 20, 27]))
    model, offsets, enc = build_case(shape, **kw)
    _check_decode(shape, model, offsets, enc, N, S)


# ------------------------------------------------------------------ streaming

def _push_in_pieces(tbs, shape, offsets, enc, piece_of, flush_last=True):
    """Feed every utterance its frames in pieces of piece_of(u, call) frames until all are in."""
    U = len(offsets) - 1
    T = np.diff(offsets)
    sent = np.zeros(U, dtype=np.int64)
    tbs.stream_begin(U)
    call = 0
    while (sent < T).any():
        n = np.array([min(int(piece_of(u, call)), int(T[u] - sent[u])) for u in range(U)])
        off = np.concatenate([[0], np.cumsum(n)]).astype(np.int32)
        rows = np.concatenate([enc[offsets[u] + sent[u]: offsets[u] + sent[u] + n[u]] for u in range(U)]) \
            if n.sum() else np.zeros((0, enc.shape[1]), np.float32)
        sent += n
        last = not (sent < T).any()
        tbs.push_segment(tbs.upload_frames(rows), off, flush=(last and flush_last))
        call += 1
    if T.sum() == 0:
        tbs.push_segment(None, np.zeros(U + 1, np.int32), flush=True)


@pytest.mark.parametrize("N,S,pieces", [(4, 3, "random"), (3, 4, "one"), (5, 3, "segment"), (2, 5, "uneven")])
def test_streaming_in_pieces_equals_decode(N, S, pieces):
    """Encoder frames arriving in pieces (frame by frame, in decoder-sized segments, in random
    sizes different per utterance, or some utterances much faster than others) and a flush at
    the end give what tbs_decode gives on the whole utterances (Section 3.2: the encoder's
    segment size need not be the decoder's): the segments of an utterance are the same either
    way, so the results are required to be identical; tbs_decode itself is checked against the
    oracle."""
    shape = small_bf16_shape(n_utts=7, vocab=64, d=128, hidden=128, layers=1)
    lengths = np.array([0, 1, 4, 9, 13, 22, 30])
    model, offsets, enc = build_case(shape, n_utts=7, lengths=lengths)
    rng = np.random.default_rng(5)
    draws = rng.integers(0, 2 * S + 2, size=(7, 200))
    piece_of = {"random": lambda u, c: draws[u, c], "one": lambda u, c: 1, "segment": lambda u, c: S,
                "uneven": lambda u, c: (u % 3) * 3 + 1}[pieces]
    whole, st0 = _gpu_decode(shape, model, offsets, enc, N, S)
    tbs = make_tbs(shape, model, offsets, N, S, stream_buffer_frames=3 * S + 2)
    _push_in_pieces(tbs, shape, offsets, enc, piece_of)
    got = tbs.result()
    st = tbs.stats()
    tbs.close()
    for a, b in zip(got, whole):
        assert [h[0] for h in a] == [h[0] for h in b]
        np.testing.assert_allclose([h[1] for h in a], [h[1] for h in b], rtol=1e-5, atol=1e-5)
    assert st["frames"] == int(lengths.sum()) and st["joined_frames"] == st0["joined_frames"]
    _check_decode(shape, model, offsets, enc, N, S)


def test_streaming_partial_results_and_limits():
    """Between pushes B holds the result for the frames decoded so far: with no flush, that is the
    decode of each utterance's whole segments.  A push beyond the buffer is refused and
    changes nothing; step calls and pushes do not mix."""
    from paper_2302_14357_amd.tbs import TbsError
    shape = small_bf16_shape(n_utts=3, vocab=48, d=64, hidden=64)
    N, S = 3, 4
    lengths = np.array([10, 17, 6])
    model, offsets, enc = build_case(shape, n_utts=3, lengths=lengths)
    tbs = make_tbs(shape, model, offsets, N, S, stream_buffer_frames=12)
    with pytest.raises(TbsError):
        tbs.push_segment(None, np.zeros(4, np.int32))          # no stream begun
    _push_in_pieces(tbs, shape, offsets, enc, lambda u, c: 5, flush_last=False)
    got = tbs.result()
    done = (lengths // S) * S
    off2 = np.concatenate([[0], np.cumsum(done)]).astype(np.int32)
    enc2 = np.concatenate([enc[offsets[u]: offsets[u] + done[u]] for u in range(3)])
    part, _ = _gpu_decode(shape, model, off2, enc2, N, S)
    for a, b in zip(got, part):
        assert [h[0] for h in a] == [h[0] for h in b]
        np.testing.assert_allclose([h[1] for h in a], [h[1] for h in b], rtol=1e-5, atol=1e-5)
    _check_decode(shape, model, off2, enc2, N, S)
    # 2, 1, 2 frames are still buffered; 11 more do not fit into 12
    with pytest.raises(TbsError):
        tbs.push_segment(tbs.upload_frames(np.zeros((11, 64), np.float32)), np.array([0, 11, 11, 11], np.int32))
    with pytest.raises(TbsError):
        tbs.segment_begin(0)
    assert tbs.result() == got
    # the rest of the stream still decodes: flush the leftovers
    tbs.push_segment(None, np.zeros(4, np.int32), flush=True)
    rest = tbs.result()
    tbs.close()
    whole, _ = _gpu_decode(shape, model, offsets, enc, N, S)
    for a, b in zip(rest, whole):
        assert [h[0] for h in a] == [h[0] for h in b]
        np.testing.assert_allclose([h[1] for h in a], [h[1] for h in b], rtol=1e-5, atol=1e-5)
    _check_decode(shape, model, offsets, enc, N, S)


def _step_by_step(shape, model, offsets, enc, N, S, max_rounds=0, **kw):
    """Drive the step entry points over a batch and compare A and B of every utterance with the
    oracle's trace after every round, up to the utterance's first close decision (from there on its
    run may legitimately differ and it is only followed).  Lists are compared as sets of token
    sequences with their scores: the order inside A changes no score.  Returns what was covered."""
    from paper_2302_14357_amd import BUF
    tol, score_tol = tolerance(shape, model)
    U = len(offsets) - 1
    T = np.diff(offsets)
    okw = dict(max_rounds=max_rounds) if max_rounds else {}
    ref = _oracle_decode(shape, model, offsets, enc, N, S, **okw)
    gkw = dict(kw)
    if max_rounds:
        gkw["max_rounds_per_segment"] = max_rounds
    tbs = make_tbs(shape, model, offsets, N, S, debug=1, **gkw)
    tbs.begin(tbs.upload_frames(enc), offsets)
    trace = [{(r.seg, r.round): r for r in ref[u].rounds} for u in range(U)]
    stop = [ref[u].first_ambiguous_segment(tol) for u in range(U)]
    cov = {"rounds": 0, "merges": 0, "max_len": 0, "deep_merges": 0}
    nseg = (int(T.max()) + S - 1) // S if U else 0
    for seg in range(nseg):
        rows = tbs.segment_begin(seg)
        rnd = 0
        prev_nb = [0] * U
        while rows > 0:
            rnd += 1
            a_now = tbs.debug_hyps(0)
            tbs.joiner_segment()
            tbs.expand()
            live = tbs.select_merge()
            b_now = tbs.debug_hyps(1, cap=N * (max_rounds or 32))
            a_new = tbs.debug_hyps(0)
            dh = tbs.debug_read(BUF.A_DHAT)
            for u in range(U):
                if stop[u] is not None and seg >= stop[u]:
                    continue
                r = trace[u].get((seg, rnd))
                if r is None:
                    assert a_now[u] == [] or seg * S >= T[u], (u, seg, rnd)
                    continue
                cov["rounds"] += 1
                assert {y for y, _ in a_now[u]} == set(r.a_tokens), (u, seg, rnd)
                want = dict(zip(r.a_tokens, r.a_scores))
                for y, sc in a_now[u]:
                    assert abs(sc - want[y]) <= score_tol, (u, seg, rnd, y)
                assert [y for y, _ in b_now[u]] == r.b_tokens, (u, seg, rnd)     # insertion order is unique
                np.testing.assert_allclose([sc for _, sc in b_now[u]], r.b_scores, atol=score_tol)
                new_tokens = [r.a_tokens[h] + (k,) for h, k in r.new_pairs]
                if max_rounds and rnd >= max_rounds:
                    new_tokens = []      # the round cap: what the last allowed round creates is dropped
                assert {y for y, _ in a_new[u]} == set(new_tokens), (u, seg, rnd)
                for i, (y, sc) in enumerate(a_new[u]):
                    j = new_tokens.index(y)
                    assert abs(sc - r.new_scores[j]) <= score_tol
                    np.testing.assert_allclose(dh[u, i, :r.S], r.new_d[j], rtol=10 * tol, atol=1e-7)
                merged = prev_nb[u] + len(r.a_tokens) - len(r.b_tokens)
                cov["merges"] += merged
                if merged:
                    cov["deep_merges"] += sum(1 for y in r.a_tokens if len(y) >= 3 and y in r.b_tokens[:prev_nb[u]])
                prev_nb[u] = len(r.b_tokens)
                cov["max_len"] = max([cov["max_len"]] + [len(y) for y in r.b_tokens])
            tbs.predictor_step()
            rows = tbs.counts()["rows"]
    final = tbs.result()
    for u in range(U):
        if stop[u] is None:
            why = nbest_agrees(final[u], ref[u], score_tol, tol)
            assert why is None, (u, why)
    tbs.close()
    return cov


def test_decode_step_by_step_matches_oracle_trace():
    """One utterance at the benchmark models' scale: A and B after every round."""
    shape = small_bf16_shape(n_utts=1, vocab=48, d=64, hidden=64)
    model, offsets, enc = build_case(shape, n_utts=1, lengths=np.array([38]))
    cov = _step_by_step(shape, model, offsets, enc, 3, 4)
    assert cov["merges"] > 0 and cov["rounds"] > 10, cov


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_step_by_step_peaked_batch(dtype):
    """A batch with a peaked model: A and B of every utterance after every round while the
    hypotheses grow long, including merges between sequences of three and more tokens (a sequence
    carried into a segment meeting the same sequence re-created in it)."""
    import dataclasses
    shape = _peaked(dataclasses.replace(small_bf16_shape(n_utts=5, vocab=12, d=64, hidden=64), dtype=dtype), 8.0, 8.0)
    lengths = np.array([30, 21, 38, 14, 26])
    model, offsets, enc = build_case(shape, n_utts=5, lengths=lengths)
    cov = _step_by_step(shape, model, offsets, enc, 5, 3, max_rounds=6)
    print(cov)
    assert cov["max_len"] >= 5, cov
    if dtype == "f32":   # (the tighter tolerance keeps these runs comparable to their ends)
        assert cov["deep_merges"] >= 10 and cov["max_len"] >= 10, cov


@pytest.mark.parametrize("d,limit", [(64, 2), (128, 2), (128, 1)])
def test_round_limit_matches_oracle(d, limit):
    """Hypotheses still emitting after `limit` rounds of a segment are dropped (Section 3.2 mentions
    such a limit).  Width 128 takes the path on which a segment's head and first round are enqueued
    in one go (with limit 1 the drop falls into that first round), width 64 the step-by-step one."""
    shape = small_bf16_shape(n_utts=2, vocab=32, d=d, hidden=d)
    model, offsets, enc = build_case(shape, n_utts=2, lengths=np.array([9, 6]))
    _check_decode(shape, model, offsets, enc, 4, 3, max_rounds=limit)


def test_batch_equals_each_alone_and_is_deterministic():
    shape = small_bf16_shape(n_utts=4, vocab=64, d=64, hidden=64)
    model, offsets, enc = build_case(shape, n_utts=4, lengths=np.array([11, 4, 17, 8]))
    together, _ = _gpu_decode(shape, model, offsets, enc, 3, 3)
    again, _ = _gpu_decode(shape, model, offsets, enc, 3, 3)
    assert together == again
    for u in range(4):
        o = np.array([0, offsets[u + 1] - offsets[u]], np.int32)
        alone, _ = _gpu_decode(shape, model, o, enc[offsets[u]:offsets[u + 1]], 3, 3)
        assert [y for y, _ in alone[0]] == [y for y, _ in together[u]]
        np.testing.assert_allclose([s for _, s in alone[0]], [s for _, s in together[u]], atol=1e-5)


def test_decode_librispeech_headline_batch():
    """The benchmark's own batch in the benchmark's launch configuration (64 utterances, 17983
    frames, Dj=512, V=1024, LSTM 640, N=5, S=3): every utterance against the oracle, whole where
    all its decisions were clear and up to its first close decision otherwise."""
    shape = SHAPES["librispeech"]
    model = make_model(shape)
    offsets, enc = make_utterances(shape, model)
    info = _check_decode(shape, model, offsets, enc, 5, 3, report="Librispeech-like headline batch")
    assert info["tot"] == 64
    # flat synthetic distributions put thousands of expansion scores within 1e-3 of each other, so
    # every utterance meets a close decision within its first segments and the part the rule
    # makes strict is short; the whole-utterance count above it is reported (the kernels' actual
    # error is ~1e-6, so in practice the whole batch agrees)
    assert info.get("prefix_frames", int(offsets[-1])) >= 500, info


@pytest.mark.parametrize("index,N,S", [(11, 5, 3), (23, 5, 3), (37, 4, 5), (41, 10, 2)])
def test_decode_librispeech_widths_other_draws(index, N, S):
    """The headline widths (Dj=512, V=1024, LSTM 640) with other draws of the model and of the frames
    than the benchmark's, and utterance lengths around the segment size and its multiples (empty,
    shorter than a segment, a ragged last segment, one frame more or less than whole segments):
    the fixed-place form against the oracle."""
    import dataclasses
    shape = dataclasses.replace(SHAPES["librispeech"], index=index, n_utts=12)
    lengths = np.array([0, 1, 2, S, S + 1, 2 * S - 1, 40, 77, 30 * S, 30 * S + 1, 30 * S - 1, 211])
    model, offsets, enc = build_case(shape, n_utts=12, lengths=lengths)
    _, st = _gpu_decode(shape, model, offsets, enc, N, S)
    assert st["path"]["fixed_places"]
    _check_decode(shape, model, offsets, enc, N, S)


@pytest.mark.parametrize("U,N,S", [(70, 5, 3), (100, 5, 3), (273, 5, 3), (274, 5, 3), (90, 4, 1)])
def test_decode_fixed_places_with_more_tiles_than_cus(U, N, S):
    """The headline widths with so many utterances that the GEMMs of a round have more 64x64 tiles
    than the chip has CUs (up to 1024 joiner tiles: the fixed-place form still runs, its GEMMs with two
    LDS stages a workgroup and two workgroups a CU, K tiles refilled as they are read), one utterance
    more (the row-list form), and one-frame segments without logits: short utterances, all against
    the oracle."""
    import dataclasses
    shape = dataclasses.replace(SHAPES["librispeech"], index=53, n_utts=U)
    rng = np.random.default_rng(U)
    lengths = rng.integers(0, 14, size=U)
    model, offsets, enc = build_case(shape, n_utts=U, lengths=lengths)
    _, st = _gpu_decode(shape, model, offsets, enc, N, S)
    assert st["path"]["fixed_places"] == (U <= 273)
    _check_decode(shape, model, offsets, enc, N, S)


@pytest.mark.parametrize("name,N,S", [("assistant", 10, 3), ("throughput", 10, 5)])
def test_decode_large_shapes_short_utterances(name, N, S):
    """Whole decodes at the widths of the two large configurations (V=4096, Dj=1024, LSTM 2x1024 /
    1x1024) on a few short utterances, against the oracle."""
    import dataclasses
    shape = dataclasses.replace(SHAPES[name], n_utts=4)
    lengths = np.array([7, 16, 23, 30])
    model, offsets, enc = build_case(shape, n_utts=4, lengths=lengths)
    _check_decode(shape, model, offsets, enc, N, S, report=name)


@pytest.mark.parametrize("N,S", [(2, 1), (2, 5), (10, 1), (10, 2), (10, 5), (5, 2), (5, 5)])
def test_decode_librispeech_like_beam_and_segment_sweep(N, S):
    """The Librispeech-like configuration's sweep of beam and segment sizes, at its widths, on three
    utterances of 30-60 frames, whole decode against the oracle."""
    import dataclasses
    shape = dataclasses.replace(SHAPES["librispeech"], n_utts=3)
    lengths = np.array([31, 44, 60])
    model, offsets, enc = build_case(shape, n_utts=3, lengths=lengths)
    _check_decode(shape, model, offsets, enc, N, S)


@pytest.mark.parametrize("S", [10, 20, 50])
def test_decode_long_segments(S):
    """The long-segment configuration (Librispeech-like widths, N=5, S in {10, 20, 50}): the scan of
    Eq. 3 over long segments and the expansion kernels for S beyond the register-resident range."""
    import dataclasses
    shape = dataclasses.replace(SHAPES["librispeech"], n_utts=2)
    lengths = np.array([75, 128])
    model, offsets, enc = build_case(shape, n_utts=2, lengths=lengths)
    # a segment of S frames can take more rounds than the default workspace is sized for
    # (with blank probabilities of a few percent the blank products over such segments span ~1e-85:
    # this is the case that needs the forward variable and d carried with extended range)
    _check_decode(shape, model, offsets, enc, 5, S, rounds_capacity=4 * S, report=f"S={S}")


def test_decode_largest_segment_and_smallest_vocabulary():
    """The limits of the configuration: S = 128 (the largest segment the library takes; one full
    segment and a ragged one) with a small model, and V = 2 (blank and one token: every hypothesis
    has one expansion, top-N and threshold degenerate) at several beam widths."""
    shape = small_bf16_shape(n_utts=2, vocab=24, d=64, hidden=64)
    lengths = np.array([140, 131])
    model, offsets, enc = build_case(shape, n_utts=2, lengths=lengths)
    _check_decode(shape, model, offsets, enc, 3, 128, rounds_capacity=512)
    shape2 = small_bf16_shape(n_utts=3, vocab=2, d=64, hidden=64)
    model2, off2, enc2 = build_case(shape2, n_utts=3, lengths=np.array([5, 11, 2]))
    for N, S in ((1, 1), (3, 2), (4, 5)):
        _check_decode(shape2, model2, off2, enc2, N, S)


@pytest.mark.parametrize("name,N,S,U", [("assistant", 10, 3, 300), ("throughput", 10, 5, 200)])
def test_decode_large_batch_contains_the_small_one(name, N, S, U):
    """The large configurations' widths with enough utterances that every round runs on the kernels
    chosen at scale (256x256-tile joiner GEMM, 80- or 48-logit-per-thread expansion, LSTM cell
    update as its own kernel behind a large gate GEMM): the first eight utterances against the
    oracle under the gap rule, decoded inside the large batch."""
    import dataclasses
    shape = dataclasses.replace(SHAPES[name], n_utts=U)
    lengths = np.concatenate([np.array([7, 16, 23, 30, 5, 11, 19, 26]), np.full(U - 8, 12)])
    model, offsets, enc = build_case(shape, n_utts=U, lengths=lengths)
    tol, score_tol = tolerance(shape, model)
    full, st = _gpu_decode(shape, model, offsets, enc, N, S)
    assert st["frames"] == int(offsets[-1])
    off8 = offsets[:9].copy()
    ref = _oracle_decode(shape, model, off8, enc[:off8[-1]], N, S)
    same, amb, tot = compare_nbest(full[:8], ref, score_tol=score_tol, gap_tol=tol)
    # the same eight cut back to before their first close decision, again inside a large batch
    offp, encp, keep = strict_prefixes(ref, off8, enc[:off8[-1]], S, tol)
    lengths2 = np.concatenate([keep, np.full(U - 8, 12)])
    off2 = np.concatenate([[0], np.cumsum(lengths2)]).astype(np.int32)
    enc2 = np.concatenate([encp, enc[off8[-1]:]])
    full2, _ = _gpu_decode(shape, model, off2, enc2, N, S)
    ref2 = _oracle_decode(shape, model, offp, encp, N, S)
    assert_all_agree(full2[:8], ref2, score_tol, tol)
    print(f"{name}: identical {same}/{tot} whole, strict prefix frames {int(keep.sum())}/{int(off8[-1])}")


@pytest.mark.parametrize("N,S,V,peaked", [(3, 3, 96, False), (4, 5, 1024, False), (5, 3, 1024, False), (8, 5, 512, True),
                                          (10, 3, 1024, False), (16, 4, 200, True), (5, 3, 96, True), (2, 1, 64, True)])
def test_round_in_one_kernel_equals_separate_kernels(N, S, V, peaked):
    """Inside tbs_decode, expansion and select/merge of a round run as one kernel (a workgroup per
    utterance) where the shape allows; debug bit 7 keeps them two kernels.  Beam widths and
    vocabularies that take each of the kernel's forms (4, 8 or 16 columns per thread, with and without
    a wave of its own for the select step), ragged utterances, flat and peaked models: the two forms must give the same hypotheses, and the
    one-kernel form is checked against the oracle."""
    shape = small_bf16_shape(n_utts=6, vocab=V, d=128, hidden=128)
    cap = 0
    if peaked:
        shape, cap = _peaked(shape, 8.0, 8.0), 5
    lengths = np.array([0, 2, 7, 12, 23, 31])
    model, offsets, enc = build_case(shape, n_utts=6, lengths=lengths)
    kw = dict(max_rounds_per_segment=cap) if cap else {}
    # default: every hypothesis in a fixed place, four kernels a round; 256: the one-kernel round with
    # row lists made by a kernel of their own; 128: expansion and select/merge as two kernels as well
    one, st1 = _gpu_decode(shape, model, offsets, enc, N, S, **kw)
    for dbg in (256, 128):
        two, st2 = _gpu_decode(shape, model, offsets, enc, N, S, debug=dbg, **kw)
        for a, b in zip(one, two):
            assert [h[0] for h in a] == [h[0] for h in b], dbg
            np.testing.assert_allclose([h[1] for h in a], [h[1] for h in b], rtol=1e-6, atol=1e-5)
        assert st1["joiner_calls"] == st2["joiner_calls"] and st1["joined_frames"] == st2["joined_frames"], dbg
        assert st1["launches"] == st2["launches"] and st1["frames"] == st2["frames"], dbg
    _check_decode(shape, model, offsets, enc, N, S, max_rounds=cap)
    _check_decode(shape, model, offsets, enc, N, S, max_rounds=cap, debug=256)
    _check_decode(shape, model, offsets, enc, N, S, max_rounds=cap, debug=128)


@pytest.mark.parametrize("N,V,blank,peaked", [(1, 64, 0, False), (2, 96, 0, True), (4, 1024, 0, False), (5, 1024, 0, True),
                                              (5, 200, 7, True), (8, 512, 511, True), (10, 4096, 0, False),
                                              (16, 100, 64, True), (3, 68, 67, False)])
def test_standard_search_without_logits_equals_the_one_with(N, V, blank, peaked):
    """S = 1 is the standard breadth-first search (Eq. 1).  The joiner GEMM can then keep no logits: its
    epilogue leaves each row's softmax sums, blank logit and N best tokens per 16-column piece (or, debug
    bit 14, merged per tile of 64 columns) and the round kernel merges them.  That form runs by default
    for beams up to 4 and where the vocabulary is too large for the form with logits, and with debug bit
    15 everywhere; debug bit 9 asks for the logits.  Vocabularies of one tile, of many and with a ragged last tile, blank
    first, last, at a tile edge and inside a tile, every list length the round kernel has (4, 8, 16),
    flat and peaked models, ragged and empty utterances: the forms give the same hypotheses, and each is
    checked against the oracle."""
    import dataclasses
    shape = dataclasses.replace(small_bf16_shape(n_utts=6, vocab=V, d=128, hidden=128), blank_id=blank)
    cap = 0
    if peaked:
        shape, cap = _peaked(shape, 8.0, 8.0), 5
    lengths = np.array([0, 1, 7, 12, 23, 31])
    model, offsets, enc = build_case(shape, n_utts=6, lengths=lengths)
    kw = dict(max_rounds_per_segment=cap) if cap else {}
    dflt, st0 = _gpu_decode(shape, model, offsets, enc, N, 1, **kw)
    one, st1 = _gpu_decode(shape, model, offsets, enc, N, 1, debug=32768, **kw)
    two, st2 = _gpu_decode(shape, model, offsets, enc, N, 1, debug=512, **kw)
    # (the form with logits keeps a hypothesis' logits in registers: vocabularies up to 1024 entries)
    # (by default the form without logits serves beams up to 4 and the vocabularies the other cannot hold)
    assert st0["path"] == {"fixed_places": True, "one_frame_no_logits": V > 1024 or N <= 4}
    assert st1["path"] == {"fixed_places": True, "one_frame_no_logits": True}
    assert st2["path"] == {"fixed_places": V <= 1024, "one_frame_no_logits": False}
    assert dflt == (one if (V > 1024 or N <= 4) else two)
    tol, score_tol = tolerance(shape, model)
    # (bit 14: the partials of a tile's four 16-column pieces merged by the GEMM instead of the round kernel:
    # the same arithmetic in another order of the sums)
    three, st3 = _gpu_decode(shape, model, offsets, enc, N, 1, debug=32768 + 16384, **kw)
    assert st3["path"] == st1["path"]
    for other in (two, three):
        for a, b in zip(one, other):
            # (the forms round differently: log(exp(l - m) / Z) against (l - m) - log Z)
            assert [h[0] for h in a] == [h[0] for h in b]
            np.testing.assert_allclose([h[1] for h in a], [h[1] for h in b], rtol=0, atol=score_tol)
    assert st1["joiner_calls"] == st2["joiner_calls"] and st1["joined_frames"] == st2["joined_frames"]
    assert st1["launches"] == st2["launches"] and st1["frames"] == st2["frames"]
    _check_decode(shape, model, offsets, enc, N, 1, max_rounds=cap, debug=32768)
    _check_decode(shape, model, offsets, enc, N, 1, max_rounds=cap, debug=512)
    _check_decode(shape, model, offsets, enc, N, 1, max_rounds=cap, debug=32768 + 16384)


def test_standard_search_without_logits_librispeech_batch():
    """The in-house baseline of the benchmark (64 Librispeech-like utterances, N = 5, S = 1) in the form
    without logits agrees with the oracle under the gap rule."""
    shape = SHAPES["librispeech"]
    model, offsets, enc = build_case(shape)
    _, st = _gpu_decode(shape, model, offsets[:3], enc[:offsets[2]], 5, 1, debug=32768)
    assert st["path"]["one_frame_no_logits"]
    info = _check_decode(shape, model, offsets, enc, 5, 1, report="Librispeech-like, standard search (S=1)",
                         debug=32768)
    assert info["tot"] == 64


@pytest.mark.parametrize("N,S,U", [(5, 3, 6), (4, 5, 6), (10, 2, 70), (3, 1, 130)])
def test_first_round_rows_from_the_segment_head_equal_those_of_their_own_kernel(N, S, U):
    """In the layout with fixed places the kernel that starts a segment also forms the joiner input
    rows of the segment's first round, with one, two or four workgroups per utterance depending on the
    batch; debug bit 10 forms them in a kernel of their own.  Ragged and empty utterances, batches of
    every workgroup count: identical hypotheses, and the oracle on the first utterances."""
    shape = small_bf16_shape(n_utts=U, vocab=128, d=128, hidden=128)
    rng = np.random.default_rng(7)
    lengths = rng.integers(0, 20, size=U)
    lengths[:6] = [0, 1, 7, 12, 23, 31]
    model, offsets, enc = build_case(shape, n_utts=U, lengths=lengths)
    one, st1 = _gpu_decode(shape, model, offsets, enc, N, S)
    # (bit 11: the later rounds' rows, from the projection's epilogue, by one workgroup per tile instead of
    # one per tile and frame)
    # (bit 12: the joiner GEMM's tiles spread over the XCDs as the other GEMMs' are, instead of a range of
    # rows per XCD with the round kernel's workgroups placed to match)
    for dbg in (1024, 2048, 4096, 1024 + 2048 + 4096):
        two, st2 = _gpu_decode(shape, model, offsets, enc, N, S, debug=dbg)
        assert st1["path"]["fixed_places"] and st2["path"]["fixed_places"]
        assert one == two, dbg
        assert st1["joiner_calls"] == st2["joiner_calls"] and st1["joined_frames"] == st2["joined_frames"]
    _check_decode(shape, model, offsets[:7], enc[:offsets[6]], N, S)


@pytest.mark.parametrize("N,S,d", [(5, 3, 64), (3, 12, 64), (10, 2, 128), (4, 5, 144)])
def test_joiner_rows_by_pair_equal_those_by_row(N, S, d):
    """With row lists the joiner input rows act(e + p) come from a kernel of their own: a thread per
    pair and 8 columns (all frames of the pair), or with debug bit 13 a thread per row and 8 columns.
    Identical hypotheses required, and the oracle's on the default form."""
    shape = small_bf16_shape(n_utts=6, vocab=96, d=d, hidden=64)
    lengths = np.array([0, 1, 7, 12, 23, 31])
    model, offsets, enc = build_case(shape, n_utts=6, lengths=lengths)
    kw = dict(rounds_capacity=4 * S) if S > 8 else {}
    one, st1 = _gpu_decode(shape, model, offsets, enc, N, S, debug=256, **kw)
    two, st2 = _gpu_decode(shape, model, offsets, enc, N, S, debug=256 + 8192, **kw)
    assert not st1["path"]["fixed_places"]
    assert one == two
    assert st1["joiner_calls"] == st2["joiner_calls"] and st1["joined_frames"] == st2["joined_frames"]
    _check_decode(shape, model, offsets, enc, N, S, debug=256, **kw)


@pytest.mark.parametrize("chunk", [1, 11, 40])
def test_decode_with_joiner_calls_in_pieces(chunk):
    """Whole decodes whose every joiner call of more than `chunk` rows runs in pieces."""
    shape = small_bf16_shape(n_utts=6, vocab=64, d=64, hidden=64, layers=2)
    lengths = np.array([0, 1, 2, 7, 12, 23])
    model, offsets, enc = build_case(shape, n_utts=6, lengths=lengths)
    _check_decode(shape, model, offsets, enc, 5, 3, joiner_chunk_rows=chunk)
    whole, _ = _gpu_decode(shape, model, offsets, enc, 5, 3, joiner_chunk_rows=0)
    parts, _ = _gpu_decode(shape, model, offsets, enc, 5, 3, joiner_chunk_rows=chunk)
    assert whole == parts      # the same arithmetic per row, whatever the pieces


@pytest.mark.parametrize("N,S", [(32, 2), (17, 3)])
def test_decode_wide_beams(N, S):
    """Beams up to the library's maximum: the list kernels' general paths (more than 64 candidates
    per utterance, B lists of hundreds of entries)."""
    shape = small_bf16_shape(n_utts=3, vocab=96, d=64, hidden=64)
    lengths = np.array([5, 11, 18])
    model, offsets, enc = build_case(shape, n_utts=3, lengths=lengths)
    _check_decode(shape, model, offsets, enc, N, S)


def test_errors_are_codes_not_crashes():
    from paper_2302_14357_amd import TbsError
    shape = small_bf16_shape(n_utts=2)
    model, offsets, enc = build_case(shape, n_utts=2, lengths=np.array([5, 6]))
    tbs = make_tbs(shape, model, offsets, 2, 2)
    with pytest.raises(TbsError) as e:
        tbs.expand()            # before begin / joiner
    assert e.value.code == -2
    enc_dev = tbs.upload_frames(enc)
    tbs.begin(enc_dev, offsets)
    with pytest.raises(TbsError) as e:
        tbs.joiner_segment()    # before segment_begin
    assert e.value.code == -2
    with pytest.raises(TbsError) as e:
        tbs.begin(enc_dev, np.array([0, 5, 11, 12], np.int32))   # more utterances than capacity
    assert e.value.code == -1
    tbs.close()
    # rounds capacity of one: the second round of a segment overflows cleanly
    tbs = make_tbs(shape, model, offsets, 2, 2, rounds_capacity=1)
    with pytest.raises(TbsError) as e:
        tbs.decode(tbs.upload_frames(enc), offsets)
    assert e.value.code == -5
    tbs.close()
    # the same at a width whose segments are enqueued head and first round in one go, and the
    # context still decodes afterwards when given the room
    shape = small_bf16_shape(n_utts=2, d=128, hidden=128)
    model, offsets, enc = build_case(shape, n_utts=2, lengths=np.array([5, 6]))
    tbs = make_tbs(shape, model, offsets, 2, 2, rounds_capacity=1)
    with pytest.raises(TbsError) as e:
        tbs.decode(tbs.upload_frames(enc), offsets)
    assert e.value.code == -5
    tbs.close()
    _check_decode(shape, model, offsets, enc, 2, 2)
