"""Pins of the CPU oracle against things other than itself (CPU only).

What fixes each part:
 * Eq. 3-7 and the driver's use of them: brute-force enumeration of every
   alignment, the transducer forward recursion for every S, conservation of
   probability mass, the S=1 closed form (Eq. 1), an O(S) forward scan.
 * the driver at S=1: an independently written frame-wise beam search.
 * softmax, dense layers, LSTM cell, bf16 rounding: library routines.
 * the beam policy (threshold rule, joint top-N): a hand-worked example from
   the text of Algorithm 1 (tests/golden/alg1_hand_example.txt).
 * planted mistakes: each must break at least one of the above.
"""

import math
import os

import numpy as np
import pytest

import oracle
from tbs_inputs import make_table_logits
from independent import (Lattice, enumerate_paths, last_emission_profile, forward_probability,
                         framewise_beam_search, alpha_scan, softmax_np)

HUGE_N = 100000


def table_fn(seed, V, blank_bias=0.5):
    return lambda frame, toks: make_table_logits(seed, frame, toks, V, 0, blank_bias)


def oracle_all_hyps(fn, V, T, S, L, raw=False, trace=False):
    m = oracle.TableModel(fn, V, 0)
    return oracle.decode(m, T, HUGE_N, S, max_rounds=L + 1, raw_prob=raw, trace=trace)


# ------------------------------------------------------------------ brute force

@pytest.mark.parametrize("T,S,L", [(1, 1, 2), (2, 2, 2), (3, 3, 2), (4, 4, 2), (4, 2, 2), (5, 3, 1), (3, 5, 3)])
@pytest.mark.parametrize("raw", [False, True])
def test_brute_force_all_alignments(T, S, L, raw):
    V = 3
    fn = table_fn(100 + T * 10 + S, V)
    want = enumerate_paths(Lattice(fn, V), T, S, L)
    got = oracle_all_hyps(fn, V, T, S, L, raw=raw)
    got_map = {tok: math.exp(ls) for tok, ls in got.nbest}
    assert set(got_map) == set(want)
    for y, p in want.items():
        assert got_map[y] == pytest.approx(p, rel=1e-11), y


def test_brute_force_last_emission_distribution():
    """d of every hypothesis created in the first segment = mass of the paths
    whose last token falls in each frame (Eq. 5)."""
    V, S, L = 3, 4, 3
    fn = table_fn(7, V)
    prof = last_emission_profile(Lattice(fn, V), S, L)
    got = oracle_all_hyps(fn, V, S, S, L, raw=True, trace=True)
    seen = 0
    for r in got.rounds:
        assert r.seg == 0
        for (h, k), sc, d in zip(r.new_pairs, r.new_scores, r.new_d):
            y = r.a_tokens[h] + (k,)
            if len(y) > L:
                continue
            np.testing.assert_allclose(d, prof[y], rtol=1e-11, atol=0)
            assert sc == pytest.approx(prof[y].sum(), rel=1e-11)
            seen += 1
    assert seen == 2 + 4 + 8


# ------------------------------------------------------------------ forward recursion, S-invariance

@pytest.mark.parametrize("S", [1, 2, 3, 4, 6, 7])
def test_forward_probability_every_segment_size(S):
    V, T, L = 3, 6, 2
    fn = table_fn(42, V)
    lat = Lattice(fn, V)
    got = oracle_all_hyps(fn, V, T, S, L)
    checked = 0
    for y, ls in got.nbest:
        if len(y) <= L:   # every alignment of y has at most L emissions in any segment
            assert math.exp(ls) == pytest.approx(forward_probability(lat, T, y), rel=1e-10)
            checked += 1
    assert checked == 1 + 2 + 4


def test_log_domain_equals_raw_probabilities():
    V, T = 4, 7
    fn = table_fn(5, V, blank_bias=1.0)
    for S in (1, 3, 7):
        a = oracle.decode(oracle.TableModel(fn, V), T, 3, S, raw_prob=True)
        b = oracle.decode(oracle.TableModel(fn, V), T, 3, S, raw_prob=False)
        assert [y for y, _ in a.nbest] == [y for y, _ in b.nbest]
        np.testing.assert_allclose([s for _, s in a.nbest], [s for _, s in b.nbest], rtol=0, atol=1e-11)


# ------------------------------------------------------------------ algebra

def random_case(seed, H, S, V):
    rng = np.random.default_rng(seed)
    logits = rng.standard_normal((H, S, V)) * 2.0
    logits[..., 0] += 1.0
    d_old = rng.random((H, S))
    d_old[rng.random((H, S)) < 0.3] = 0.0
    d_old[:, 0] += 0.1
    return logits, d_old


@pytest.mark.parametrize("H,S,V", [(1, 1, 5), (3, 3, 7), (2, 10, 33), (4, 50, 17)])
def test_mass_conservation(H, S, V):
    logits, d_old = random_case(1, H, S, V)
    J, Bl, d, dnb, dphi = oracle.expansion_scores(logits, d_old, 0)
    total = dphi + d.sum(axis=(1, 2))
    np.testing.assert_allclose(total, d_old.sum(axis=1), rtol=1e-12)
    np.testing.assert_allclose(dnb, d.sum(axis=2), rtol=1e-13)
    assert (d[:, 0, :] == 0).all()


def test_blank_product_definition():
    """Eq. 3 entry by entry with numpy.prod on a small case."""
    logits, _ = random_case(2, 2, 4, 5)
    J = oracle.softmax(logits)
    Bl = oracle.blank_product(J, 0)
    for h in range(2):
        for t1 in range(1, 6):
            for t2 in range(1, 6):
                want = 0.0 if t1 > t2 else float(np.prod(J[h, t1 - 1:t2 - 1, 0]))
                assert Bl[h, t1 - 1, t2 - 1] == pytest.approx(want, rel=1e-14, abs=0)


def test_segment_of_one_frame_is_eq1():
    """S=1: delta_nb = s*J(k), delta_blank = s*J(blank) (Eq. 1)."""
    rng = np.random.default_rng(3)
    H, V = 4, 9
    logits = rng.standard_normal((H, 1, V))
    s = rng.random((H, 1)) + 0.1
    J, Bl, d, dnb, dphi = oracle.expansion_scores(logits, s, 0)
    Jn = np.stack([softmax_np(logits[h, 0]) for h in range(H)])
    np.testing.assert_allclose(dphi, s[:, 0] * Jn[:, 0], rtol=1e-13)
    np.testing.assert_allclose(dnb[:, 1:], s * Jn[:, 1:], rtol=1e-13)


@pytest.mark.parametrize("S", [1, 2, 5, 50])
def test_table_form_equals_forward_scan(S):
    """The O(S^2) table of Eq. 3-7 against the O(S) forward variable."""
    H, V = 3, 11
    logits, d_old = random_case(4 + S, H, S, V)
    J, Bl, d, dnb, dphi = oracle.expansion_scores(logits, d_old, 0)
    for h in range(H):
        alpha, db = alpha_scan(J[h, :, 0], d_old[h])
        assert dphi[h] == pytest.approx(db, rel=1e-12)
        np.testing.assert_allclose(d[h, 1:, :], (alpha[None, :] * J[h, :, 1:].T), rtol=1e-12, atol=1e-300)


# ------------------------------------------------------------------ S=1 driver vs frame-wise search

@pytest.mark.parametrize("seed,N,V,T", [(1, 1, 4, 6), (2, 2, 5, 8), (3, 3, 6, 7), (4, 5, 8, 6)])
def test_segment_one_equals_framewise_search(seed, N, V, T):
    fn = table_fn(200 + seed, V, blank_bias=1.5)
    want = framewise_beam_search(Lattice(fn, V), T, N)
    got = oracle.decode(oracle.TableModel(fn, V), T, N, 1)
    assert [y for y, _ in got.nbest] == [y for y, _ in want]
    np.testing.assert_allclose([math.exp(s) for _, s in got.nbest], [p for _, p in want], rtol=1e-11)


# ------------------------------------------------------------------ hand-worked examples (policy)

def _read_golden(name):
    """{section: {key: value}}; lines before the first [section] go to section ''."""
    path = os.path.join(os.path.dirname(__file__), "golden", name)
    out, cur = {"": {}}, ""
    with open(path) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if not line:
                continue
            if line.startswith("[") and line.endswith("]"):
                cur = line[1:-1]
                out[cur] = {}
                continue
            k, v = line.split("=")
            out[cur][k.strip()] = v.strip()
    return out


def _run_golden(g):
    probs = {}
    for k, v in g.items():
        if k.startswith("J("):
            frame, toks = k[2:-1].split("|")
            probs[(int(frame), tuple(int(x) for x in toks.split()))] = [float(x) for x in v.split()]

    def fn(frame, toks):
        # (a table the file does not hold, asked for only by a run that has already gone wrong: blank only)
        with np.errstate(divide="ignore"):
            return np.log(np.array(probs.get((frame, toks), [1.0, 0.0, 0.0])))

    res = oracle.decode(oracle.TableModel(fn, 3), int(g["T"]), int(g["N"]), int(g["S"]), raw_prob=True, trace=True)
    want = []
    for item in g["nbest"].split(";"):
        toks, p = item.split(":")
        want.append((tuple(int(x) for x in toks.split()), float(p)))
    return res, want


def _check_golden(g):
    res, want = _run_golden(g)
    assert [y for y, _ in res.nbest] == [y for y, _ in want]
    np.testing.assert_allclose([math.exp(s) for _, s in res.nbest], [p for _, p in want], rtol=1e-12)
    assert res.joiner_calls == int(g["joiner_calls"])
    for k, v in g.items():   # (parent, token) of the hypotheses each round creates, rounds counted over the run
        if k.startswith("new("):
            pairs = [tuple(int(x) for x in it.split()) for it in v.split(";") if it.strip()]
            assert res.rounds[int(k[4:-1]) - 1].new_pairs == pairs, k
    return res


def test_hand_worked_example():
    _check_golden(_read_golden("alg1_hand_example.txt")[""])


def test_hand_worked_decision_gaps():
    """The gap bookkeeping that decides how strictly two decodes are compared: every head-of-segment
    and per-round gap of the hand-worked run, from the values worked out beside it."""
    g = _read_golden("alg1_hand_example.txt")[""]
    res, _ = _run_golden(g)

    def val(key):
        v = g[key]
        if v == "none":
            return math.inf
        a, b = (float(x) for x in v.split())
        return abs(math.log(a) - math.log(b))

    seen = set()
    for r in res.rounds:
        assert r.head_gap == pytest.approx(val(f"head({r.seg})"), rel=1e-12), (r.seg, r.round)
        assert r.gap == pytest.approx(val(f"gap({r.seg},{r.round})"), rel=1e-12), (r.seg, r.round)
        seen.add((r.seg, r.round))
    assert seen == {(0, 1), (0, 2), (1, 1), (1, 2)}
    assert res.final_gap == val("final")
    assert res.min_gap == pytest.approx(abs(math.log(0.12) - math.log(0.1134)), rel=1e-12)
    assert res.first_ambiguous_segment(0.05) is None
    assert res.first_ambiguous_segment(0.06) == 1       # segment 1, round 1: 0.12 against 0.1134
    assert res.first_ambiguous_segment(0.09) == 0       # segment 0, round 2: 0.174 against 0.189
    # with N = 1 the final list of two entries is cut: its gap is that of the two results
    res1 = oracle.decode(oracle.TableModel(lambda f, t: np.log(np.array([0.5, 0.3, 0.2])), 3), 1, 1, 1, raw_prob=True)
    assert res1.nbest[0][0] == () and res1.final_gap == pytest.approx(math.inf)   # 0.3 <= threshold 0.5: B = {[]}
    res2 = oracle.decode(oracle.TableModel(lambda f, t: np.log(np.array([0.3, 0.5, 0.2])), 3), 1, 1, 1, raw_prob=True)
    # B = {[]:0.3}, threshold 0.3 < 0.5: [1] enters, takes its blank (0.15) into B; final cut: 0.3 vs 0.15
    assert res2.nbest[0][0] == () and res2.final_gap == pytest.approx(math.log(2.0), rel=1e-12)


@pytest.mark.parametrize("case", ["strict", "joint"])
def test_policy_examples(case):
    """Hand-worked runs in which a non-strict threshold test, or N expansions per hypothesis
    instead of N in all, would give another result."""
    _check_golden(_read_golden("alg1_policy_examples.txt")[case])


# ------------------------------------------------------------------ library pins

def test_softmax_against_scipy():
    from scipy.special import softmax as sp_softmax
    rng = np.random.default_rng(0)
    x = rng.standard_normal((13, 37)) * 5
    np.testing.assert_allclose(oracle.softmax(x), sp_softmax(x, axis=-1), rtol=1e-13)


def test_bf16_rounding_against_torch():
    import torch
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(4000), rng.standard_normal(1000) * 1e-3,
                        np.array([0.0, 1.0, -1.0, 1.00390625, 1.01171875, 0.99609375])])
    want = torch.tensor(x, dtype=torch.float64).to(torch.float32).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(oracle.round_bf16(x), want)


def _small_model(layers=2, quant=False, act="tanh"):
    from tbs_inputs import TbsShape, make_model, make_utterances
    shape = TbsShape("t", 9, 1, 7, 7, 12, 16, 10, 0, layers, 24, 20, "bf16" if quant else "f32", act)
    model = make_model(shape)
    offs, enc = make_utterances(shape, model)
    return shape, model, enc


@pytest.mark.parametrize("layers", [1, 2])
def test_lstm_predictor_against_torch(layers):
    import torch
    shape, model, enc = _small_model(layers)
    W = oracle.LstmWeights(model, 0)
    m = oracle.LstmModel(W, enc)
    lstm = torch.nn.LSTM(shape.pred_embed, shape.pred_hidden, num_layers=layers).double()
    with torch.no_grad():
        for l, (wi, wh, b) in enumerate(model["lstm"]):
            getattr(lstm, f"weight_ih_l{l}").copy_(torch.tensor(wi, dtype=torch.float64))
            getattr(lstm, f"weight_hh_l{l}").copy_(torch.tensor(wh, dtype=torch.float64))
            getattr(lstm, f"bias_ih_l{l}").copy_(torch.tensor(b, dtype=torch.float64))
            getattr(lstm, f"bias_hh_l{l}").zero_()
    toks = [3, 7, 1, 9, 3]
    s = m.init_state()
    p0, h0, c0 = m.get_state(s)
    np.testing.assert_array_equal(p0, model["pred_init"].astype(np.float64))
    assert (h0 == 0).all() and (c0 == 0).all()
    hc = None
    for tk in toks:
        s = m.update_state(s, tk)
        x = torch.tensor(model["embed"][tk], dtype=torch.float64).view(1, 1, -1)
        with torch.no_grad():
            out, hc = lstm(x, hc)
        p, h, c = m.get_state(s)
        np.testing.assert_allclose(h, hc[0][:, 0].numpy(), rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(c, hc[1][:, 0].numpy(), rtol=1e-12, atol=1e-14)
        want_p = model["w_proj"].astype(np.float64) @ out[0, 0].numpy() + model["b_proj"]
        np.testing.assert_allclose(p, want_p, rtol=1e-12, atol=1e-14)


@pytest.mark.parametrize("act", ["tanh", "relu"])
def test_joiner_against_numpy(act):
    shape, model, enc = _small_model(1, act=act)
    W = oracle.LstmWeights(model, 0, act=act)
    rng = np.random.default_rng(1)
    p = rng.standard_normal(shape.d_joint)
    x = enc[2].astype(np.float64) + p
    a = np.tanh(x) if act == "tanh" else np.maximum(x, 0)
    want = model["w_out"].astype(np.float64) @ a + model["b_out"]
    np.testing.assert_allclose(W.joiner_vec(enc[2], p), want, rtol=1e-12, atol=1e-14)


def test_joiner_quantised_mode_rounds_the_activation():
    import torch
    shape, model, enc = _small_model(1, quant=True)
    W = oracle.LstmWeights(model, 0, quant_bf16=True)
    rng = np.random.default_rng(1)
    p = rng.standard_normal(shape.d_joint).astype(np.float32).astype(np.float64)
    a = np.tanh(enc[1].astype(np.float64) + p)
    a = torch.tensor(a).to(torch.float32).to(torch.bfloat16).to(torch.float64).numpy()
    want = model["w_out"].astype(np.float64) @ a + model["b_out"]
    np.testing.assert_allclose(W.joiner_vec(enc[1], p), want, rtol=1e-12, atol=1e-14)


def test_lstm_decode_runs_and_counts():
    shape, model, enc = _small_model(1)
    W = oracle.LstmWeights(model, 0)
    res, used = oracle.decode_lstm_batch(W, enc, np.array([0, 7], np.int32), 2, 3, threads=1)
    r = res[0]
    assert r.frames == 7 and 1 <= len(r.nbest) <= 2
    # joined frames = sum over calls of the frames in the call's segment
    assert r.joined_frames <= r.joiner_calls * 3 and r.joiner_calls >= 3
    single = oracle.decode(oracle.LstmModel(W, enc), 7, 2, 3)
    assert single.nbest == r.nbest


# ------------------------------------------------------------------ planted mistakes are noticed

def _score_pins():
    test_brute_force_all_alignments(3, 3, 2, False)
    test_brute_force_all_alignments(4, 2, 2, False)
    test_brute_force_last_emission_distribution()
    test_forward_probability_every_segment_size(3)
    test_mass_conservation(3, 3, 7)


def _policy_pins():
    test_hand_worked_example()
    test_policy_examples("strict")
    test_policy_examples("joint")


# 1 blank product off by a frame, 2 no same-frame emission, 4 merge keeps the larger score, 5 the
# frame of the last token forgotten, 6 blank expansion a frame short, 8 no merging at all: caught by
# the score pins.  9 threshold test not strict, 10 N expansions per hypothesis, 11 threshold one
# place too far down B: caught by the hand-worked runs of Algorithm 1.
@pytest.mark.parametrize("mutant,pins", [(1, _score_pins), (2, _score_pins), (4, _score_pins), (5, _score_pins),
                                         (6, _score_pins), (8, _score_pins), (9, _policy_pins),
                                         (10, _policy_pins), (11, _policy_pins)])
def test_planted_mistake_is_caught(mutant, pins):
    oracle.set_mutant(mutant)
    try:
        with pytest.raises(AssertionError):
            pins()
    finally:
        oracle.set_mutant(0)
    pins()


@pytest.mark.parametrize("mutant,case", [(9, "strict"), (10, "joint")])
def test_each_policy_example_catches_its_own_reading(mutant, case):
    oracle.set_mutant(mutant)
    try:
        with pytest.raises(AssertionError):
            test_policy_examples(case)
    finally:
        oracle.set_mutant(0)
