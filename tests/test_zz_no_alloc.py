"""The entry point that allocates nothing (tbs_debug_hyps_noalloc) against the entry point it is a
variant of (tbs_debug_hyps), through the C ABI: identical outputs (integers, and scores copied bit
for bit), on calls in a row that share the one static scratch array, the later ones smaller than
the first, and a request beyond the array's size refused with its own code."""

import dataclasses

import numpy as np
import pytest

from helpers import build_case, make_tbs, small_bf16_shape

pytestmark = pytest.mark.gpu


def _same(a, b):
    for x, y in zip(a, b):
        np.testing.assert_array_equal(x, y)


def test_no_alloc_variant_equals_the_allocating_one():
    from paper_2302_14357_amd import TbsError
    # a peaked model mid-decode: lists A and B with sequences of several tokens
    shape = dataclasses.replace(small_bf16_shape(n_utts=6, vocab=12, d=64, hidden=64), logit_scale=8.0, blank_bias=8.0)
    lengths = np.array([30, 21, 38, 14, 26, 9])
    model, offsets, enc = build_case(shape, n_utts=6, lengths=lengths)
    N, S = 5, 3
    tbs = make_tbs(shape, model, offsets, N, S, max_rounds_per_segment=6)
    tbs.begin(tbs.upload_frames(enc), offsets)
    for seg in range(4):                      # stop inside segment 3, after two rounds
        rows = tbs.segment_begin(seg)
        rounds = 0
        while rows > 0 and not (seg == 3 and rounds == 2):
            tbs.joiner_segment()
            tbs.expand()
            tbs.select_merge()
            tbs.predictor_step()
            rows = tbs.counts()["rows"]
            rounds += 1
    # first call: the long list B of all six utterances, wide outputs
    want = tbs.debug_hyps_raw(1, cap=N * 6, max_len=24)
    got = tbs.debug_hyps_raw(1, cap=N * 6, max_len=24, noalloc=True, fill=-9)
    _same(got, want)
    assert want[3].max() >= N and want[1].max() >= 3      # B holds more than N entries, sequences of 3+ tokens
    # second call right after it, smaller in every dimension (group A, narrow outputs): nothing of
    # what the first call left in the scratch may show
    want2 = tbs.debug_hyps_raw(0, cap=N, max_len=2)
    got2 = tbs.debug_hyps_raw(0, cap=N, max_len=2, noalloc=True, fill=-9)
    _same(got2, want2)
    assert want2[3].sum() > 0
    # third: a smaller batch on the same context and device
    off3 = offsets[:3].copy()
    tbs.decode(tbs.upload_frames(enc[:off3[-1]]), off3)
    want3 = tbs.debug_hyps_raw(1, cap=3, max_len=5)
    got3 = tbs.debug_hyps_raw(1, cap=3, max_len=5, noalloc=True, fill=-9)
    _same(got3, want3)
    assert got3[0].shape == (2, 3, 5)
    # beyond the fixed scratch: refused with its own code, the caller's arrays untouched
    with pytest.raises(TbsError) as e:
        tbs.debug_hyps_raw(1, cap=4096, max_len=256, noalloc=True)
    assert e.value.code == -6
    tbs.close()
