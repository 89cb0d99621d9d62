"""CPU-side checks of the C-ABI library: it loads, exports every symbol the
header declares, and rejects bad configurations before touching a GPU."""

import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _lib():
    from paper_2302_14357_amd import tbs
    return tbs.load_library(), tbs


def test_library_exports_every_declared_symbol():
    L, tbs = _lib()
    header = open(os.path.join(ROOT, "include", "tbs.h")).read()
    declared = set(re.findall(r"\b(tbs_[a-z0-9_]+)\s*\(", header))
    assert declared, "no declarations found"
    assert declared == set(tbs.EXPORTED_SYMBOLS)
    for name in declared:
        assert hasattr(L, name), name


def test_strerror_and_invalid_configs():
    L, tbs = _lib()
    assert L.tbs_strerror(0) == b"ok"
    assert b"order" in L.tbs_strerror(-2)
    cfg = tbs._Config()
    w = tbs._Weights()
    ctx = C.c_void_p()
    assert L.tbs_init(None, None, None) == -1
    # all-zero configuration
    assert L.tbs_init(C.byref(cfg), C.byref(w), C.byref(ctx)) == -1
    good = dict(d_joint=64, vocab=32, blank_id=0, beam_n=2, seg_s=3, max_utts=1, max_frames_total=50,
                pred_layers=1, pred_hidden=64, pred_embed=64, act=0, dtype=0)
    for bad in (dict(beam_n=0), dict(beam_n=33), dict(seg_s=0), dict(vocab=1), dict(blank_id=32),
                dict(pred_layers=5), dict(dtype=2), dict(act=3), dict(max_utts=0), dict(dtype=1, d_joint=60),
                dict(stream_buffer_frames=2), dict(stream_buffer_frames=-1)):
        c = tbs._Config(**{**good, **bad})
        assert L.tbs_init(C.byref(c), C.byref(w), C.byref(ctx)) == -1, bad
        assert not ctx.value
    # good shape but null weight pointers
    c = tbs._Config(**good)
    assert L.tbs_init(C.byref(c), C.byref(w), C.byref(ctx)) == -1
    # null context on every entry point
    assert L.tbs_joiner_segment(None) == -1 and L.tbs_expand(None) == -1
    assert L.tbs_select_merge(None, None) == -1 and L.tbs_predictor_step(None) == -1
    assert L.tbs_gemm_bf16(None, None, None, None, 1, 1, 8, 0, None) == -1
    assert L.tbs_stream_begin(None, 1) == -1 and L.tbs_push_segment(None, None, None, 0) == -1
    L.tbs_free(None)


def test_binding_has_no_oracle_or_cpu_path():
    """The product package must not import the oracle."""
    import paper_2302_14357_amd
    pkg = os.path.dirname(paper_2302_14357_amd.__file__)
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text and "liborc" not in text, f
