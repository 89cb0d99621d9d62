"""Seeded generators: model weights, utterance lengths, projected encoder frames.

All matrices are laid out [out_features, in_features], row-major, so that the
reduction index is the contiguous one.  Everything is returned as float32 numpy
arrays; for "bf16" shapes every value is already rounded to a bf16-representable
number (round-to-nearest-even), so that converting to a bf16 tensor is exact and
the oracle (which reads the same arrays as float64) sees the same data.
"""

from __future__ import annotations

import numpy as np

from .shapes import TbsShape

SEED_WEIGHTS = 1234
SEED_FRAMES = 2345
SEED_LENGTHS = 3456


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16-representable float32
    (ties to even), by integer arithmetic on the bit pattern."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32).astype(np.uint64)
    lsb = (bits >> 16) & 1
    rounded = (bits + 0x7FFF + lsb) & 0xFFFF0000
    out = rounded.astype(np.uint32).view(np.float32).reshape(x.shape)
    # keep NaN/inf as they were (not expected in these inputs)
    bad = ~np.isfinite(x)
    if bad.any():
        out = out.copy()
        out[bad] = x[bad]
    return out


def _xavier(rng: np.random.Generator, out_f: int, in_f: int) -> np.ndarray:
    bound = np.sqrt(6.0 / (in_f + out_f))
    return rng.uniform(-bound, bound, size=(out_f, in_f)).astype(np.float32)


def _small(rng: np.random.Generator, n: int, scale: float = 0.05) -> np.ndarray:
    return rng.uniform(-scale, scale, size=(n,)).astype(np.float32)


def make_model(shape: TbsShape, seed: int = SEED_WEIGHTS) -> dict:
    """Weights of the joiner, the LSTM prediction network and the two
    projections into the joint space.  Keys:

    w_enc [Dj, D_enc], b_enc [Dj]      encoder-side projection (used by make_utterances)
    w_out [V, Dj], b_out [V]           joiner output layer; b_out[blank] carries the blank bias
    embed [V, E]                       token embedding
    lstm  list of (w_ih [4H, in], w_hh [4H, H], b [4H]), gate order i, f, g, o
    w_proj [Dj, H], b_proj [Dj]        predictor-side projection
    pred_init [Dj]                     predictor output of the empty hypothesis
    """
    rng = np.random.default_rng([seed, shape.index])
    H, E, Dj, V = shape.pred_hidden, shape.pred_embed, shape.d_joint, shape.vocab
    m = {}
    m["w_enc"] = _xavier(rng, Dj, shape.d_enc)
    m["b_enc"] = _small(rng, Dj)
    m["w_out"] = _xavier(rng, V, Dj) * np.float32(shape.logit_scale)
    b_out = _small(rng, V)
    b_out[shape.blank_id] += np.float32(shape.blank_bias)
    m["b_out"] = b_out
    m["embed"] = _xavier(rng, V, E)
    lstm = []
    for layer in range(shape.pred_layers):
        in_f = E if layer == 0 else H
        lstm.append((_xavier(rng, 4 * H, in_f), _xavier(rng, 4 * H, H), _small(rng, 4 * H)))
    m["lstm"] = lstm
    m["w_proj"] = _xavier(rng, Dj, H)
    m["b_proj"] = _small(rng, Dj)
    m["pred_init"] = _xavier(rng, 1, Dj).reshape(Dj)
    if shape.dtype == "bf16":
        for k in ("w_enc", "w_out", "embed", "w_proj"):
            m[k] = round_to_bf16(m[k])
        m["lstm"] = [(round_to_bf16(a), round_to_bf16(b), c) for (a, b, c) in m["lstm"]]
    return m


def make_utterances(shape: TbsShape, model: dict, seed_frames: int = SEED_FRAMES,
                    seed_lengths: int = SEED_LENGTHS, n_utts: int | None = None,
                    lengths: np.ndarray | None = None):
    """Utterance lengths and projected encoder frames.

    Returns (frame_offsets int32 [U+1], enc_proj float32 [sum T_u, Dj]).
    Raw frames are i.i.d. N(0,1) of width d_enc; enc_proj = frames @ w_enc^T + b_enc,
    rounded to bf16 values for bf16 shapes.  Each utterance draws from its own
    stream (seeded by its index), so utterance u has the same frames whatever
    the batch it is generated in.
    """
    U = shape.n_utts if n_utts is None else n_utts
    if lengths is None:
        lrng = np.random.default_rng([seed_lengths, shape.index])
        lengths = lrng.integers(shape.len_lo, shape.len_hi + 1, size=U)
    lengths = np.asarray(lengths, dtype=np.int64)
    assert lengths.shape == (U,)
    offsets = np.zeros(U + 1, dtype=np.int32)
    offsets[1:] = np.cumsum(lengths)
    total = int(offsets[-1])
    enc = np.empty((total, shape.d_joint), dtype=np.float32)
    w = model["w_enc"].astype(np.float32)
    b = model["b_enc"].astype(np.float32)
    for u in range(U):
        T = int(lengths[u])
        if T == 0:
            continue
        frng = np.random.default_rng([seed_frames, shape.index, u])
        raw = frng.standard_normal(size=(T, shape.d_enc), dtype=np.float32)
        enc[offsets[u]:offsets[u + 1]] = raw @ w.T + b
    if shape.dtype == "bf16":
        enc = round_to_bf16(enc)
    return offsets, enc


def make_table_logits(seed: int, frame: int, tokens, vocab: int, blank_id: int = 0,
                      blank_bias: float = 0.0, scale: float = 1.5) -> np.ndarray:
    """Logits of a toy transducer whose joiner output is an arbitrary fixed
    function of (frame, token tuple): N(0, scale^2) draws from a stream keyed
    by the frame and the tokens.  Used to pin the search algebra without any
    network in the loop."""
    key = [int(seed), int(frame), len(tokens)] + [int(t) for t in tokens]
    rng = np.random.default_rng(key)
    out = rng.standard_normal(vocab) * scale
    out[blank_id] += blank_bias
    return out
