"""Seeded synthetic inputs for token-wise RNN-T beam search.

This module is the only code shared by the CPU oracle and the HIP path.  It
draws model weights, utterance lengths and encoder frames from fixed seeds and
hands them out as plain numpy arrays.  It holds none of the search arithmetic
(no joiner, no softmax, no expansion scores, no selection): the one matrix
product here is the encoder-side projection of raw frames into the joint
space, which the paper treats as part of the pre-computed encoder output
(Section 3.2, last paragraphs: the encoder output is assumed to be available
before decoding starts).

The inputs stand in for the paper's Librispeech and in-house test sets and
trained models (Section 4.1), none of which are available: shapes, vocabulary
sizes and length mixes follow the benchmark configurations, weights are
Xavier-uniform, frames are i.i.d. normal, and the blank logit carries a bias so
that blank is the most likely single symbol, as it is for a trained model.
"""

from .shapes import TbsShape, SHAPES, shape_by_name
from .generate import (
    round_to_bf16,
    make_model,
    make_utterances,
    make_table_logits,
    SEED_WEIGHTS,
    SEED_FRAMES,
    SEED_LENGTHS,
)

__all__ = [
    "TbsShape",
    "SHAPES",
    "shape_by_name",
    "round_to_bf16",
    "make_model",
    "make_utterances",
    "make_table_logits",
    "SEED_WEIGHTS",
    "SEED_FRAMES",
    "SEED_LENGTHS",
]
