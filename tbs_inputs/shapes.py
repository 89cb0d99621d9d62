"""Workload shapes.  Each entry fixes the tensor sizes of one benchmark
configuration; beam size N and segment size S are chosen by the caller."""

from dataclasses import dataclass, replace


@dataclass(frozen=True)
class TbsShape:
    name: str
    index: int            # added to the seeds so configurations draw distinct streams
    n_utts: int           # U
    len_lo: int           # utterance lengths are uniform on [len_lo, len_hi] frames
    len_hi: int
    d_enc: int            # raw encoder frame width before projection
    d_joint: int          # Dj: width of the joint space
    vocab: int            # V, including blank
    blank_id: int
    pred_layers: int      # LSTM layers of the prediction network
    pred_hidden: int
    pred_embed: int       # token embedding width (first LSTM layer input)
    dtype: str            # "f32" or "bf16": storage type of weights and projected frames
    act: str = "tanh"     # joiner activation: "tanh" or "relu"
    blank_bias: float = 3.0
    logit_scale: float = 1.0   # multiplies the Xavier draw of the joiner output matrix: > 1 gives peaked output
                               # distributions (as a trained model has), so that hypotheses grow to many tokens

    def with_utts(self, n_utts: int) -> "TbsShape":
        return replace(self, n_utts=n_utts)


SHAPES = {
    # 1 utterance of 50 frames, everything 64 wide, V=32, fp32
    "tiny": TbsShape("tiny", 0, 1, 50, 50, 64, 64, 32, 0, 1, 64, 64, "f32"),
    # 64 utterances of 150-400 frames, Dj=512, V=1024, LSTM 1x640
    "librispeech": TbsShape("librispeech", 1, 64, 150, 400, 512, 512, 1024, 0, 1, 640, 640, "bf16"),
    # 256 utterances of 100-600 frames, Dj=1024, V=4096, LSTM 2x1024
    "assistant": TbsShape("assistant", 2, 256, 100, 600, 1024, 1024, 4096, 0, 2, 1024, 1024, "bf16"),
    # 1024 utterances of exactly 300 frames, Dj=1024, V=4096, LSTM 1x1024
    "throughput": TbsShape("throughput", 4, 1024, 300, 300, 1024, 1024, 4096, 0, 1, 1024, 1024, "bf16"),
}


def shape_by_name(name: str) -> TbsShape:
    if name not in SHAPES:
        raise KeyError(f"unknown shape {name!r}; have {sorted(SHAPES)}")
    return SHAPES[name]
