#!/usr/bin/env python3
"""Benchmark of the token-wise RNN-T beam-search hot path on one MI355X.

One "step" = one whole decode (Algorithm 1, all segments and rounds: joiner,
softmax statistics, Eq. 3-7 expansion scores, selection/merge, predictor) of
one synthetic batch whose projected encoder frames are already resident in
HBM.  Prints ONE JSON line: decoded frames/s, the roofline figures of the
dominant kernel measured with HIP events inside this run, and the CPU oracle
timed on a bounded sample of the same workload.
"""

from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# MI355X published peaks
PEAK_BF16_TFLOPS = 2500.0
PEAK_HBM_GBS = 8000.0

WORKLOADS = {
    # name: (shape, N, S, utterances (None = the shape's own), oracle sample utterances)
    "librispeech": ("librispeech", 5, 3, None, 32),
    "assistant": ("assistant", 10, 3, None, 8),
    "throughput": ("throughput", 10, 5, None, 8),
    "tiny": ("tiny", 2, 3, None, 1),
}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="librispeech", choices=sorted(WORKLOADS))
    ap.add_argument("--beam", type=int, default=0)
    ap.add_argument("--seg", type=int, default=0)
    ap.add_argument("--utts", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-timing", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (each utterance is an independent search; "
              "a second GPU would only take a share of the utterances). --gpus must be 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    from tbs_inputs import SHAPES, make_model, make_utterances
    from paper_2302_14357_amd import Tbs, KERNEL

    shape_name, N, S, U, cpu_utts = WORKLOADS[args.workload]
    N = args.beam or N
    S = args.seg or S
    shape = SHAPES[shape_name]
    if args.utts:
        shape = shape.with_utts(args.utts)
    model = make_model(shape)
    offsets, enc = make_utterances(shape, model)
    U = len(offsets) - 1
    frames = int(offsets[-1])

    tbs = Tbs(model, blank_id=shape.blank_id, beam_n=N, seg_s=S, max_utts=U, max_frames_total=frames,
              dtype=shape.dtype, act=shape.act)
    enc_dev = tbs.upload_frames(enc)           # inputs resident in HBM before the timed region
    max_len = 256
    tok = np.full((U, N, max_len), -1, np.int32)
    lens = np.zeros((U, N), np.int32)
    logs = np.zeros((U, N), np.float64)
    cnt = np.zeros(U, np.int32)

    def step():
        rc = tbs.decode_raw(enc_dev, offsets, tok, lens, logs, cnt, max_len)
        if rc != 0:
            raise RuntimeError(f"tbs_decode failed with {rc}")

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    value = frames / (ms_per_step / 1e3)
    stats = tbs.stats()

    # ---- per-kernel timing with HIP events on the library's stream (separate, untimed passes)
    kernels = {}
    roofline = None
    if not args.no_kernel_timing:
        H, E, Dj, V, L = shape.pred_hidden, shape.pred_embed, shape.d_joint, shape.vocab, shape.pred_layers
        # bf16 models take the embedding half of layer 0 from a table made at init: no flops per round
        in0 = 0 if shape.dtype == "bf16" else E
        pred_flops_per_hyp = sum(2 * 4 * H * ((in0 if l == 0 else H) + H) for l in range(L)) + 2 * H * Dj
        for name, kid in (("joiner_gemm", KERNEL.JOINER), ("joiner_prep", KERNEL.PREP), ("expand", KERNEL.EXPAND),
                          ("select_merge", KERNEL.SELECT), ("predictor", KERNEL.PREDICTOR)):
            tbs.profile_select(kid)
            step()
            r = tbs.profile_read()
            kernels[name] = r
        tbs.profile_select(-1)
        for name, r in kernels.items():
            n, ms, units = max(r["launches"], 1), r["total_ms"], r["units"]
            r["avg_us"] = ms / n * 1e3
            if name == "joiner_gemm":
                r.update(bound="mfma", unit="TFLOP/s", peak=PEAK_BF16_TFLOPS,
                         achieved=(2.0 * units * Dj * V) / (ms * 1e-3) / 1e12 if ms > 0 else 0.0)
            elif name == "expand":
                r.update(bound="hbm", unit="GB/s", peak=PEAK_HBM_GBS,
                         achieved=(units * V * 4.0) / (ms * 1e-3) / 1e9 if ms > 0 else 0.0)
            elif name == "joiner_prep":
                per_row = Dj * (2 + 4 + 2) if shape.dtype == "bf16" else Dj * 12
                r.update(bound="hbm", unit="GB/s", peak=PEAK_HBM_GBS,
                         achieved=(units * per_row) / (ms * 1e-3) / 1e9 if ms > 0 else 0.0)
            elif name == "predictor":
                r.update(bound="mfma", unit="TFLOP/s", peak=PEAK_BF16_TFLOPS,
                         achieved=(units * pred_flops_per_hyp) / (ms * 1e-3) / 1e12 if ms > 0 else 0.0)
            else:
                r.update(bound="hbm", unit="GB/s", peak=PEAK_HBM_GBS, achieved=0.0)
            r["frac"] = r["achieved"] / r["peak"]
        dom = max(("joiner_gemm", "expand", "predictor"), key=lambda k: kernels[k]["total_ms"])
        d = kernels[dom]
        roofline = {"kernel": dom, "bound": d["bound"], "achieved": d["achieved"], "peak": d["peak"],
                    "unit": d["unit"], "frac": d["frac"], "traffic": None, "avg_us": d["avg_us"],
                    "launches": d["launches"]}

    # ---- CPU oracle on a bounded sample of the same workload
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        W = oracle.LstmWeights(model, shape.blank_id, act=shape.act, quant_bf16=(shape.dtype == "bf16"))
        nu = min(cpu_utts, U)
        sub_off = offsets[:nu + 1].copy()
        sub_enc = enc[:sub_off[-1]]
        threads = oracle.max_threads()
        t0 = time.perf_counter()
        _, used = oracle.decode_lstm_batch(W, sub_enc, sub_off, N, S, threads=threads)
        ct = time.perf_counter() - t0
        cpu = {"value": float(sub_off[-1]) / ct, "unit": "frames/s", "cores": int(min(used, nu)), "kind": "oracle",
               "sample": f"first {nu} of {U} utterances ({int(sub_off[-1])} frames), fp64 C oracle, "
                         f"OpenMP over utterances, {ct:.1f} s"}

    out = {
        "metric": "decoded_frames_per_sec",
        "value": value,
        "unit": "frames/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if shape.dtype == "bf16" else "f32",
        "data": "synthetic",
        "config": {"workload": f"{shape.name}-like: {U} utterances, {frames} frames, Dj={shape.d_joint}, "
                               f"V={shape.vocab}, LSTM {shape.pred_layers}x{shape.pred_hidden}, N={N}, S={S}",
                   "beam_n": N, "seg_s": S, "utterances": U, "frames": frames},
        "calls_per_frame": stats["joiner_calls"] / max(frames, 1),
        "joins_per_frame": stats["joined_frames"] / max(frames, 1),
        "joiner_launches_per_step": stats["launches"],
        "roofline": roofline,
        "cpu_baseline": cpu,
        "kernels": kernels,
    }
    tbs.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
