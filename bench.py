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


def read_traffic(kernel, workload):
    """HBM bytes per launch of the dominant kernel, from the committed rocprofv3 counter summary
    (FETCH_SIZE + WRITE_SIZE, scaled by a copy kernel of known size); None if there is none."""
    path = os.path.join(ROOT, "profiles", f"traffic_{kernel}_{workload}.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":", 1)[1])
    except OSError:
        pass
    return None


def quick_decode(workload, steps=2, warmup=1, seg=0, beam=0, debug=0):
    """frames/s of another configuration's whole decode (tbs_decode, inputs resident in HBM), timed
    like the headline but over a couple of steps: reported beside the headline, not as `value`."""
    import torch
    from tbs_inputs import SHAPES, make_model, make_utterances
    from paper_2302_14357_amd import Tbs
    shape_name, N, S, _, _ = WORKLOADS[workload]
    N, S = beam or N, seg or S
    shape = SHAPES[shape_name]
    model = make_model(shape)
    offsets, enc = make_utterances(shape, model)
    U, frames = len(offsets) - 1, int(offsets[-1])
    t = Tbs(model, blank_id=shape.blank_id, beam_n=N, seg_s=S, max_utts=U, max_frames_total=frames,
            dtype=shape.dtype, act=shape.act, debug=debug)
    try:
        enc_dev = t.upload_frames(enc)
        max_len = 256
        tok = np.full((U, N, max_len), -1, np.int32)
        lens, logs, cnt = np.zeros((U, N), np.int32), np.zeros((U, N), np.float64), np.zeros(U, np.int32)
        for _ in range(warmup):
            if t.decode_raw(enc_dev, offsets, tok, lens, logs, cnt, max_len):
                raise RuntimeError("decode failed")
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            if t.decode_raw(enc_dev, offsets, tok, lens, logs, cnt, max_len):
                raise RuntimeError("decode failed")
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) / steps * 1e3
        st = t.stats()
        path = t.path()
        return {"workload": f"{shape.name}-like: {U} utterances, {frames} frames, Dj={shape.d_joint}, V={shape.vocab}, "
                            f"LSTM {shape.pred_layers}x{shape.pred_hidden}, N={N}, S={S}",
                "kernels": ("four kernels a round, hypotheses in fixed places" if path["fixed_places"] else
                            "row lists, kernels sized by the round's rows") +
                           ("; joiner GEMM keeps row softmax sums and best tokens, no logits" if path["one_frame_no_logits"] else ""),
                "frames_per_sec": frames / (ms / 1e3), "ms_per_step": ms, "steps": steps,
                "calls_per_frame": st["joiner_calls"] / max(frames, 1),
                "joins_per_frame": st["joined_frames"] / max(frames, 1), "joiner_launches_per_step": st["launches"]}
    finally:
        t.close()


def measure_at_scale(iters=6, chunk_rows=0):
    """One joiner + expansion call on the shape of the largest configuration (1024 utterances,
    N=10, S=5, Dj=1024, V=4096: 51200 joiner rows, a full beam everywhere), where the two kernels
    are throughput-bound: the figures the roofline targets are stated for."""
    import dataclasses
    from tbs_inputs import SHAPES, make_model, make_utterances
    from paper_2302_14357_amd import Tbs, BUF, KERNEL
    U, N, S = 1024, 10, 5
    shape = dataclasses.replace(SHAPES["throughput"], len_lo=S, len_hi=S)
    model = make_model(shape)
    offsets, enc = make_utterances(shape, model)
    t = Tbs(model, blank_id=shape.blank_id, beam_n=N, seg_s=S, max_utts=U, max_frames_total=int(offsets[-1]),
            dtype=shape.dtype, act=shape.act, joiner_chunk_rows=chunk_rows)
    try:
        enc_dev = t.upload_frames(enc)
        rng = np.random.default_rng(0)
        t.begin(enc_dev, offsets)
        t.debug_write(BUF.A_COUNT, np.full(U, N, np.int32))
        t.debug_write(BUF.A_LOGS, -rng.random((U, N)) * 10)
        t.debug_write(BUF.A_PRED, (rng.standard_normal((U, N, shape.d_joint)) * 0.5).astype(np.float32))
        dh = rng.random((U, N, S)).astype(np.float32)
        t.debug_write(BUF.A_DHAT, dh / dh.sum(-1, keepdims=True))
        out = {"workload": f"one joiner + expansion call, {U} utterances x {N} hypotheses x {S} frames, "
                           f"Dj={shape.d_joint}, V={shape.vocab}"}
        for name, kid in (("joiner_gemm", KERNEL.JOINER), ("expand", KERNEL.EXPAND), ("joiner_prep", KERNEL.PREP)):
            t.profile_select(kid)
            rows = 0
            for _ in range(iters):
                rows = t.debug_rebuild(0)
                t.joiner_segment()
                t.expand()
            r = t.profile_read()
            # a call this large runs in pieces (one GEMM and one expansion launch per piece): the
            # figures are per launch, work and time summed over all launches of the family
            n, sec, units = max(r["launches"], 1), r["total_ms"] * 1e-3, r["units"]
            us = sec / n * 1e6
            if name == "joiner_prep":
                out[name] = {"avg_us": us, "launches_per_call": n / iters, "us_per_call": sec / iters * 1e6}
            elif name == "joiner_gemm":
                ach = 2.0 * units * shape.d_joint * shape.vocab / sec / 1e12
                out[name] = {"bound": "mfma", "achieved": ach, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                             "frac": ach / PEAK_BF16_TFLOPS, "avg_us": us, "rows_per_call": rows,
                             "launches_per_call": n / iters, "us_per_call": sec / iters * 1e6,
                             "traffic": read_traffic("gemm", "at_scale")}
            else:
                ach = units * shape.vocab * 4.0 / sec / 1e9
                out[name] = {"bound": "hbm", "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                             "frac": ach / PEAK_HBM_GBS, "avg_us": us, "rows_per_call": rows,
                             "launches_per_call": n / iters, "us_per_call": sec / iters * 1e6,
                             "traffic": read_traffic("expand", "at_scale")}
        t.profile_select(-1)
        return out
    finally:
        t.close()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--workload", default="librispeech", choices=sorted(WORKLOADS))
    ap.add_argument("--beam", type=int, default=0)
    ap.add_argument("--seg", type=int, default=0)
    ap.add_argument("--utts", type=int, default=0)
    ap.add_argument("--stream-piece", type=int, default=0,
                    help="decode through tbs_push_segment, every utterance receiving this many frames per "
                         "push (0 = tbs_decode on whole utterances, the headline)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="skip the short decodes of the other configurations reported beside the headline")
    ap.add_argument("--debug", type=int, default=0, help="tbs_config.debug of the timed context (kernel variants)")
    ap.add_argument("--no-kernel-timing", action="store_true")
    ap.add_argument("--at-scale-only", action="store_true",
                    help="only the joiner + expansion call on the largest configuration's shape (for profiling)")
    ap.add_argument("--chunk-rows", type=int, default=0,
                    help="joiner_chunk_rows of the library (0 = joiner calls are not split)")
    ap.add_argument("--calibrate", action="store_true",
                    help="also run one device copy of 256 MiB (the yardstick for the rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (each utterance is an independent search; "
              "a second GPU would only take a share of the utterances). --gpus must be 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    from tbs_inputs import SHAPES, make_model, make_utterances
    from paper_2302_14357_amd import Tbs, KERNEL

    if args.calibrate:   # reads 256 MiB and writes 256 MiB: torch's elementwise copy kernel
        src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if args.at_scale_only:
        print(json.dumps({"roofline_at_scale": measure_at_scale(chunk_rows=args.chunk_rows)}))
        return

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

    piece = args.stream_piece
    tbs = Tbs(model, blank_id=shape.blank_id, beam_n=N, seg_s=S, max_utts=U, max_frames_total=frames,
              dtype=shape.dtype, act=shape.act, stream_buffer_frames=(piece + S) if piece else 0,
              joiner_chunk_rows=args.chunk_rows, debug=args.debug,
              rounds_capacity=(4 * S if S > 16 else 0))   # (a long segment can take more rounds than the default 32)
    enc_dev = tbs.upload_frames(enc)           # inputs resident in HBM before the timed region
    max_len = 256
    tok = np.full((U, N, max_len), -1, np.int32)
    lens = np.zeros((U, N), np.int32)
    logs = np.zeros((U, N), np.float64)
    cnt = np.zeros(U, np.int32)

    pushes = []
    if piece:   # the pieces of every push, resident in HBM like the whole utterances of the headline
        T = np.diff(offsets)
        for start in range(0, int(T.max()), piece):
            n = np.clip(T - start, 0, piece)
            idx = np.concatenate([np.arange(offsets[u] + start, offsets[u] + start + n[u]) for u in range(U)])
            pushes.append((enc_dev[torch.from_numpy(idx).to(enc_dev.device)].contiguous(),
                           np.concatenate([[0], np.cumsum(n)]).astype(np.int32)))
        torch.cuda.synchronize()
        args.no_kernel_timing = args.no_cpu_baseline = True

    def step():
        if piece:
            tbs.stream_begin(U)
            for i, (e, off) in enumerate(pushes):
                tbs.push_segment(e, off, flush=(i + 1 == len(pushes)))
            rc = tbs.L.tbs_result(tbs.ctx, tok.ctypes.data, lens.ctypes.data, logs.ctypes.data, cnt.ctypes.data, max_len)
        else:
            rc = tbs.decode_raw(enc_dev, offsets, tok, lens, logs, cnt, max_len)
        if rc != 0:
            raise RuntimeError(f"decode failed with {rc}")

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
    at_scale = None
    if not args.no_kernel_timing:
        H, E, Dj, V, L = shape.pred_hidden, shape.pred_embed, shape.d_joint, shape.vocab, shape.pred_layers
        bf16 = shape.dtype == "bf16"
        # (small batches run expansion + select/merge as one kernel, "round"; timing "expand" or
        # "select_merge" there reads nothing, or the two-kernel form where the batch keeps row lists)
        for name, kid in (("gemm", KERNEL.GEMM), ("joiner_gemm", KERNEL.JOINER), ("joiner_prep", KERNEL.PREP),
                          ("round", KERNEL.ROUND), ("expand", KERNEL.EXPAND), ("select_merge", KERNEL.SELECT),
                          ("predictor", KERNEL.PREDICTOR)):
            tbs.profile_select(kid)
            step()
            r = tbs.profile_read()
            if r["launches"]:
                kernels[name] = r
        tbs.profile_select(-1)
        event_cost = tbs.profile_overhead(200)
        for name, r in kernels.items():
            n, ms, units = max(r["launches"], 1), r["total_ms"], r["units"]
            sec = ms * 1e-3
            r["avg_us"] = ms / n * 1e3
            if name == "gemm":            # every launch of the GEMM kernel (joiner and predictor); units = M*N*K
                r.update(bound="mfma", unit="TFLOP/s", peak=PEAK_BF16_TFLOPS if bf16 else 157.3,
                         achieved=2.0 * units / sec / 1e12 if ms > 0 else 0.0)
            elif name == "joiner_gemm":   # units = joiner rows
                r.update(bound="mfma", unit="TFLOP/s", peak=PEAK_BF16_TFLOPS if bf16 else 157.3,
                         achieved=2.0 * units * Dj * V / sec / 1e12 if ms > 0 else 0.0)
            elif name == "expand":        # algorithmic bytes: every logit read once
                r.update(bound="hbm", unit="GB/s", peak=PEAK_HBM_GBS, achieved=units * V * 4.0 / sec / 1e9 if ms > 0 else 0.0)
            elif name == "joiner_prep":   # one encoder row (2 B/elt) + one predictor row (4 B) in, one bf16 row out
                per_row = Dj * (2 + 4 + 2) if bf16 else Dj * 12
                r.update(bound="hbm", unit="GB/s", peak=PEAK_HBM_GBS, achieved=units * per_row / sec / 1e9 if ms > 0 else 0.0)
            else:                         # kernel groups with no single roofline
                r.update(bound=None, unit=None, peak=None, achieved=None)
            r["frac"] = r["achieved"] / r["peak"] if r["peak"] else None
        # the dominant single kernel of this workload: the GEMM kernel (three launches a round) or
        # the expansion kernel, whichever took longer in total
        dom = max((k for k in ("gemm", "expand") if k in kernels), key=lambda k: kernels[k]["total_ms"])
        d = kernels[dom]
        roofline = {"kernel": {"gemm": "k_gemm_small / k_gemm_bf16 (all launches)", "expand": "k_expand_reg"}[dom],
                    "bound": d["bound"], "achieved": d["achieved"], "peak": d["peak"], "unit": d["unit"],
                    "frac": d["frac"], "traffic": read_traffic(dom, args.workload), "avg_us": d["avg_us"],
                    "launches": d["launches"],
                    "note": "achieved = summed algorithmic work / summed HIP-event durations over every launch of "
                            "the kernel in one decode; an event pair reads event_pair_around_empty_kernel_us around "
                            "a kernel that does nothing, so microsecond kernels read long (profiles/ has the "
                            "kernels' own durations); a problem of at most 1 GFLOP per launch is latency-bound: "
                            "the throughput-bound figures are roofline_at_scale",
                    # the same event pair around a kernel that does nothing: what events add to every
                    # launch of a microsecond-scale kernel (a kernel trace shows that kernel's own time)
                    "event_pair_around_empty_kernel_us": event_cost}
        at_scale = measure_at_scale()

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
        # and on one core (the paper's CPU figures are single-core), on a smaller sample
        n1 = min(2, nu)
        one_off = offsets[:n1 + 1].copy()
        t0 = time.perf_counter()
        oracle.decode_lstm_batch(W, enc[:one_off[-1]], one_off, N, S, threads=1)
        c1 = time.perf_counter() - t0
        cpu["single_core"] = {"value": float(one_off[-1]) / c1, "unit": "frames/s", "cores": 1,
                              "sample": f"first {n1} utterances ({int(one_off[-1])} frames), {c1:.1f} s"}

    # ---- the other configurations, briefly (not `value`): the large-assistant and throughput shapes,
    # and the headline shapes at S = 1, i.e. the standard breadth-first search the method generalises
    others = None
    if not args.no_other_workloads and not piece and args.workload == "librispeech":
        tbs.close()
        others = {"librispeech_s1_standard_search": quick_decode("librispeech", steps=4, warmup=1, seg=1),
                  "librispeech_s1_standard_search_no_logits": quick_decode("librispeech", steps=4, warmup=1, seg=1,
                                                                           debug=32768),
                  "assistant_n10_s3": quick_decode("assistant", steps=2, warmup=1),
                  "throughput_n10_s5": quick_decode("throughput", steps=2, warmup=1)}

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
                   "beam_n": N, "seg_s": S, "utterances": U, "frames": frames,
                   "entry": f"tbs_push_segment, {piece} frames per utterance and push" if piece else "tbs_decode"},
        "calls_per_frame": stats["joiner_calls"] / max(frames, 1),
        "joins_per_frame": stats["joined_frames"] / max(frames, 1),
        "joiner_launches_per_step": stats["launches"],
        "roofline": roofline,
        "roofline_at_scale": at_scale,
        "other_workloads": others,
        "cpu_baseline": cpu,
        "kernels": kernels,
    }
    tbs.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
