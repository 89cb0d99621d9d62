"""ctypes binding of libtbs.so (include/tbs.h).  Argument marshalling only."""

from __future__ import annotations

import ctypes as C
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libtbs.so")

EXPORTED_SYMBOLS = [
    "tbs_init", "tbs_free", "tbs_begin", "tbs_segment_begin", "tbs_joiner_segment", "tbs_expand",
    "tbs_select_merge", "tbs_predictor_step", "tbs_decode", "tbs_result", "tbs_stats", "tbs_debug_read",
    "tbs_debug_write", "tbs_debug_rebuild", "tbs_debug_hyps", "tbs_profile_select", "tbs_profile_read",
    "tbs_strerror", "tbs_last_hip_error", "tbs_gemm_bf16", "tbs_stream_begin", "tbs_push_segment",
    "tbs_profile_overhead", "tbs_debug_hyps_noalloc", "tbs_path",
]

TBS_MAX_LAYERS = 4


class BUF:
    A_COUNT, A_LOGS, A_DHAT, A_PRED, LOGITS, ROW_STATS, DELTA_BLANK, DELTA_NB = range(8)
    CAND_SCORE, CAND_TOKEN, PAIR_UTT, PAIR_HYP, PAIR_ROW0, PAIR_LEN, COUNTS = range(8, 15)


class KERNEL:
    JOINER, EXPAND, SELECT, PREDICTOR, PREP, GEMM, ROUND = range(7)


class TbsError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"tbs error {code}: {msg}")
        self.code = code


class _Config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "d_joint", "vocab", "blank_id", "beam_n", "seg_s", "max_utts", "max_frames_total", "pred_layers",
        "pred_hidden", "pred_embed", "act", "dtype", "max_rounds_per_segment", "rounds_capacity", "max_nodes",
        "debug", "stream_buffer_frames", "max_result_len", "joiner_chunk_rows", "device_id")] + [("stream", C.c_void_p)]


class _Weights(C.Structure):
    _fields_ = [("w_out", C.c_void_p), ("b_out", C.c_void_p), ("embed", C.c_void_p),
                ("w_ih", C.c_void_p * TBS_MAX_LAYERS), ("w_hh", C.c_void_p * TBS_MAX_LAYERS),
                ("b_lstm", C.c_void_p * TBS_MAX_LAYERS),
                ("w_proj", C.c_void_p), ("b_proj", C.c_void_p), ("pred_init", C.c_void_p)]


_lib = None


def load_library():
    """Load libtbs.so; raises if it has not been built (there is no fallback)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2302_14357_amd.build` "
                          "(there is no CPU fallback)")
    # PyTorch owns the device memory handed to the library, so both must share one
    # HIP runtime: torch is imported first and libtbs then binds to the runtime
    # torch has already loaded (two runtimes in one process do not see each
    # other's allocations).
    import torch  # noqa: F401
    L = C.CDLL(LIB_PATH)
    vp, i32, i64p = C.c_void_p, C.c_int32, C.POINTER(C.c_int64)
    L.tbs_init.argtypes = [C.POINTER(_Config), C.POINTER(_Weights), C.POINTER(vp)]
    L.tbs_free.argtypes = [vp]
    L.tbs_free.restype = None
    L.tbs_begin.argtypes = [vp, vp, vp, i32]
    L.tbs_segment_begin.argtypes = [vp, i32, C.POINTER(i32)]
    L.tbs_joiner_segment.argtypes = [vp]
    L.tbs_expand.argtypes = [vp]
    L.tbs_select_merge.argtypes = [vp, C.POINTER(i32)]
    L.tbs_predictor_step.argtypes = [vp]
    L.tbs_decode.argtypes = [vp, vp, vp, i32, vp, vp, vp, vp, i32]
    L.tbs_result.argtypes = [vp, vp, vp, vp, vp, i32]
    L.tbs_stream_begin.argtypes = [vp, i32]
    L.tbs_push_segment.argtypes = [vp, vp, vp, i32]
    L.tbs_stats.argtypes = [vp, i64p, i64p, i64p, i64p]
    L.tbs_path.argtypes = [vp]
    L.tbs_debug_read.argtypes = [vp, i32, vp, C.c_size_t]
    L.tbs_debug_write.argtypes = [vp, i32, vp, C.c_size_t]
    L.tbs_debug_rebuild.argtypes = [vp, i32, C.POINTER(i32)]
    L.tbs_debug_hyps.argtypes = [vp, i32, vp, vp, vp, vp, i32, i32]
    L.tbs_debug_hyps_noalloc.argtypes = [vp, i32, vp, vp, vp, vp, i32, i32]
    L.tbs_profile_select.argtypes = [vp, i32]
    L.tbs_profile_read.argtypes = [vp, i64p, C.POINTER(C.c_double), i64p]
    L.tbs_profile_overhead.argtypes = [vp, i32, C.POINTER(C.c_double)]
    L.tbs_strerror.argtypes = [C.c_int]
    L.tbs_strerror.restype = C.c_char_p
    L.tbs_last_hip_error.argtypes = [vp]
    L.tbs_gemm_bf16.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, vp]
    _lib = L
    return L


def _check(rc, ctx=None):
    if rc != 0:
        L = load_library()
        msg = L.tbs_strerror(rc).decode()
        if rc == -4 and ctx is not None:
            msg += f" (hipError {L.tbs_last_hip_error(ctx)})"
        raise TbsError(rc, msg)


def _hp(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


class Tbs:
    """One decoding context (fixed model, beam size N and segment size S)."""

    def __init__(self, model: dict, *, blank_id: int, beam_n: int, seg_s: int, max_utts: int,
                 max_frames_total: int, dtype: str = "bf16", act: str = "tanh", max_rounds_per_segment: int = 0,
                 rounds_capacity: int = 0, max_nodes: int = 0, debug: int = 0, stream_buffer_frames: int = 0,
                 max_result_len: int = 0, joiner_chunk_rows: int = 0, device: int = 0, stream=None):
        import torch
        self.torch = torch
        self.L = load_library()
        if not torch.cuda.is_available():
            raise RuntimeError("tbs needs a GPU: torch.cuda.is_available() is False")
        self.device = torch.device("cuda", device)
        self.dtype = dtype
        mat = torch.bfloat16 if dtype == "bf16" else torch.float32
        self.mat_dtype = mat

        def dev(a, dt):
            return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(self.device).to(dt).contiguous()

        V, Dj = model["w_out"].shape
        H = model["w_proj"].shape[1]
        E = model["embed"].shape[1]
        L_ = len(model["lstm"])
        self.V, self.Dj, self.H, self.E, self.layers = V, Dj, H, E, L_
        self.N, self.S, self.max_utts = beam_n, seg_s, max_utts
        self.t = {
            "w_out": dev(model["w_out"], mat), "b_out": dev(model["b_out"], torch.float32),
            "embed": dev(model["embed"], mat), "w_proj": dev(model["w_proj"], mat),
            "b_proj": dev(model["b_proj"], torch.float32), "pred_init": dev(model["pred_init"], torch.float32),
        }
        w = _Weights()
        for l, (wi, wh, b) in enumerate(model["lstm"]):
            self.t[f"w_ih{l}"], self.t[f"w_hh{l}"] = dev(wi, mat), dev(wh, mat)
            self.t[f"b{l}"] = dev(b, torch.float32)
            w.w_ih[l], w.w_hh[l], w.b_lstm[l] = (self.t[f"w_ih{l}"].data_ptr(), self.t[f"w_hh{l}"].data_ptr(),
                                                   self.t[f"b{l}"].data_ptr())
        for k in ("w_out", "b_out", "embed", "w_proj", "b_proj", "pred_init"):
            setattr(w, k, self.t[k].data_ptr())
        self.stream = stream if stream is not None else torch.cuda.Stream(self.device)
        cfg = _Config(Dj, V, blank_id, beam_n, seg_s, max_utts, max_frames_total, L_, H, E,
                      {"tanh": 0, "relu": 1}[act], 1 if dtype == "bf16" else 0, max_rounds_per_segment,
                      rounds_capacity, max_nodes, int(debug), int(stream_buffer_frames), int(max_result_len), int(joiner_chunk_rows), device,
                      self.stream.cuda_stream)
        torch.cuda.synchronize(self.device)
        self.ctx = C.c_void_p()
        _check(self.L.tbs_init(C.byref(cfg), C.byref(w), C.byref(self.ctx)))
        self.U = 0
        self._enc = None
        self._offsets = None

    def close(self):
        if getattr(self, "ctx", None) is not None and self.ctx.value:
            self.L.tbs_free(self.ctx)
            self.ctx = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- inputs
    def upload_frames(self, enc_proj: np.ndarray):
        """Projected encoder frames [sum T, Dj] -> device tensor in the model's storage type."""
        t = self.torch.from_numpy(np.ascontiguousarray(enc_proj, dtype=np.float32)).to(self.device)
        t = t.to(self.mat_dtype).contiguous()
        self.torch.cuda.synchronize(self.device)
        return t

    def _bind(self, enc_dev, offsets):
        offsets = np.ascontiguousarray(offsets, dtype=np.int32)
        assert enc_dev.dtype == self.mat_dtype and enc_dev.is_contiguous()
        self._enc, self._offsets, self.U = enc_dev, offsets, len(offsets) - 1
        return offsets

    # ---- C ABI, same names
    def begin(self, enc_dev, offsets):
        offsets = self._bind(enc_dev, offsets)
        _check(self.L.tbs_begin(self.ctx, enc_dev.data_ptr(), _hp(offsets), self.U), self.ctx)

    def segment_begin(self, seg_index: int) -> int:
        rows = C.c_int32(0)
        _check(self.L.tbs_segment_begin(self.ctx, seg_index, C.byref(rows)), self.ctx)
        return rows.value

    def joiner_segment(self):
        _check(self.L.tbs_joiner_segment(self.ctx), self.ctx)

    def expand(self):
        _check(self.L.tbs_expand(self.ctx), self.ctx)

    def select_merge(self) -> int:
        live = C.c_int32(0)
        _check(self.L.tbs_select_merge(self.ctx, C.byref(live)), self.ctx)
        return live.value

    def predictor_step(self):
        _check(self.L.tbs_predictor_step(self.ctx), self.ctx)

    def _result_arrays(self, max_len):
        U, N = self.U, self.N
        return (np.full((U, N, max_len), -1, np.int32), np.zeros((U, N), np.int32), np.zeros((U, N), np.float64),
                np.zeros(U, np.int32))

    @staticmethod
    def _nbest(tok, lens, logs, cnt):
        out = []
        for u in range(len(cnt)):
            out.append([(tuple(int(x) for x in tok[u, i, :lens[u, i]]), float(logs[u, i]))
                        for i in range(cnt[u])])
        return out

    def decode(self, enc_dev, offsets, max_len: int = 256):
        """Algorithm 1 on the whole batch; returns per utterance [(tokens, log score)], best first."""
        offsets = self._bind(enc_dev, offsets)
        tok, lens, logs, cnt = self._result_arrays(max_len)
        _check(self.L.tbs_decode(self.ctx, enc_dev.data_ptr(), _hp(offsets), self.U, _hp(tok), _hp(lens),
                                 _hp(logs), _hp(cnt), max_len), self.ctx)
        return self._nbest(tok, lens, logs, cnt)

    def decode_raw(self, enc_dev, offsets, tok, lens, logs, cnt, max_len):
        """tbs_decode into caller-provided host arrays (no Python work in the timed region)."""
        return self.L.tbs_decode(self.ctx, enc_dev.data_ptr(), _hp(offsets), len(offsets) - 1, _hp(tok), _hp(lens),
                                 _hp(logs), _hp(cnt), max_len)

    def stream_begin(self, n_utts: int):
        self.U = int(n_utts)
        _check(self.L.tbs_stream_begin(self.ctx, self.U), self.ctx)

    def push_segment(self, enc_dev, offsets, flush: bool = False):
        """Append offsets[u+1]-offsets[u] new frames to every utterance u and decode what is ready."""
        offsets = np.ascontiguousarray(offsets, dtype=np.int32)
        assert enc_dev is None or (enc_dev.dtype == self.mat_dtype and enc_dev.is_contiguous())
        ptr = enc_dev.data_ptr() if enc_dev is not None and enc_dev.numel() > 0 else None
        _check(self.L.tbs_push_segment(self.ctx, ptr, _hp(offsets), 1 if flush else 0), self.ctx)

    def result(self, max_len: int = 256):
        tok, lens, logs, cnt = self._result_arrays(max_len)
        _check(self.L.tbs_result(self.ctx, _hp(tok), _hp(lens), _hp(logs), _hp(cnt), max_len), self.ctx)
        return self._nbest(tok, lens, logs, cnt)

    def stats(self):
        a, b, c, d = C.c_int64(), C.c_int64(), C.c_int64(), C.c_int64()
        _check(self.L.tbs_stats(self.ctx, C.byref(a), C.byref(b), C.byref(c), C.byref(d)))
        return {"joiner_calls": a.value, "joined_frames": b.value, "frames": c.value, "launches": d.value}

    def path(self):
        v = self.L.tbs_path(self.ctx)
        if v < 0:
            _check(v, self.ctx)
        return {"fixed_places": bool(v & 1), "one_frame_no_logits": bool(v & 2)}

    # ---- inspection
    def counts(self):
        out = np.zeros(4, np.int32)
        _check(self.L.tbs_debug_read(self.ctx, BUF.COUNTS, _hp(out), out.nbytes), self.ctx)
        return {"pairs": int(out[0]), "rows": int(out[1]), "nodes": int(out[2]), "err": int(out[3])}

    def debug_read(self, which: int) -> np.ndarray:
        U, N, S, V, Dj = self.U, self.N, self.S, self.V, self.Dj
        c = self.counts()
        pairs, rows = c["pairs"], c["rows"]
        shapes = {
            BUF.A_COUNT: ((U,), np.int32), BUF.A_LOGS: ((U, N), np.float64), BUF.A_DHAT: ((U, N, S), np.float32),
            BUF.A_PRED: ((U, N, Dj), np.float32), BUF.LOGITS: ((rows, V), np.float32),
            BUF.ROW_STATS: ((rows, 3), np.float32), BUF.DELTA_BLANK: ((pairs,), np.float32),
            BUF.DELTA_NB: ((pairs, V), np.float32), BUF.CAND_SCORE: ((pairs, N), np.float32),
            BUF.CAND_TOKEN: ((pairs, N), np.int32), BUF.PAIR_UTT: ((pairs,), np.int32),
            BUF.PAIR_HYP: ((pairs,), np.int32), BUF.PAIR_ROW0: ((pairs,), np.int32),
            BUF.PAIR_LEN: ((pairs,), np.int32), BUF.COUNTS: ((4,), np.int32),
        }
        shape, dt = shapes[which]
        out = np.zeros(shape, dt)
        if out.size:
            _check(self.L.tbs_debug_read(self.ctx, which, _hp(out), out.nbytes), self.ctx)
        return out

    def debug_write(self, which: int, arr: np.ndarray):
        dt = {BUF.A_COUNT: np.int32, BUF.A_LOGS: np.float64, BUF.A_DHAT: np.float32, BUF.A_PRED: np.float32}[which]
        a = np.ascontiguousarray(arr, dtype=dt)
        _check(self.L.tbs_debug_write(self.ctx, which, _hp(a), a.nbytes), self.ctx)

    def debug_rebuild(self, seg_index: int) -> int:
        rows = C.c_int32(0)
        _check(self.L.tbs_debug_rebuild(self.ctx, seg_index, C.byref(rows)), self.ctx)
        return rows.value

    def debug_hyps(self, group: int, cap: int = 0, max_len: int = 256):
        """group 0 = A, 1 = B; per utterance [(tokens, log score)] in stored order."""
        tok, lens, logs, cnt = self.debug_hyps_raw(group, cap, max_len)
        return self._nbest(tok, lens, logs, cnt)

    def debug_hyps_raw(self, group: int, cap: int = 0, max_len: int = 256, noalloc: bool = False, fill: int = -1):
        """The four output arrays of tbs_debug_hyps (or of tbs_debug_hyps_noalloc), pre-filled with `fill`."""
        cap = cap or (self.N if group == 0 else self.N * 64)
        U = self.U
        tok = np.full((U, cap, max_len), fill, np.int32)
        lens = np.full((U, cap), fill, np.int32)
        logs = np.full((U, cap), float(fill), np.float64)
        cnt = np.full(U, fill, np.int32)
        fn = self.L.tbs_debug_hyps_noalloc if noalloc else self.L.tbs_debug_hyps
        _check(fn(self.ctx, group, _hp(tok), _hp(lens), _hp(logs), _hp(cnt), cap, max_len), self.ctx)
        return tok, lens, logs, cnt

    # ---- timing
    def profile_select(self, kernel_id: int):
        _check(self.L.tbs_profile_select(self.ctx, kernel_id), self.ctx)

    def profile_overhead(self, n: int = 200) -> float:
        """Microseconds an event pair reads around a kernel that does nothing."""
        us = C.c_double(0.0)
        _check(self.L.tbs_profile_overhead(self.ctx, n, C.byref(us)), self.ctx)
        return us.value

    def profile_read(self):
        n, ms, units = C.c_int64(), C.c_double(), C.c_int64()
        _check(self.L.tbs_profile_read(self.ctx, C.byref(n), C.byref(ms), C.byref(units)), self.ctx)
        return {"launches": n.value, "total_ms": ms.value, "units": units.value}


def gemm_bf16(a, b, bias=None, kernel=0):
    """C = a @ b.T (+ bias) through the library's MFMA GEMM; a [M,K], b [N,K] bf16 torch tensors."""
    import torch
    L = load_library()
    M, K = a.shape
    N = b.shape[0]
    out = torch.empty((M, N), dtype=torch.float32, device=a.device)
    st = torch.cuda.current_stream(a.device).cuda_stream
    _check(L.tbs_gemm_bf16(a.data_ptr(), b.data_ptr(), bias.data_ptr() if bias is not None else None,
                           out.data_ptr(), M, N, K, kernel, st))
    return out
