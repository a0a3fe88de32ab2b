"""ctypes binding of include/rnnt_greedy.h.  Argument marshalling only.

Tensors are anything with .data_ptr() (torch tensors on the GPU, fp32 / int32,
contiguous); torch is used for device memory and streams, nothing else.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

HERE = os.path.dirname(os.path.abspath(__file__))

RNNT_OK = 0
RNNT_DEV_LEN_CLAMPED, RNNT_DEV_OVERFLOW, RNNT_DEV_ABORTED = 1, 2, 4

EXPORTS = (
    "rnnt_engine_create", "rnnt_engine_destroy", "rnnt_greedy_decode",
    "rnnt_label_looping_decode", "tdt_label_looping_decode", "rnnt_encoder_projection",
    "rnnt_engine_status", "rnnt_engine_stats", "rnnt_engine_configure", "rnnt_status_string",
    "rnnt_engine_set_logp_output",
    "rnnt_engine_set_done_flags", "rnnt_engine_set_wait_limit",
    "rnnt_label_looping_decode_noalloc",
    "rnnt_engine_phase_timers",
    "rnnt_probe_stream", "rnnt_probe_exchange", "rnnt_probe_mfma", "rnnt_probe_e4m3_widening",
    "rnnt_quantize_rows_e4m3", "rnnt_quantize_blocks_e2m1", "rnnt_probe_e2m1_widening",
)


RNNT_FLAG_BF16_WEIGHTS = 1
RNNT_FLAG_FP8_WEIGHTS = 2
RNNT_FLAG_PLAIN_LAUNCH = 4
RNNT_FLAG_BF16_ARITHMETIC = 8
RNNT_FLAG_MULTI_BLANK = 16
RNNT_FLAG_FP4_WEIGHTS = 32
RNNT_FP4_BLOCK = 128


class RnntError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"rnnt_greedy error {code}: {text}")
        self.code = code


class _ModelDesc(C.Structure):
    _fields_ = [
        ("F", C.c_int32), ("E", C.c_int32), ("H", C.c_int32), ("L", C.c_int32),
        ("J", C.c_int32), ("V1", C.c_int32), ("blank", C.c_int32), ("D", C.c_int32),
        ("durations", C.POINTER(C.c_int32)),
        ("emb", C.c_void_p),
        ("w_ih", C.POINTER(C.c_void_p)), ("w_hh", C.POINTER(C.c_void_p)),
        ("b_ih", C.POINTER(C.c_void_p)), ("b_hh", C.POINTER(C.c_void_p)),
        ("w_enc", C.c_void_p), ("b_enc", C.c_void_p),
        ("w_pred", C.c_void_p), ("b_pred", C.c_void_p),
        ("w_out", C.c_void_p), ("b_out", C.c_void_p),
    ]


class RnntStats(C.Structure):
    _fields_ = [
        ("pred_steps", C.c_int64), ("joint_steps", C.c_int64),
        ("max_pred_steps", C.c_int64), ("max_joint_steps", C.c_int64),
        ("joint_samples", C.c_int64), ("barrier_polls", C.c_int64),
        ("n_teams", C.c_int32), ("team_size", C.c_int32),
        ("lookahead", C.c_int32), ("xcd_mismatch", C.c_int32),
        ("joint_groups", C.c_int32), ("search_steps", C.c_int32),
        ("projection_ms", C.c_float), ("decode_ms", C.c_float),
    ]

    def as_dict(self) -> dict:
        return {name: (float(getattr(self, name)) if name.endswith("_ms")
                       else int(getattr(self, name))) for name, _ in self._fields_}


def lib_path() -> str:
    return os.path.join(HERE, "librnnt_greedy.so")


_LIB = None


def load_library():
    """Load librnnt_greedy.so; raise if it has not been built."""
    global _LIB
    if _LIB is None:
        path = lib_path()
        if not os.path.exists(path):
            raise ImportError(
                f"{path} is missing: build it with `python -m paper_2406_03791_amd.build` "
                "(there is no fallback path)")
        # PyTorch ships its own HIP runtime; it has to be in the process before this library
        # pulls in the system one, or the two runtimes disagree about the device.
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        lib = C.CDLL(path)
        dec_args = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32,
                    C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]
        lib.rnnt_engine_create.argtypes = [C.POINTER(_ModelDesc), C.c_int32, C.c_int32, C.c_int32,
                                           C.POINTER(C.c_void_p)]
        lib.rnnt_engine_destroy.argtypes = [C.c_void_p]
        lib.rnnt_greedy_decode.argtypes = dec_args + [C.c_void_p]
        lib.rnnt_label_looping_decode.argtypes = dec_args + [C.c_void_p]
        lib.rnnt_label_looping_decode_noalloc.argtypes = dec_args + [C.c_void_p]
        lib.tdt_label_looping_decode.argtypes = dec_args + [C.c_void_p, C.c_void_p]
        lib.rnnt_encoder_projection.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
                                                C.c_int32, C.c_void_p, C.c_void_p]
        lib.rnnt_engine_status.argtypes = [C.c_void_p, C.POINTER(C.c_int32)]
        lib.rnnt_engine_stats.argtypes = [C.c_void_p, C.POINTER(RnntStats)]
        lib.rnnt_engine_configure.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32]
        lib.rnnt_engine_set_logp_output.argtypes = [C.c_void_p, C.c_void_p]
        lib.rnnt_engine_set_done_flags.argtypes = [C.c_void_p, C.c_void_p]
        lib.rnnt_engine_set_wait_limit.argtypes = [C.c_void_p, C.c_int64]
        lib.rnnt_engine_phase_timers.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_double), C.c_int32]
        lib.rnnt_probe_stream.argtypes = [C.c_int32, C.POINTER(C.c_double), C.POINTER(C.c_double)]
        lib.rnnt_probe_exchange.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_double)]
        lib.rnnt_probe_mfma.argtypes = [C.c_int32, C.POINTER(C.c_double)]
        lib.rnnt_probe_e4m3_widening.argtypes = [C.c_float, C.POINTER(C.c_uint16)]
        for name in ("rnnt_quantize_rows_e4m3", "rnnt_quantize_blocks_e2m1"):
            getattr(lib, name).argtypes = [C.POINTER(C.c_float), C.c_int64, C.c_int64,
                                           C.POINTER(C.c_float), C.POINTER(C.c_float)]
        lib.rnnt_probe_e2m1_widening.argtypes = [C.c_float, C.POINTER(C.c_uint16)]
        lib.rnnt_status_string.argtypes = [C.c_int]
        lib.rnnt_status_string.restype = C.c_char_p
        for name in EXPORTS:
            if name != "rnnt_status_string":
                getattr(lib, name).restype = C.c_int
        _LIB = lib
    return _LIB


def rnnt_status_string(code: int) -> str:
    return load_library().rnnt_status_string(int(code)).decode()


def _check(code: int) -> None:
    if code != RNNT_OK:
        raise RnntError(code, rnnt_status_string(code))


def _p(t) -> Optional[int]:
    return None if t is None else C.c_void_p(t.data_ptr())


def rnnt_engine_create(dims, weights: dict, max_B: int, max_T: int, flags: int = 0):
    """dims: object with F, E, H, L, J, V1, blank, durations; weights: name ->
    device tensor (emb, w_ih0.., w_hh0.., b_ih0.., b_hh0.., w_enc, b_enc, w_pred,
    b_pred, w_out, b_out).  Returns the engine handle."""
    L = int(dims.L)
    dur = list(dims.durations)
    # a multi-blank model's extra output columns are its big blanks: their spans travel in the
    # descriptor's durations and the flag says what they are
    spans = list(getattr(dims, "big_blanks", ()))
    if spans:
        assert not dur, "a model has durations or big blanks, not both"
        dur, flags = spans, flags | RNNT_FLAG_MULTI_BLANK
    d = _ModelDesc()
    d.F, d.E, d.H, d.L, d.J, d.V1 = int(dims.F), int(dims.E), int(dims.H), L, int(dims.J), int(dims.V1)
    d.blank, d.D = int(dims.blank), len(dur)
    dur_arr = (C.c_int32 * max(1, len(dur)))(*dur)
    d.durations = C.cast(dur_arr, C.POINTER(C.c_int32))
    arrs = {}
    for key in ("w_ih", "w_hh", "b_ih", "b_hh"):
        arrs[key] = (C.c_void_p * L)(*[weights[f"{key}{l}"].data_ptr() for l in range(L)])
        setattr(d, key, C.cast(arrs[key], C.POINTER(C.c_void_p)))
    for key in ("emb", "w_enc", "b_enc", "w_pred", "b_pred", "w_out", "b_out"):
        setattr(d, key, weights[key].data_ptr())
    out = C.c_void_p()
    _check(load_library().rnnt_engine_create(C.byref(d), int(max_B), int(max_T), int(flags),
                                             C.byref(out)))
    return out


def rnnt_engine_destroy(eng) -> None:
    _check(load_library().rnnt_engine_destroy(eng))


def rnnt_engine_set_logp_output(eng, logp_out) -> None:
    _check(load_library().rnnt_engine_set_logp_output(eng, _p(logp_out)))


def rnnt_engine_set_done_flags(eng, done) -> None:
    _check(load_library().rnnt_engine_set_done_flags(eng, _p(done)))


def rnnt_engine_set_wait_limit(eng, polls: int = -1) -> None:
    _check(load_library().rnnt_engine_set_wait_limit(eng, int(polls)))


def rnnt_engine_configure(eng, n_teams: int = 0, joint_groups: int = 0, lookahead: int = 0,
                          search_steps: int = 0) -> None:
    _check(load_library().rnnt_engine_configure(eng, int(n_teams), int(joint_groups),
                                                int(lookahead), int(search_steps)))


def _decode(fn, eng, enc_out, enc_len, B, T, max_symbols, tokens_out, tok_len_out, cap,
            frames_out, logit_out, extra, stream):
    args = [eng, _p(enc_out), _p(enc_len), int(B), int(T), int(max_symbols), _p(tokens_out),
            _p(tok_len_out), int(cap), _p(frames_out), _p(logit_out)]
    args += extra
    args.append(C.c_void_p(stream) if stream else None)
    _check(fn(*args))


def rnnt_greedy_decode(eng, enc_out, enc_len, B, T, max_symbols, tokens_out, tok_len_out, cap,
                       frames_out=None, logit_out=None, stream: int = 0) -> None:
    _decode(load_library().rnnt_greedy_decode, eng, enc_out, enc_len, B, T, max_symbols,
            tokens_out, tok_len_out, cap, frames_out, logit_out, [], stream)


def rnnt_label_looping_decode(eng, enc_out, enc_len, B, T, max_symbols, tokens_out, tok_len_out,
                              cap, frames_out=None, logit_out=None, stream: int = 0) -> None:
    _decode(load_library().rnnt_label_looping_decode, eng, enc_out, enc_len, B, T, max_symbols,
            tokens_out, tok_len_out, cap, frames_out, logit_out, [], stream)


def rnnt_label_looping_decode_noalloc(eng, enc_out, enc_len, B, T, max_symbols, tokens_out,
                                      tok_len_out, cap, frames_out=None, logit_out=None,
                                      stream: int = 0) -> None:
    _decode(load_library().rnnt_label_looping_decode_noalloc, eng, enc_out, enc_len, B, T,
            max_symbols, tokens_out, tok_len_out, cap, frames_out, logit_out, [], stream)


def tdt_label_looping_decode(eng, enc_out, enc_len, B, T, max_symbols, tokens_out, tok_len_out,
                             cap, frames_out=None, logit_out=None, durations_out=None,
                             stream: int = 0) -> None:
    _decode(load_library().tdt_label_looping_decode, eng, enc_out, enc_len, B, T, max_symbols,
            tokens_out, tok_len_out, cap, frames_out, logit_out, [_p(durations_out)], stream)


def rnnt_encoder_projection(eng, enc_out, enc_len, B, T, proj_out, stream: int = 0) -> None:
    _check(load_library().rnnt_encoder_projection(eng, _p(enc_out), _p(enc_len), int(B), int(T),
                                                  _p(proj_out),
                                                  C.c_void_p(stream) if stream else None))


def rnnt_engine_status(eng) -> int:
    out = C.c_int32(0)
    _check(load_library().rnnt_engine_status(eng, C.byref(out)))
    return int(out.value)


def rnnt_engine_phase_timers(eng, team: int, n: int = 24):
    """Microseconds per phase for rank 0 of `team` (profile builds only)."""
    out = (C.c_double * n)()
    _check(load_library().rnnt_engine_phase_timers(eng, int(team), out, int(n)))
    return [float(v) for v in out]


def rnnt_probe_stream(from_l2: bool):
    """(GB/s over the device, GB/s per compute unit)"""
    a, b = C.c_double(0), C.c_double(0)
    _check(load_library().rnnt_probe_stream(int(bool(from_l2)), C.byref(a), C.byref(b)))
    return float(a.value), float(b.value)


def rnnt_probe_exchange(team_size: int, length: int, tagged: bool) -> float:
    out = C.c_double(0)
    _check(load_library().rnnt_probe_exchange(int(team_size), int(length), int(bool(tagged)), C.byref(out)))
    return float(out.value)


def rnnt_probe_e4m3_widening(scale: float = 1.0):
    """[4][256] uint16 array: the bf16 code each e4m3 code becomes under the scale operand,
    per byte position."""
    import numpy as np
    out = np.zeros((4, 256), dtype=np.uint16)
    _check(load_library().rnnt_probe_e4m3_widening(C.c_float(scale), out.ctypes.data_as(C.POINTER(C.c_uint16))))
    return out


def rnnt_quantize_rows_e4m3(w):
    """(quantised copy, row scales) of a 2-D float32 numpy array: every row as e4m3 values
    times a power of two (host-side helper of the library, no device work)."""
    import numpy as np
    w = np.ascontiguousarray(w, dtype=np.float32)
    assert w.ndim == 2
    out = np.empty_like(w)
    scales = np.empty(w.shape[0], dtype=np.float32)
    fp = C.POINTER(C.c_float)
    _check(load_library().rnnt_quantize_rows_e4m3(w.ctypes.data_as(fp), w.shape[0], w.shape[1],
                                                  out.ctypes.data_as(fp), scales.ctypes.data_as(fp)))
    return out, scales


def rnnt_quantize_blocks_e2m1(w):
    """(quantised copy, block scales [rows, ceil(cols / 128)]) of a 2-D float32 numpy array:
    every block of 128 consecutive weights of a row as e2m1 values times a power of two."""
    import numpy as np
    w = np.ascontiguousarray(w, dtype=np.float32)
    assert w.ndim == 2
    out = np.empty_like(w)
    scales = np.empty((w.shape[0], (w.shape[1] + RNNT_FP4_BLOCK - 1) // RNNT_FP4_BLOCK), dtype=np.float32)
    fp = C.POINTER(C.c_float)
    _check(load_library().rnnt_quantize_blocks_e2m1(w.ctypes.data_as(fp), w.shape[0], w.shape[1],
                                                    out.ctypes.data_as(fp), scales.ctypes.data_as(fp)))
    return out, scales


def rnnt_probe_e2m1_widening(scale: float = 1.0):
    """[4][256][2] uint16 array: the two bf16 codes a byte of two e2m1 codes becomes under the
    scale operand, per byte position (low nibble first)."""
    import numpy as np
    out = np.zeros((4, 256, 2), dtype=np.uint16)
    _check(load_library().rnnt_probe_e2m1_widening(C.c_float(scale), out.ctypes.data_as(C.POINTER(C.c_uint16))))
    return out


def rnnt_probe_mfma(shape: int) -> float:
    out = C.c_double(0)
    _check(load_library().rnnt_probe_mfma(int(shape), C.byref(out)))
    return float(out.value)


def rnnt_engine_stats(eng) -> RnntStats:
    out = RnntStats()
    _check(load_library().rnnt_engine_stats(eng, C.byref(out)))
    return out


class Engine:
    """Convenience owner of an engine handle plus output allocation with torch.
    Holds no decode logic: each method forwards to the C entry point of the
    same name."""

    def __init__(self, model, max_B: int, max_T: int, device: str = "cuda:0", flags: int = 0):
        import torch
        self.torch = torch
        self.device = torch.device(device)
        self.dims = model.dims
        self.weights = {k: torch.from_numpy(v).to(self.device).contiguous()
                        for k, v in model.arrays().items()}
        torch.cuda.synchronize(self.device)
        self.handle = rnnt_engine_create(self.dims, self.weights, max_B, max_T, flags)

    def close(self) -> None:
        if getattr(self, "handle", None):
            rnnt_engine_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def configure(self, n_teams: int = 0, joint_groups: int = 0, lookahead: int = 0,
                  search_steps: int = 0) -> None:
        rnnt_engine_configure(self.handle, n_teams, joint_groups, lookahead, search_steps)

    def set_wait_limit(self, polls: int = -1) -> None:
        """Polls a device-side wait may repeat before the call gives up (-1 = default)."""
        rnnt_engine_set_wait_limit(self.handle, polls)

    def alloc_outputs(self, B: int, cap: int, pinned: bool = False):
        """Output tensors on the device, or (pinned=True) in pinned host memory,
        which a host thread can read while a decode call runs."""
        t = self.torch
        kw = dict(pin_memory=True) if pinned else dict(device=self.device)
        out = dict(tokens=t.empty((B, cap), dtype=t.int32, **kw),
                   tok_len=t.empty((B,), dtype=t.int32, **kw),
                   frames=t.empty((B, cap), dtype=t.int32, **kw),
                   logits=t.empty((B, cap), dtype=t.float32, **kw))
        if self.dims.D:
            out["durs"] = t.empty((B, cap), dtype=t.int32, **kw)
        return out

    def decode(self, variant: str, enc_out, enc_len, max_symbols: int, out=None,
               cap: Optional[int] = None, logp: bool = False, done=None):
        """enc_out [B,T,F] fp32 and enc_len [B] int32 device tensors.  Queues the
        decode on the current stream and returns the output tensors (device).
        logp=True also asks for the log-probabilities (out["logps"]); done is an
        int32 [B] tensor of completion flags the caller has zeroed."""
        B, T = int(enc_out.shape[0]), int(enc_out.shape[1])
        if cap is None:
            cap = T * max_symbols
        if out is None:
            out = self.alloc_outputs(B, cap)
        if logp and "logps" not in out:
            out["logps"] = self.torch.empty((B, cap), dtype=self.torch.float32, device=self.device)
        rnnt_engine_set_logp_output(self.handle, out["logps"] if logp else None)
        rnnt_engine_set_done_flags(self.handle, done)
        stream = self.torch.cuda.current_stream(self.device).cuda_stream
        common = (self.handle, enc_out, enc_len, B, T, max_symbols, out["tokens"], out["tok_len"],
                  cap, out["frames"], out["logits"])
        if variant == "frame":
            rnnt_greedy_decode(*common, stream=stream)
        elif variant == "label":
            rnnt_label_looping_decode(*common, stream=stream)
        elif variant == "label_noalloc":
            rnnt_label_looping_decode_noalloc(*common, stream=stream)
        elif variant == "tdt":
            tdt_label_looping_decode(*common, durations_out=out.get("durs"), stream=stream)
        else:
            raise ValueError(variant)
        return out

    def encoder_projection(self, enc_out, enc_len):
        B, T = int(enc_out.shape[0]), int(enc_out.shape[1])
        proj = self.torch.zeros((B, T, self.dims.J), dtype=self.torch.float32, device=self.device)
        stream = self.torch.cuda.current_stream(self.device).cuda_stream
        rnnt_encoder_projection(self.handle, enc_out, enc_len, B, T, proj, stream)
        return proj

    def status(self) -> int:
        return rnnt_engine_status(self.handle)

    def stats(self) -> dict:
        return rnnt_engine_stats(self.handle).as_dict()

    def phase_timers(self, team: int, n: int = 24):
        return rnnt_engine_phase_timers(self.handle, team, n)
