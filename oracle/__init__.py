"""ctypes front end of the CPU oracle (oracle/rnnt_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the
benchmark's cpu_baseline leg.  The HIP path never imports this package and this
package never imports the HIP path.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import numpy as np

from . import build as _build

_LIBS = {}


def _lib(real: str):
    if real not in _LIBS:
        path = _build.lib_path(real)
        if not os.path.exists(path) or os.path.getmtime(path) < os.path.getmtime(_build.SRC):
            _build.build()
        lib = C.CDLL(path)
        lib.orc_lstm_net_create.restype = C.c_void_p
        lib.orc_table_net_create.restype = C.c_void_p
        lib.orc_net_destroy.argtypes = [C.c_void_p]
        lib.orc_real_size.restype = C.c_int
        for name in ("orc_decode_frame_looping", "orc_decode_label_looping",
                     "orc_decode_sequential"):
            getattr(lib, name).argtypes = [C.c_void_p, C.c_void_p]
            getattr(lib, name).restype = C.c_int
        lib.orc_follow_sequential.restype = C.c_int
        lib.orc_net_as_multi_blank.argtypes = [C.c_void_p]
        lib.orc_net_as_multi_blank.restype = None
        lib.orc_lstm_net_emulate_bf16.argtypes = [C.c_void_p]
        lib.orc_lstm_net_emulate_bf16.restype = None
        lib.orc_round_bf16.argtypes = [C.c_float if real == "float" else C.c_double]
        lib.orc_round_bf16.restype = C.c_float if real == "float" else C.c_double
        lib.orc_quantize_rows_e4m3.argtypes = [C.c_void_p, C.c_long, C.c_long, C.c_void_p, C.c_void_p]
        lib.orc_quantize_rows_e4m3.restype = None
        lib.orc_quantize_blocks_e2m1.argtypes = [C.c_void_p, C.c_long, C.c_long, C.c_long, C.c_void_p, C.c_void_p]
        lib.orc_quantize_blocks_e2m1.restype = None
        _LIBS[real] = lib
    return _LIBS[real]


def _np_real(real: str):
    return np.float32 if real == "float" else np.float64


class _DecodeIO(C.Structure):
    _fields_ = [
        ("B", C.c_int32), ("T", C.c_int32), ("S", C.c_int32), ("cap", C.c_int32),
        ("rec_cap", C.c_int32), ("skip_masked", C.c_int32),
        ("n_threads", C.c_int32), ("status", C.c_int32),
        ("x", C.c_void_p), ("len", C.c_void_p),
        ("tokens", C.c_void_p), ("frames", C.c_void_p), ("scores", C.c_void_p),
        ("durs", C.c_void_p), ("tok_len", C.c_void_p),
        ("rec_t", C.c_void_p), ("rec_u", C.c_void_p), ("rec_k", C.c_void_p),
        ("rec_d", C.c_void_p), ("rec_top", C.c_void_p), ("rec_margin", C.c_void_p),
        ("rec_dmargin", C.c_void_p), ("rec_len", C.c_void_p),
        ("stat_outer", C.c_int64), ("stat_inner", C.c_int64),
        ("stat_pred", C.c_int64), ("stat_pred_rows", C.c_int64),
        ("stat_joint_rows", C.c_int64),
        ("logps", C.c_void_p),
    ]


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


class Net:
    """Base: owns the C net handle and the arrays it points into."""

    def __init__(self, real: str):
        self.real = real
        self.lib = _lib(real)
        self.dtype = _np_real(real)
        self.handle = None
        self._keep = []

    def __del__(self):
        if getattr(self, "handle", None):
            self.lib.orc_net_destroy(self.handle)
            self.handle = None

    # sub-network access for the numerics tests ------------------------------
    def prep(self, x_row: np.ndarray) -> np.ndarray:
        x = np.ascontiguousarray(x_row, dtype=self.dtype)
        out = np.empty(self.p_size, dtype=self.dtype)
        self.lib.orc_net_prep(C.c_void_p(self.handle), _ptr(x), _ptr(out))
        return out

    def pred(self, last: int, state: np.ndarray):
        s_in = np.ascontiguousarray(state, dtype=self.dtype)
        s_out = np.empty(self.state_size, dtype=self.dtype)
        g = np.empty(self.g_size, dtype=self.dtype)
        self.lib.orc_net_pred(C.c_void_p(self.handle), C.c_int(int(last)), _ptr(s_in),
                              _ptr(s_out), _ptr(g))
        return g, s_out

    def joint(self, p_row: np.ndarray, g: np.ndarray) -> np.ndarray:
        p = np.ascontiguousarray(p_row, dtype=self.dtype)
        gg = np.ascontiguousarray(g, dtype=self.dtype)
        out = np.empty(self.n_out, dtype=self.dtype)
        self.lib.orc_net_joint(C.c_void_p(self.handle), _ptr(p), _ptr(gg), _ptr(out))
        return out


class LstmNet(Net):
    """Embedding + stacked LSTM prediction network and the additive joint."""

    def __init__(self, model, real: str = "float", bf16: bool = False):
        """bf16=True: bfloat16 emulation (weights and every input of a dense product rounded
        to bfloat16, float accumulation), the reference of the engine's bfloat16 mode."""
        super().__init__(real)
        d = model.dims
        dt = self.dtype
        cv = lambda a: np.ascontiguousarray(a, dtype=dt)
        emb, w_enc, b_enc = cv(model.emb), cv(model.w_enc), cv(model.b_enc)
        w_pred, b_pred = cv(model.w_pred), cv(model.b_pred)
        w_out, b_out = cv(model.w_out), cv(model.b_out)
        w_ih = [cv(a) for a in model.w_ih]
        w_hh = [cv(a) for a in model.w_hh]
        b_ih = [cv(a) for a in model.b_ih]
        b_hh = [cv(a) for a in model.b_hh]
        # a multi-blank model's extra output columns are its big blanks; the net is created
        # with them in the place of durations and then told what they are
        spans = tuple(getattr(d, "big_blanks", ()))
        assert not (spans and d.D), "a model has durations or big blanks, not both"
        dur = np.ascontiguousarray(spans if spans else model.durations, dtype=np.int32)
        n_extra = len(spans) if spans else d.D
        self._keep = [emb, w_enc, b_enc, w_pred, b_pred, w_out, b_out, w_ih, w_hh,
                      b_ih, b_hh, dur]
        PA = C.c_void_p * d.L
        arr = lambda lst: PA(*[a.ctypes.data for a in lst])
        self.handle = self.lib.orc_lstm_net_create(
            C.c_int(d.F), C.c_int(d.E), C.c_int(d.H), C.c_int(d.L), C.c_int(d.J),
            C.c_int(d.V1), C.c_int(n_extra), C.c_int(d.blank), _ptr(dur), _ptr(emb),
            arr(w_ih), arr(w_hh), arr(b_ih), arr(b_hh), _ptr(w_enc), _ptr(b_enc),
            _ptr(w_pred), _ptr(b_pred), _ptr(w_out), _ptr(b_out))
        self.x_size, self.p_size = d.F, d.J
        self.state_size, self.g_size = 2 * d.L * d.H, d.H
        self.V1, self.D, self.blank, self.n_out = d.V1, d.D, d.blank, d.n_out
        self.durations = dur
        self.big_blanks = spans
        if spans:
            self.D = 0
            self.lib.orc_net_as_multi_blank(C.c_void_p(self.handle))
        self.bf16 = bool(bf16)
        if bf16:
            self.lib.orc_lstm_net_emulate_bf16(C.c_void_p(self.handle))


class TableNet(Net):
    """Logits read from a table indexed by (utterance, frame, labels emitted so
    far, last label).  table has shape [B, T, U, V1, V1 + D]; a table that does
    not depend on the last label may be given as [B, T, U, V1 + D]."""

    def __init__(self, table: np.ndarray, V1: int, durations: Sequence[int] = (),
                 real: str = "float", big_blanks: Sequence[int] = ()):
        """big_blanks: spans of a multi-blank model's big-blank symbols, which then take the
        place of the duration columns (last axis V1 + len(big_blanks))."""
        super().__init__(real)
        assert not (len(durations) and len(big_blanks))
        if len(big_blanks):
            durations = big_blanks
        D = len(durations)
        t = np.asarray(table, dtype=self.dtype)
        if t.ndim == 4:
            t = np.repeat(t[:, :, :, None, :], V1, axis=3)
        assert t.ndim == 5 and t.shape[3] == V1 and t.shape[4] == V1 + D
        t = np.ascontiguousarray(t)
        dur = np.ascontiguousarray(durations, dtype=np.int32)
        self._keep = [t, dur]
        self.B, self.T, self.U = t.shape[0], t.shape[1], t.shape[2]
        self.handle = self.lib.orc_table_net_create(
            C.c_int(V1), C.c_int(D), C.c_int(V1 - 1), _ptr(dur), C.c_int(self.U), _ptr(t))
        self.x_size, self.p_size, self.state_size, self.g_size = 1, 1, 1, 2
        self.V1, self.D, self.blank, self.n_out = V1, D, V1 - 1, V1 + D
        self.durations = dur
        self.big_blanks = tuple(big_blanks)
        if len(big_blanks):
            self.D = 0
            self.lib.orc_net_as_multi_blank(C.c_void_p(self.handle))

    def frames(self) -> np.ndarray:
        """The encoder 'output' that carries each cell's index."""
        return np.arange(self.B * self.T, dtype=self.dtype).reshape(self.B, self.T, 1)


@dataclass
class Records:
    t: List[np.ndarray]
    u: List[np.ndarray]
    k: List[np.ndarray]
    d: List[np.ndarray]
    top: List[np.ndarray]
    margin: List[np.ndarray]
    dmargin: List[np.ndarray]


@dataclass
class Decoded:
    tokens: List[np.ndarray]
    frames: List[np.ndarray]
    scores: List[np.ndarray]       # maximum token logit of each emission
    logps: List[np.ndarray]        # its log-softmax value over the token columns
    durs: List[np.ndarray]
    tok_len: np.ndarray
    status: int
    stats: dict
    records: Optional[Records] = None
    raw_tokens: Optional[np.ndarray] = None   # [B, cap] with -1 fill


_SCHEDULES = {"frame": "orc_decode_frame_looping", "label": "orc_decode_label_looping",
              "tdt": "orc_decode_label_looping", "seq": "orc_decode_sequential"}


def decode(net: Net, enc_out: np.ndarray, enc_len: np.ndarray, max_symbols: int,
           schedule: str = "seq", *, cap: Optional[int] = None, record: bool = False,
           n_threads: int = 1, skip_masked: bool = False) -> Decoded:
    """schedule 'frame' is Algorithm 1 as written: both networks run for every row at every
    inner step.  skip_masked=True passes over rows that are already masked (same outputs,
    pinned by tests; only for timing large batches)."""
    x = np.ascontiguousarray(enc_out, dtype=net.dtype)
    B, T = int(x.shape[0]), int(x.shape[1])
    assert x.shape[2] == net.x_size
    ln = np.ascontiguousarray(enc_len, dtype=np.int32)
    assert ln.shape == (B,)
    S = int(max_symbols)
    if cap is None:
        cap = max(1, T * S)
    rec_cap = T * (S + 1) + 1 if record else 0
    i32 = lambda *s: np.zeros(s, dtype=np.int32)
    rl = lambda *s: np.zeros(s, dtype=net.dtype)
    tokens, frames, scores, durs = i32(B, cap), i32(B, cap), rl(B, cap), i32(B, cap)
    logps = rl(B, cap)
    tok_len = i32(B)
    io = _DecodeIO()
    io.B, io.T, io.S, io.cap, io.rec_cap = B, T, S, cap, rec_cap
    io.skip_masked, io.n_threads = int(skip_masked), int(n_threads)
    io.x, io.len = _ptr(x), _ptr(ln)
    io.tokens, io.frames, io.scores = _ptr(tokens), _ptr(frames), _ptr(scores)
    io.durs, io.tok_len = _ptr(durs), _ptr(tok_len)
    io.logps = _ptr(logps)
    recs = None
    if record:
        recs = dict(t=i32(B, rec_cap), u=i32(B, rec_cap), k=i32(B, rec_cap),
                    d=i32(B, rec_cap), top=rl(B, rec_cap), margin=rl(B, rec_cap),
                    dmargin=rl(B, rec_cap), len=i32(B))
        io.rec_t, io.rec_u, io.rec_k = _ptr(recs["t"]), _ptr(recs["u"]), _ptr(recs["k"])
        io.rec_d, io.rec_top = _ptr(recs["d"]), _ptr(recs["top"])
        io.rec_margin, io.rec_dmargin = _ptr(recs["margin"]), _ptr(recs["dmargin"])
        io.rec_len = _ptr(recs["len"])
    fn = getattr(net.lib, _SCHEDULES[schedule])
    rc = fn(C.c_void_p(net.handle), C.byref(io))
    if rc != 0:
        raise ValueError(f"oracle schedule '{schedule}' refused this net (rc={rc})")
    n = np.minimum(tok_len, cap)
    out = Decoded(
        tokens=[tokens[b, :n[b]].copy() for b in range(B)],
        frames=[frames[b, :n[b]].copy() for b in range(B)],
        scores=[scores[b, :n[b]].copy() for b in range(B)],
        logps=[logps[b, :n[b]].copy() for b in range(B)],
        durs=[durs[b, :n[b]].copy() for b in range(B)],
        tok_len=tok_len.copy(), status=int(io.status),
        stats=dict(outer=int(io.stat_outer), inner=int(io.stat_inner),
                   pred=int(io.stat_pred), pred_rows=int(io.stat_pred_rows),
                   joint_rows=int(io.stat_joint_rows)),
        raw_tokens=tokens)
    if record:
        m = np.minimum(recs["len"], rec_cap)
        cut = lambda key: [recs[key][b, :m[b]].copy() for b in range(B)]
        out.records = Records(cut("t"), cut("u"), cut("k"), cut("d"), cut("top"),
                              cut("margin"), cut("dmargin"))
    return out


@dataclass
class Followed:
    departures: int            # -1: the hypothesis cannot be produced by any walk
    worst_gap: float
    where: List[dict] = field(default_factory=list)


def follow(net: Net, enc_out_b: np.ndarray, length: int, max_symbols: int,
           tokens: Sequence[int], frames: Sequence[int],
           durs: Optional[Sequence[int]] = None, max_report: int = 64, tol: float = 0.0) -> Followed:
    """Walk utterance b along a hypothesis; see follow_sequential in the C file.  tol > 0 (TDT):
    the durations taken on blanks, which a hypothesis does not record, may be any whose logit
    lies less than tol below the maximum, as long as the walk reaches the next label's frame."""
    x = np.ascontiguousarray(enc_out_b, dtype=net.dtype)
    T = int(x.shape[0])
    tk = np.ascontiguousarray(tokens, dtype=np.int32)
    fr = np.ascontiguousarray(frames, dtype=np.int32)
    du = np.ascontiguousarray(durs if durs is not None else np.zeros(len(tk)), dtype=np.int32)
    rep = [np.zeros(max_report, dtype=np.int32) for _ in range(4)]
    gap = np.zeros(max_report, dtype=net.dtype)
    worst = np.zeros(1, dtype=net.dtype)
    n = net.lib.orc_follow_sequential(
        C.c_void_p(net.handle), _ptr(x), C.c_int(T), C.c_int(int(length)),
        C.c_int(int(max_symbols)), _ptr(tk), _ptr(fr), _ptr(du), C.c_int(len(tk)),
        C.c_int(max_report), _ptr(rep[0]), _ptr(rep[1]), _ptr(rep[2]), _ptr(rep[3]),
        _ptr(gap), _ptr(worst), (C.c_float if net.real == "float" else C.c_double)(tol))
    where = [dict(t=int(rep[0][i]), u=int(rep[1][i]), want=int(rep[2][i]),
                  got=int(rep[3][i]), gap=float(gap[i]))
             for i in range(max(0, min(n, max_report)))]
    return Followed(int(n), float(worst[0]), where)


def quantize_rows_e4m3(w: np.ndarray, real: str = "float"):
    """(quantised copy, row scales) of a 2-D matrix: every row as e4m3 values times a power
    of two of its own (orc_quantize_rows_e4m3)."""
    dt = _np_real(real)
    w = np.ascontiguousarray(w, dtype=dt)
    assert w.ndim == 2
    out = np.empty_like(w)
    scales = np.empty(w.shape[0], dtype=dt)
    _lib(real).orc_quantize_rows_e4m3(w.ctypes.data, w.shape[0], w.shape[1], out.ctypes.data,
                                      scales.ctypes.data)
    return out, scales


def quantize_blocks_e2m1(w: np.ndarray, block: int = 128, real: str = "float"):
    """(quantised copy, block scales [rows, ceil(cols / block)]) of a 2-D matrix: every block
    of `block` consecutive weights of a row as e2m1 values times a power of two
    (orc_quantize_blocks_e2m1)."""
    dt = _np_real(real)
    w = np.ascontiguousarray(w, dtype=dt)
    assert w.ndim == 2
    out = np.empty_like(w)
    scales = np.empty((w.shape[0], (w.shape[1] + block - 1) // block), dtype=dt)
    _lib(real).orc_quantize_blocks_e2m1(w.ctypes.data, w.shape[0], w.shape[1], block, out.ctypes.data,
                                        scales.ctypes.data)
    return out, scales
