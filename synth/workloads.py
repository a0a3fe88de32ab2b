"""Synthetic decoder weights and encoder outputs with the shapes of the five
benchmark configurations (tiny, small, Parakeet-1.1B-shaped RNN-T with frame
looping and label looping, TDT-shaped).

Nothing here evaluates the networks: the module draws numbers, scales them and
stores them in the PyTorch layout (Linear / LSTM weights are [out, in], LSTM
gate order i, f, g, o).
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, List, Optional, Tuple

import numpy as np

from . import rng


@dataclass(frozen=True)
class ModelDims:
    F: int            # encoder output features
    E: int            # embedding width
    H: int            # LSTM hidden width
    L: int            # LSTM layers
    J: int            # joint hidden width
    V1: int           # vocabulary including blank
    durations: Tuple[int, ...] = ()   # TDT durations; empty for RNN-T
    big_blanks: Tuple[int, ...] = ()  # multi-blank transducer: spans of the big-blank symbols

    @property
    def D(self) -> int:
        return len(self.durations)

    @property
    def NB(self) -> int:
        return len(self.big_blanks)

    @property
    def blank(self) -> int:
        return self.V1 - 1

    @property
    def n_out(self) -> int:
        return self.V1 + self.D + self.NB


def param_count(d: ModelDims) -> int:
    """Number of decoder parameters (embedding, LSTM with two bias vectors per
    layer, the three joint linears)."""
    n = d.V1 * d.E
    for l in range(d.L):
        n_in = d.E if l == 0 else d.H
        n += 4 * d.H * (n_in + d.H) + 8 * d.H
    n += d.F * d.J + d.J
    n += d.H * d.J + d.J
    n += d.J * d.n_out + d.n_out
    return n


@dataclass
class Model:
    dims: ModelDims
    emb: np.ndarray                 # [V1, E]
    w_ih: List[np.ndarray]          # L x [4H, in_l]
    w_hh: List[np.ndarray]          # L x [4H, H]
    b_ih: List[np.ndarray]          # L x [4H]
    b_hh: List[np.ndarray]          # L x [4H]
    w_enc: np.ndarray               # [J, F]
    b_enc: np.ndarray               # [J]
    w_pred: np.ndarray              # [J, H]
    b_pred: np.ndarray              # [J]
    w_out: np.ndarray               # [V1 + D, J]
    b_out: np.ndarray               # [V1 + D]
    durations: np.ndarray           # int32 [D]

    def arrays(self) -> Dict[str, np.ndarray]:
        out = {"emb": self.emb, "w_enc": self.w_enc, "b_enc": self.b_enc,
               "w_pred": self.w_pred, "b_pred": self.b_pred,
               "w_out": self.w_out, "b_out": self.b_out}
        for l in range(self.dims.L):
            out[f"w_ih{l}"] = self.w_ih[l]
            out[f"w_hh{l}"] = self.w_hh[l]
            out[f"b_ih{l}"] = self.b_ih[l]
            out[f"b_hh{l}"] = self.b_hh[l]
        return out


def make_model(dims: ModelDims, seed: int, *, weight_range: float = 0.1,
               emb_gain: float = 1.0, pred_gain: float = 1.0,
               blank_bias: float = 0.0,
               dur_bias: Optional[Tuple[float, ...]] = None,
               big_blank_bias: Optional[Tuple[float, ...]] = None,
               tie: Optional[Tuple[float, float, float]] = None) -> Model:
    """Weights ~ U(-weight_range, weight_range).

    emb_gain scales the embedding table and pred_gain the prediction-side joint
    projection, so that the logits move after each emitted label as they do in
    a trained model.  The embedding row of the blank index is zero: it is the
    start-of-sequence input.  blank_bias is added to the blank logit's bias,
    dur_bias to the duration logits' biases and big_blank_bias to the biases of a
    multi-blank model's big-blank logits (the output columns after the V1 tokens).

    tie = (beta, s, gamma), for E == H == J only, adds structure that makes an
    emitted label lower its own logit on the next step, as a trained transducer
    does: the embedding of label k gets -beta times row k of the output
    projection (tied input and output embeddings), the cell-candidate block of
    every LSTM layer's input weights gets s times the identity, and the
    prediction-side joint projection gets gamma times the identity, so the
    direction of the last label's output row passes through to the joint.
    """
    a = weight_range
    s = 0

    def U(shape):
        nonlocal s
        s += 1
        return rng.uniform(seed, s, shape, -a, a)

    emb = U((dims.V1, dims.E)) * np.float32(emb_gain)
    emb[dims.blank, :] = 0.0
    w_ih, w_hh, b_ih, b_hh = [], [], [], []
    for l in range(dims.L):
        n_in = dims.E if l == 0 else dims.H
        w_ih.append(U((4 * dims.H, n_in)))
        w_hh.append(U((4 * dims.H, dims.H)))
        b_ih.append(U((4 * dims.H,)))
        b_hh.append(U((4 * dims.H,)))
    w_enc = U((dims.J, dims.F))
    b_enc = U((dims.J,))
    w_pred = U((dims.J, dims.H)) * np.float32(pred_gain)
    b_pred = U((dims.J,))
    w_out = U((dims.n_out, dims.J))
    b_out = U((dims.n_out,))
    b_out[dims.blank] += np.float32(blank_bias)
    if tie is not None:
        beta, s_id, gamma = (np.float32(v) for v in tie)
        assert dims.E == dims.H == dims.J, "tie needs E == H == J"
        H = dims.H
        eye = np.eye(H, dtype=np.float32)
        for k in range(dims.V1):
            if k != dims.blank:
                emb[k, :] -= beta * w_out[k, :]
        for l in range(dims.L):
            w_ih[l][2 * H:3 * H, :] += s_id * eye
        w_pred += gamma * eye
    if dur_bias is not None:
        assert len(dur_bias) == dims.D
        b_out[dims.V1:dims.V1 + dims.D] += np.asarray(dur_bias, dtype=np.float32)
    if big_blank_bias is not None:
        assert len(big_blank_bias) == dims.NB
        b_out[dims.V1 + dims.D:] += np.asarray(big_blank_bias, dtype=np.float32)
    return Model(dims, emb, w_ih, w_hh, b_ih, b_hh, w_enc, b_enc, w_pred,
                 b_pred, w_out, b_out,
                 np.asarray(dims.durations, dtype=np.int32))


def make_inputs(seed: int, B: int, T: int, F: int, len_lo: int, len_hi: int,
                *, sort_desc: bool = False, pad: str = "normal"):
    """enc_out float32 [B, T, F] ~ N(0,1) and enc_len int32 [B] uniform on
    len_lo..len_hi.  Frames at t >= enc_len[b] are padding: 'normal' leaves the
    random values, 'nan' poisons them, 'zero' clears them."""
    enc_len = rng.randint(seed, 101, (B,), len_lo, len_hi)
    if sort_desc:
        enc_len = np.sort(enc_len)[::-1].copy()
    enc_out = rng.normal(seed, 102, (B, T, F))
    if pad != "normal":
        fill = np.float32(np.nan) if pad == "nan" else np.float32(0.0)
        for b in range(B):
            enc_out[b, enc_len[b]:, :] = fill
    return enc_out, enc_len.astype(np.int32)


@dataclass
class Workload:
    name: str
    variant: str          # "frame", "label" or "tdt"
    model: Model
    enc_out: np.ndarray   # [B, T, F]
    enc_len: np.ndarray   # [B]
    max_symbols: int

    @property
    def B(self) -> int:
        return int(self.enc_out.shape[0])

    @property
    def T(self) -> int:
        return int(self.enc_out.shape[1])

    @property
    def frames(self) -> int:
        return int(self.enc_len.sum())


# Model-side knobs per configuration.  The blank biases of the Parakeet-shaped
# and TDT-shaped configurations were found by oracle/tune_blank_bias.py (it
# bisects on the blank rate of the oracle's joint evaluations).
_PARAKEET = ModelDims(F=1024, E=640, H=640, L=2, J=640, V1=1025)
_TDT = replace(_PARAKEET, durations=(0, 1, 2, 3, 4))

CONFIGS = {
    0: dict(name="tiny", variant="frame", seed=0,
            dims=ModelDims(F=64, E=64, H=64, L=1, J=64, V1=17),
            B=1, T=20, len_lo=20, len_hi=20, sort_desc=False, S=3,
            model_kw=dict()),
    1: dict(name="small", variant="frame", seed=1,
            dims=ModelDims(F=256, E=320, H=320, L=1, J=320, V1=257),
            B=8, T=200, len_lo=100, len_hi=200, sort_desc=False, S=5,
            model_kw=dict(blank_bias=2.0, tie=(5.0, 2.0, 5.0))),
    2: dict(name="parakeet_frame", variant="frame", seed=2, dims=_PARAKEET,
            B=32, T=500, len_lo=200, len_hi=500, sort_desc=True, S=10,
            model_kw=dict(blank_bias=8.21, tie=(5.0, 2.0, 5.0))),
    3: dict(name="parakeet_label", variant="label", seed=2, dims=_PARAKEET,
            B=32, T=500, len_lo=200, len_hi=500, sort_desc=True, S=10,
            model_kw=dict(blank_bias=8.21, tie=(5.0, 2.0, 5.0))),
    4: dict(name="tdt_label", variant="tdt", seed=4, dims=_TDT,
            B=32, T=500, len_lo=200, len_hi=500, sort_desc=True, S=10,
            model_kw=dict(blank_bias=7.71, tie=(5.0, 2.0, 5.0))),
    # Second workload: the smaller model of the paper's results table.  The paper does not give
    # its decoder's shape; a single LSTM layer at the same widths is this build's guess.
    5: dict(name="small_model_label", variant="label", seed=5,
            dims=replace(_PARAKEET, L=1),
            B=32, T=500, len_lo=200, len_hi=500, sort_desc=True, S=10,
            model_kw=dict(blank_bias=8.73, tie=(5.0, 2.0, 5.0))),
    # Multi-blank transducer at the Parakeet shape: two big blanks that skip 2 and 4 frames
    # (the related-work neighbour of TDT).  Biases chosen on the oracle so that the batch looks
    # like configuration 3's: 1 697 labels (at most 105 per utterance) in 8 272 joint
    # evaluations, a third of the blank decisions taken by a big blank.
    6: dict(name="multi_blank_label", variant="label", seed=6,
            dims=replace(_PARAKEET, big_blanks=(2, 4)),
            B=32, T=500, len_lo=200, len_hi=500, sort_desc=True, S=10,
            model_kw=dict(blank_bias=6.5, big_blank_bias=(5.5, 5.3), tie=(5.0, 2.0, 5.0))),
}


def make_workload(cfg: int, *, B: Optional[int] = None, pad: str = "normal",
                  T: Optional[int] = None, len_lo: Optional[int] = None,
                  len_hi: Optional[int] = None,
                  model_overrides: Optional[dict] = None) -> Workload:
    """Build configuration `cfg`.

    For the Parakeet-shaped and TDT-shaped configurations B may be any value:
    the batch is assembled from independently seeded blocks of 32 utterances
    (block j uses seed + 1000*j), so the first 32 rows of B=128 and the single
    row of B=1 are rows of the B=32 workload.  T, len_lo and len_hi shrink the
    time axis for cut-down test cases.
    """
    c = CONFIGS[cfg]
    dims: ModelDims = c["dims"]
    kw = dict(c["model_kw"])
    if model_overrides:
        kw.update(model_overrides)
    model = make_model(dims, c["seed"], **kw)
    T_ = c["T"] if T is None else T
    lo = c["len_lo"] if len_lo is None else len_lo
    hi = c["len_hi"] if len_hi is None else len_hi
    base_B = c["B"]
    want_B = base_B if B is None else B
    blocks_x, blocks_len = [], []
    n_blocks = (want_B + base_B - 1) // base_B
    for j in range(n_blocks):
        x, ln = make_inputs(c["seed"] + 1000 * j, base_B, T_, dims.F, lo, hi,
                            sort_desc=c["sort_desc"], pad=pad)
        blocks_x.append(x)
        blocks_len.append(ln)
    enc_out = np.concatenate(blocks_x, axis=0)[:want_B].copy()
    enc_len = np.concatenate(blocks_len, axis=0)[:want_B].copy()
    return Workload(c["name"], c["variant"], model, enc_out, enc_len, c["S"])


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """float32 array with every value rounded to the nearest bf16 value (ties to even) and
    stored as float32 again."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    r = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16) << 16
    return r.astype(np.uint32).view(np.float32).reshape(a.shape)


def round_to_e4m3(a: np.ndarray) -> np.ndarray:
    """float32 array with every value rounded to the nearest value of the 8-bit OCP e4m3
    format (1 sign, 4 exponent bits with bias 7, 3 mantissa bits; subnormals are multiples of
    2^-9; largest value 448, larger inputs saturate), ties to even, stored as float32."""
    x = np.ascontiguousarray(a, dtype=np.float32).astype(np.float64)
    mag = np.minimum(np.abs(x), 448.0)
    _, e = np.frexp(mag)                       # mag = m * 2^e, 0.5 <= m < 1
    quantum = np.ldexp(1.0, np.maximum(e - 1, -6) - 3)
    r = np.minimum(np.rint(mag / quantum) * quantum, 448.0)
    return np.copysign(r, x).astype(np.float32).reshape(a.shape)


def _with_streamed_weights(model: Model, f) -> Model:
    w_ih = [w if l == 0 else f(w) for l, w in enumerate(model.w_ih)]
    w_hh = [f(w) for w in model.w_hh]
    return replace(model, w_ih=w_ih, w_hh=w_hh, w_pred=f(model.w_pred), w_out=f(model.w_out))


def with_streamed_weights(model: Model, f) -> Model:
    """A copy of `model` with f applied to each per-step streamed matrix (W_hh of every layer,
    W_ih of the layers above the first, W_pred, W_out); f maps a 2-D float32 array to one of
    the same shape (a quantiser under test, for instance)."""
    return _with_streamed_weights(model, f)


def with_fp8_streamed_weights(model: Model) -> Model:
    """Like with_bf16_streamed_weights, with e4m3 values: the model an 8-bit weight-only
    checkpoint (without scale factors) would give for the streamed matrices."""
    return _with_streamed_weights(model, round_to_e4m3)


def with_bf16_streamed_weights(model: Model) -> Model:
    """A copy of `model` whose per-step streamed matrices (W_hh of every layer, W_ih of the
    layers above the first, W_pred, W_out) hold bf16 values; everything else is unchanged.
    This is the model a bf16 checkpoint would give for those matrices; both the oracle and the
    engine take it as their fp32 input."""
    return _with_streamed_weights(model, round_to_bf16)
