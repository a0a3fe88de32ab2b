"""Adversarial encoder outputs: frames that force a blank, frames that force
max_symbols emissions, and batch patterns built from them.

The paper's discussion of batched greedy decoding rests on two such inputs: a
batch of two utterances of which one emits max_symbols labels on even frames
and a blank on odd frames while the other does the opposite (the case that
makes lock-step frame looping run max_symbols inner steps on every frame, in
the section on label looping), and the remark that an adversary can make every
frame produce max_symbols labels (the discussion of the experiments).  Real
audio is not needed for either: the frames below are solved for from the joint
network's weights.

Nothing here runs the decoder.  A frame is the least-squares solution f of
W_enc f + b_enc = p for a wanted projected frame p:
  * blank frame:  p = -s everywhere.  The joint hidden vector relu(p + q) is
    zero for every prediction-side term q smaller than s, the logits are then
    the output bias, and the configurations' blank bias makes blank the argmax.
  * emit frame:   p_j = s * max(-W_out[blank, j], 0).  Every hidden unit that
    lowers the blank logit is driven hard, so blank loses on every evaluation
    on this frame whatever q is (for |q| much smaller than s), and the frame
    emits max_symbols labels.
"""
from __future__ import annotations

import numpy as np

from .workloads import Model, Workload, make_workload

PATTERNS = ("all_blank", "always_max", "alternating", "one_slow_row")


def steer_frames(model: Model, strength: float = 1000.0):
    """(blank_frame, emit_frame), float32 [F] each."""
    d = model.dims
    if d.F < d.J:
        raise ValueError("steering needs F >= J: W_enc must reach every projected frame")
    W = model.w_enc.astype(np.float64)
    b = model.b_enc.astype(np.float64)
    w_blank = model.w_out[d.blank].astype(np.float64)
    want_blank = np.full(d.J, -strength)
    want_emit = strength * np.maximum(-w_blank, 0.0)
    f_blank = np.linalg.lstsq(W, want_blank - b, rcond=None)[0]
    f_emit = np.linalg.lstsq(W, want_emit - b, rcond=None)[0]
    return f_blank.astype(np.float32), f_emit.astype(np.float32)


def emit_mask(pattern: str, B: int, T: int) -> np.ndarray:
    """bool [B, T]: True where row b's frame t is an emit frame."""
    t = np.arange(T)[None, :]
    b = np.arange(B)[:, None]
    if pattern == "all_blank":
        return np.zeros((B, T), dtype=bool)
    if pattern == "always_max":
        return np.ones((B, T), dtype=bool)
    if pattern == "alternating":
        return (t + b) % 2 == 0
    if pattern == "one_slow_row":
        return np.broadcast_to(b == 0, (B, T)).copy()
    raise ValueError(f"unknown pattern '{pattern}' (one of {PATTERNS})")


def make_adversarial(pattern: str, *, cfg: int = 2, B: int = 2, T: int = 16) -> Workload:
    """Configuration cfg's model with a [B, T, F] batch of steered frames; every
    utterance is T frames long."""
    w = make_workload(cfg, B=1, T=1, len_lo=1, len_hi=1)
    f_blank, f_emit = steer_frames(w.model)
    mask = emit_mask(pattern, B, T)
    enc_out = np.where(mask[:, :, None], f_emit[None, None, :], f_blank[None, None, :])
    enc_out = np.ascontiguousarray(enc_out, dtype=np.float32)
    enc_len = np.full((B,), T, dtype=np.int32)
    return Workload(f"{w.name}_{pattern}", w.variant, w.model, enc_out, enc_len, w.max_symbols)
