"""Shadow copies of a synthetic MoE stack and the emulation of OD-MoE's SEP predictor with them.

The paper's predictor (Sections 1, 3.2) runs a quantised copy of the model ahead of the
full-precision one and uses its routing as the expert prediction; token / KV-cache alignment
periodically resets the copy's state to the full model's.  Here the copy is a second stack on
the same GPU whose weights went through a quantise -> dequantise round trip on the host (the
kernels still run in the storage dtype: what is emulated is the routing drift that quantisation
causes, not the copy's speed).  Its per-layer expert indices are handed to the full stack as
`predicted_idx_host`; the full stack's router verifies them (hits / reloads = recall).

There is no attention and no KV cache in this build, so a "decode iteration" is emulated by
feeding the stack's output back as the next token's input; "alignment" means the copy starts
every iteration from the full stack's input instead of its own.
"""
from __future__ import annotations

from typing import List, Sequence

import numpy as np

from . import synth


def _to_f32(stored: np.ndarray) -> np.ndarray:
    return synth.bf16_bits_to_f32(stored) if stored.dtype == np.uint16 else stored.astype(np.float32)


def quantize_dequantize(W_f32: np.ndarray, kind: str, group: int = 64) -> np.ndarray:
    """Round trip of a [rows, cols] matrix through symmetric absmax quantisation.
    kind: 'bf16' (no change), 'int8' (per row, 127 levels each side), 'int4' (per group of
    `group` elements of a row, 7 levels each side).  Rounding is half-to-even."""
    W = W_f32.astype(np.float64)
    if kind == "bf16":
        return W
    if kind == "int8":
        s = np.abs(W).max(axis=1, keepdims=True) / 127.0
        lim = 127
    elif kind == "int4":
        r, c = W.shape
        if c % group:
            raise ValueError("row length must be a multiple of the group size")
        W = W.reshape(r, c // group, group)
        s = np.abs(W).max(axis=2, keepdims=True) / 7.0
        lim = 7
    else:
        raise ValueError(kind)
    div = np.where(s > 0, s, 1.0)
    q = np.clip(np.rint(W / div), -lim, lim) * (s > 0)
    out = q * s
    return out.reshape(W_f32.shape)


def shadow_layers(cfg: synth.MoEConfig, layers: Sequence, kind: str) -> List:
    """Per-layer (Wg, b, experts) of the shadow copy, in cfg's storage dtype."""
    out = []
    H, F = cfg.hidden, cfg.ffn
    for (Wg, b, experts) in layers:
        Wg_s = synth.store(quantize_dequantize(_to_f32(Wg), kind).astype(np.float32), cfg.dtype)
        ex_s = []
        for flat in experts:
            f = _to_f32(flat)
            parts = [quantize_dequantize(f[:H * F].reshape(F, H), kind),
                     quantize_dequantize(f[H * F:2 * H * F].reshape(F, H), kind),
                     quantize_dequantize(f[2 * H * F:].reshape(H, F), kind)]
            ex_s.append(synth.store(np.concatenate([p.ravel() for p in parts]).astype(np.float32), cfg.dtype))
        out.append((Wg_s, b, ex_s))
    return out


def emulate(main, shadow, x0, n_iter: int, aligned: bool, period: int = 1):
    """Runs `n_iter` emulated decode iterations.

    main, shadow: harness.MoEStack of the same shape (main may be cacheless).  x0: device tensor [H].
    Each iteration the shadow stack produces its routing for all layers, the main stack decodes
    with those as hints, and the main stack's output becomes the next input.  aligned=True
    restarts the shadow from the main stack's input every `period` iterations (the alignment
    period of Section 3.2; 1 = every iteration) and lets it follow its own outputs in between;
    aligned=False never realigns.  Returns (recall per iteration: list of float, final main
    output tensor).
    """
    if period < 1:
        raise ValueError("period must be >= 1")
    L, k = main.cfg.n_layers, main.cfg.top_k
    x_main = x0
    x_shadow = x0
    recalls = []
    for it in range(n_iter):
        y_s, idx_s, _ = shadow.decode(x_main if (aligned and it % period == 0) else x_shadow)
        y_m, idx_m, st = main.decode(x_main, pred=idx_s)
        if main.cfg.n_slots > 0:
            hits = st.hint_hits
        else:  # resident main stack: count on the host
            hits = sum(len(set(idx_s[l]) & set(idx_m[l])) for l in range(L))
        recalls.append(hits / float(L * k))
        x_main, x_shadow = y_m, y_s
    return recalls, x_main
