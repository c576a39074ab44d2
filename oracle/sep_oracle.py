"""CPU oracle for the shadow-model side of OD-MoE's SEP predictor  --  TEST INFRASTRUCTURE ONLY.

The paper's predictor (Sections 1, 3.2) is a quantised copy of the model (FP16 / INT8 / NF4 in
the paper) that runs ahead of the full-precision model; its routing decisions are the expert
predictions, scored by the recall of Section 3.2.  The paper does not print its quantisers; the
readings taken for the synthetic emulation are the plain symmetric absmax schemes:

  int8, per weight row :  s = max|w| / 127,  q = clip(rne(w / s), -127, 127),  w' = q * s
  int4, per group of 64 consecutive weights of a row:  s = max|w| / 7,  q = clip(rne(w / s), -7, 7)

  fp16: w' = the IEEE binary16 value nearest to w (ties to even), |w| clipped to 65504 first
  (the paper's FP16 shadow of an FP32 model)

(rne = round half to even; an all-zero row / group keeps scale 0 and stays zero.)  The shadow
stack then holds w' rounded to the storage dtype.  NF4's code book is not reproduced; the 4-bit
scheme here is uniform, so its recall is not comparable to the paper's NF4 number.

Pins (tests/test_sep_cpu.py): error bound |w - w'| <= s/2, exactness on grid points, idempotence,
zero rows, sign symmetry, hand-worked rows, binary16 values worked by hand (ties, subnormals,
clipping), and agreement of the recall bookkeeping with
moe_oracle.recall.  Shares no code with the product's quantiser; tests compare the two bit for bit.
"""
from __future__ import annotations

import numpy as np


def quantize_rows_int8(W: np.ndarray):
    """Symmetric absmax int8 per row.  Returns (q int8 [R, C], scale float64 [R])."""
    W = np.asarray(W, dtype=np.float64)
    amax = np.max(np.abs(W), axis=1)
    scale = amax / 127.0
    safe = np.where(scale > 0, scale, 1.0)
    q = np.clip(np.rint(W / safe[:, None]), -127, 127)
    q = np.where(scale[:, None] > 0, q, 0.0)
    return q.astype(np.int8), scale


def quantize_groups_int4(W: np.ndarray, group: int = 64):
    """Symmetric absmax 4-bit (levels -7..7) per group of `group` consecutive elements of a row.
    Returns (q int8 [R, C] holding -7..7, scale float64 [R, C/group])."""
    W = np.asarray(W, dtype=np.float64)
    R, C = W.shape
    if C % group:
        raise ValueError("row length must be a multiple of the group size")
    G = W.reshape(R, C // group, group)
    amax = np.max(np.abs(G), axis=2)
    scale = amax / 7.0
    safe = np.where(scale > 0, scale, 1.0)
    q = np.clip(np.rint(G / safe[:, :, None]), -7, 7)
    q = np.where(scale[:, :, None] > 0, q, 0.0)
    return q.reshape(R, C).astype(np.int8), scale


def round_fp16(W: np.ndarray):
    """Nearest IEEE binary16 value (ties to even) of every element, |w| clipped to 65504.
    Returns (bits uint16, values float64)."""
    h = np.clip(np.asarray(W, dtype=np.float64), -65504.0, 65504.0).astype(np.float16)
    return h.view(np.uint16), h.astype(np.float64)


def dequantize_rows(q: np.ndarray, scale: np.ndarray) -> np.ndarray:
    return q.astype(np.float64) * np.asarray(scale, dtype=np.float64)[:, None]


def dequantize_groups(q: np.ndarray, scale: np.ndarray, group: int = 64) -> np.ndarray:
    R, C = q.shape
    return (q.astype(np.float64).reshape(R, C // group, group) * scale[:, :, None]).reshape(R, C)


def shadow_matrix(W: np.ndarray, kind: str) -> np.ndarray:
    """float64 values of the shadow copy of W ('bf16': unchanged, 'fp16', 'int8', 'int4')."""
    W = np.asarray(W, dtype=np.float64)
    if kind == "bf16":
        return W.copy()
    if kind == "fp16":
        return round_fp16(W)[1]
    if kind == "int8":
        return dequantize_rows(*quantize_rows_int8(W))
    if kind == "int4":
        return dequantize_groups(*quantize_groups_int4(W))
    raise ValueError(kind)
