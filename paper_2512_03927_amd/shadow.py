"""Shadow copies of a synthetic MoE stack for the emulation of OD-MoE's SEP predictor.

The paper's predictor (Sections 1, 3.2) runs a quantised copy of the model ahead of the
full-precision one and uses its routing as the expert prediction.  Here the copy is a second
stack on the same GPU, built from the full stack's stored weights by the library's own quantiser
(`odmoe_quantize`, `odmoe_quantize_expert`):

  'bf16'  an identical copy (the predictor that is always right)
  'fp16'  fp32 stacks only: experts rounded to IEEE binary16, read by the binary16 GEMV kernels
          (half the bytes per token): the paper's FP16 shadow of its FP32 model
  'int8'  experts as int8 codes with a scale per weight row, read by the int8 GEMV kernels (half
          the bytes per token)
  'int4'  experts as packed 4-bit codes with a scale per group of 64 weights, read by the 4-bit
          GEMV kernels (0.28 of the bytes per token)

In every quantised copy the router is quantised the same way and held dequantised in the storage
dtype (it is tiny).  This module only moves buffers and calls the library (marshalling);
`emulate` is `odmoe_sep_emulate`.
"""
from __future__ import annotations

from typing import List, Sequence

import torch

from . import binding as B
from . import harness, synth

QUANT_OF_KIND = {"int8": B.ODMOE_Q_INT8_ROW, "int4": B.ODMOE_Q_INT4_G64, "fp16": B.ODMOE_Q_F16}


def _dtype_code(cfg: synth.MoEConfig) -> int:
    return B.ODMOE_F32 if cfg.dtype == "f32" else B.ODMOE_BF16


def shadow_stack(cfg: synth.MoEConfig, layers: Sequence, kind: str, device: str = "cuda:0") -> harness.MoEStack:
    """A resident stack of cfg's shape whose weights are the `kind` copy of `layers` (stored
    per-layer (Wg, b, experts) as synth makes them)."""
    if kind not in ("bf16", "fp16", "int8", "int4"):
        raise ValueError(kind)
    rcfg = cfg.small(n_slots=0)
    if kind == "bf16":
        return harness.MoEStack(rcfg, list(layers), device=device)
    dt, td = _dtype_code(cfg), harness.torch_dtype(cfg.dtype)
    qkind = QUANT_OF_KIND[kind]
    H, F, E = cfg.hidden, cfg.ffn, cfg.n_experts
    stream = torch.cuda.current_stream(torch.device(device)).cuda_stream
    c = B.odmoe_config(H, F, E, cfg.top_k, 1, 0, dt, 0, qkind)
    q_bytes = B.odmoe_expert_bytes(c)
    if q_bytes == 0:
        raise ValueError(f"{kind} experts do not take this shape: {B.odmoe_last_error()}")
    routers, biases, experts_all = [], [], []
    for (Wg, b, experts) in layers:
        src = harness.to_device(Wg, device)
        r = torch.empty((E, H), dtype=td, device=device)
        B.odmoe_quantize(src, dt, E, H, qkind, None, None, r, stream)
        routers.append(r)
        biases.append(None if b is None else harness.to_device(b, device))
        ex: List[torch.Tensor] = []
        for flat in experts:
            src = harness.to_device(flat, device)
            dst = torch.empty(q_bytes, dtype=torch.uint8, device=device)
            B.odmoe_quantize_expert(c, qkind, src, dst, stream)
            torch.cuda.synchronize()        # src may be freed
            ex.append(dst)
        experts_all.append(ex)
    return harness.MoEStack(rcfg, device=device, device_buffers=(routers, biases, experts_all),
                            unique_layers=len(routers), expert_quant=qkind)


def emulate(main: harness.MoEStack, shadow: harness.MoEStack, x0: torch.Tensor, n_iter: int, aligned: bool):
    """`n_iter` emulated decode iterations (odmoe_sep_emulate): the shadow stack's routing is the
    main stack's prediction, main's output is its next input; aligned=True restarts the shadow from
    main's input every iteration.  Returns (recall per iteration, main's final output tensor,
    wall ms spent in the shadow's steps, wall ms spent in main's steps)."""
    x_end = torch.empty_like(x0)
    rec, shadow_ms, main_ms = B.odmoe_sep_emulate(main.handle, shadow.handle, x0, n_iter, aligned, x_end)
    return rec, x_end, shadow_ms, main_ms
