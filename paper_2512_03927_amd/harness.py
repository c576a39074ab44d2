"""Plumbing between stored NumPy buffers, torch device/pinned memory and the C-ABI handle.

No arithmetic of the method happens here: buffers are uploaded, pointers are
handed to libodmoe.so, results are downloaded.
"""
from __future__ import annotations

from typing import List, Optional, Sequence, Tuple

import numpy as np
import torch

from . import binding as B
from . import synth

LayerWeights = Tuple[np.ndarray, Optional[np.ndarray], Sequence[np.ndarray]]  # (Wg, b, experts)


def to_device(a: np.ndarray, device: str = "cuda:0") -> torch.Tensor:
    """Stored buffer -> device tensor (uint16 bf16 bit patterns become torch.bfloat16)."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(a).to(device)


def from_device(t: torch.Tensor) -> np.ndarray:
    """Device tensor -> stored buffer (bf16 comes back as uint16 bit patterns)."""
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def torch_dtype(dtype: str) -> torch.dtype:
    return {"f32": torch.float32, "bf16": torch.bfloat16}[dtype]


def pinned_like(a: np.ndarray) -> torch.Tensor:
    """Copy a stored buffer into freshly allocated pinned host memory."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        t = torch.empty(a.shape, dtype=torch.int16, pin_memory=True)
        t.numpy()[...] = a.view(np.int16)
        return t
    t = torch.empty(a.shape, dtype=torch.from_numpy(a[:0]).dtype, pin_memory=True)
    t.numpy()[...] = a
    return t


class MoEStack:
    """Owns the device / pinned copies of a stack's weights and its libodmoe handle."""

    def __init__(self, cfg: synth.MoEConfig, layers: Optional[Sequence[LayerWeights]] = None,
                 unique_layers: Optional[int] = None, device: str = "cuda:0",
                 copy_stream: Optional[torch.cuda.Stream] = None, experts_in_host_memory: bool = False,
                 buffers_of: Optional["MoEStack"] = None, buffer_layers: Optional[Sequence[int]] = None,
                 device_buffers=None, expert_quant: int = B.ODMOE_Q_NONE):
        """layers: per-layer stored weights; generated from `cfg` when None.

        experts_in_host_memory (with cfg.n_slots == 0): the experts stay in pinned host memory and
        the handle is given those addresses, so the kernels read the weights across the host link.

        unique_layers = U < L keeps only U distinct layers' weights and maps layer l to
        l mod U (same bytes moved per token, less host memory).

        buffers_of: another stack of the same layers whose router and expert buffers this one
        shares instead of making its own copies (it must outlive this stack's use);
        buffer_layers picks which of its unique layers, in order (default: all of them).

        device_buffers = (router tensors [U], bias tensors or None [U], expert tensors [U][E]):
        buffers that already exist (device memory, or pinned host memory for a slot pool), for
        example the quantised weights the library's quantiser wrote; `layers` is then not used.
        expert_quant: the odmoe_quant format of the expert buffers (int8 rows for a shadow stack).
        """
        self.cfg = cfg
        self.device = device
        L, E = cfg.n_layers, cfg.n_experts
        U = L if unique_layers is None else min(unique_layers, L)
        self.unique_layers = U
        self.expert_quant = expert_quant
        if device_buffers is not None:
            layers = [None] * len(device_buffers[0])
        elif layers is None:
            layers = [synth.layer_weights(cfg, l) for l in range(U)]
        assert len(layers) in (U, L)
        self.layers_np = list(layers)
        nl = len(self.layers_np)
        self._keep: List[torch.Tensor] = []
        router_w, router_b, expert_w = [], [], []
        uniq_router, uniq_bias, uniq_experts = [], [], []
        if buffers_of is not None:
            uniq_router, uniq_bias, uniq_experts = buffers_of._keep
            if buffer_layers is not None:
                uniq_router, uniq_bias, uniq_experts = ([lst[i] for i in buffer_layers]
                                                        for lst in (uniq_router, uniq_bias, uniq_experts))
            assert len(uniq_experts) == nl
        if device_buffers is not None:
            uniq_router, uniq_bias, uniq_experts = (list(v) for v in device_buffers)
        for (Wg, b, experts) in ([] if (buffers_of is not None or device_buffers is not None) else self.layers_np):
            uniq_router.append(to_device(Wg, device))
            uniq_bias.append(None if b is None else to_device(np.asarray(b, np.float32), device))
            if cfg.n_slots == 0 and not experts_in_host_memory:
                uniq_experts.append([to_device(e, device) for e in experts])
            else:
                uniq_experts.append([pinned_like(e) for e in experts])
        for l in range(L):
            u = l % nl
            router_w.append(uniq_router[u])
            router_b.append(uniq_bias[u])
            expert_w.extend(uniq_experts[u])
        self._keep = [uniq_router, uniq_bias, uniq_experts]
        c = B.odmoe_config(cfg.hidden, cfg.ffn, E, cfg.top_k, L, cfg.n_slots,
                           B.ODMOE_F32 if cfg.dtype == "f32" else B.ODMOE_BF16, cfg.glue, expert_quant)
        self.expert_bytes = B.odmoe_expert_bytes(c)
        self.stream = torch.cuda.current_stream(torch.device(device))
        self.copy_stream = copy_stream
        has_bias = any(b is not None for b in router_b)
        self.handle = B.odmoe_layer_init(
            c, router_w, router_b if has_bias else None, expert_w, self.stream.cuda_stream,
            None if copy_stream is None else copy_stream.cuda_stream)

    # -- small conveniences around the C calls (marshalling only) --
    def empty_x(self, n: int = 1) -> torch.Tensor:
        return torch.empty((n, self.cfg.hidden), dtype=torch_dtype(self.cfg.dtype), device=self.device)

    def route(self, layer: int, x: torch.Tensor):
        T = x.shape[0]
        idx = torch.empty((T, self.cfg.top_k), dtype=torch.int32, device=self.device)
        gate = torch.empty((T, self.cfg.top_k), dtype=torch.float32, device=self.device)
        B.odmoe_route_topk(self.handle, layer, x, T, idx, gate)
        return idx, gate

    def ffn(self, layer: int, idx, gate, x, idx_host=None, evict_after: int = 1) -> torch.Tensor:
        y = torch.empty_like(x)
        B.odmoe_expert_ffn(self.handle, layer, idx, gate, idx_host, x, x.shape[0], y, evict_after)
        return y

    def decode(self, x: torch.Tensor, pred: Optional[np.ndarray] = None, timed: bool = False):
        """One token through the stack.  Returns (y tensor [H], idx int32[L,k], stats)."""
        y = torch.empty_like(x)
        idx_out = np.zeros((self.cfg.n_layers, self.cfg.top_k), dtype=np.int32)
        st = B.odmoe_stats()
        st.t_step_ms = -1.0 if timed else 0.0
        if pred is not None:
            pred = np.ascontiguousarray(pred, dtype=np.int32)
        B.odmoe_decode_step(self.handle, x, y, pred, idx_out, st)
        return y, idx_out, st

    def close(self) -> None:
        if self.handle is not None:
            B.odmoe_layer_destroy(self.handle)
            self.handle = None
        self._keep = []

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()
