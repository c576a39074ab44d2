"""Seeded synthetic inputs for the cacheless MoE decode layer.

This module only *materialises buffers*: it holds none of the method's
arithmetic (no routing, no gate, no FFN).  The CPU oracle and the HIP path are
both fed the buffers made here, so they see the same stored bits.

Generator: counter based.  Element ``i`` of tensor ``tensor_id`` under ``seed``
depends only on ``(seed, tensor_id, i)``, so any slice of any tensor can be
regenerated on its own (the full-size parity tests regenerate single experts)
and generation can be split over threads without changing a bit.

  pair p = i >> 1 :  z = mix64(key(seed, tensor_id) + p)          (splitmix64 finaliser)
                     u1 = (top 24 bits + 1) / 2^24  in (0, 1]
                     u2 = (low 24 bits) / 2^24      in [0, 1)
                     r  = sqrt(-2 ln u1)
  element 2p   = r cos(2 pi u2),  element 2p+1 = r sin(2 pi u2)     (Box-Muller, fp32)

Shapes and distributions follow the workloads the paper runs (Section 4.1:
Mixtral-8x7B, top-2 of 8 experts, 32 layers, batch-1 decoding) with the value
distributions of the benchmark configurations: weights N(0, 0.02^2),
activations N(0, 1), optional router bias N(0, 1).
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, replace

import numpy as np

_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_GOLD = np.uint64(0x9E3779B97F4A7C15)
_CHUNK = 1 << 20  # pairs per work item


def _mix64(z: np.ndarray) -> np.ndarray:
    z = z.copy()
    z ^= z >> np.uint64(30)
    z *= _M1
    z ^= z >> np.uint64(27)
    z *= _M2
    z ^= z >> np.uint64(31)
    return z


def _key(seed: int, tensor_id: int) -> np.uint64:
    with np.errstate(over="ignore"):
        k = _mix64(np.array([np.uint64(seed & 0xFFFFFFFFFFFFFFFF)]) * _GOLD + np.uint64(1))
        k = _mix64(k + np.uint64(tensor_id & 0xFFFFFFFFFFFFFFFF) * _M2)
    return k[0]


def _pairs(key: np.uint64, p0: int, p1: int, out: np.ndarray) -> None:
    """Fill out[0 : 2*(p1-p0)] with the standard normals of pairs p0..p1-1."""
    with np.errstate(over="ignore"):
        z = _mix64((np.arange(p0, p1, dtype=np.uint64) + key) * _GOLD)
    u1 = ((z >> np.uint64(40)).astype(np.float32) + np.float32(1.0)) * np.float32(2.0 ** -24)
    u2 = (z & np.uint64(0xFFFFFF)).astype(np.float32) * np.float32(2.0 ** -24)
    r = np.sqrt(np.float32(-2.0) * np.log(u1))
    a = np.float32(2.0 * np.pi) * u2
    out[0::2] = r * np.cos(a)
    out[1::2] = r * np.sin(a)


def default_threads() -> int:
    try:
        n = len(os.sched_getaffinity(0))
    except AttributeError:  # pragma: no cover
        n = os.cpu_count() or 1
    env = os.environ.get("OMP_NUM_THREADS")
    if env and env.isdigit():
        n = min(n, int(env)) if int(env) > 0 else n
    return max(1, min(n, 16))


def normal(seed: int, tensor_id: int, n: int, std: float = 1.0, offset: int = 0,
           out: np.ndarray | None = None, threads: int | None = None) -> np.ndarray:
    """fp32 array of elements offset .. offset+n-1 of N(0, std^2) tensor `tensor_id`."""
    if out is None:
        out = np.empty(n, dtype=np.float32)
    assert out.dtype == np.float32 and out.shape == (n,) and out.flags.c_contiguous
    if n == 0:
        return out
    key = _key(seed, tensor_id)
    lo, hi = offset, offset + n
    p_lo, p_hi = lo >> 1, (hi + 1) >> 1
    std32 = np.float32(std)

    def work(p0: int, p1: int) -> None:
        buf = np.empty(2 * (p1 - p0), dtype=np.float32)
        _pairs(key, p0, p1, buf)
        if std32 != np.float32(1.0):
            buf *= std32
        e0, e1 = max(2 * p0, lo), min(2 * p1, hi)
        out[e0 - lo:e1 - lo] = buf[e0 - 2 * p0:e1 - 2 * p0]

    items = [(p, min(p + _CHUNK, p_hi)) for p in range(p_lo, p_hi, _CHUNK)]
    nthr = threads if threads is not None else default_threads()
    if nthr <= 1 or len(items) == 1:
        for p0, p1 in items:
            work(p0, p1)
    else:
        with ThreadPoolExecutor(max_workers=nthr) as ex:
            list(ex.map(lambda it: work(*it), items))
    return out


# --------------------------------------------------------------------------
# bf16 storage (bit patterns in uint16).  Storage-format conversion only.
# --------------------------------------------------------------------------
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16 bit patterns (finite inputs)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    bias = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def store(a_f32: np.ndarray, dtype: str) -> np.ndarray:
    """fp32 values -> the stored representation of `dtype` ('f32' | 'bf16')."""
    if dtype == "f32":
        return np.ascontiguousarray(a_f32, dtype=np.float32)
    if dtype == "bf16":
        return f32_to_bf16_bits(a_f32)
    raise ValueError(dtype)


def itemsize(dtype: str) -> int:
    return {"f32": 4, "bf16": 2}[dtype]


# --------------------------------------------------------------------------
# Workload descriptions
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class MoEConfig:
    """Shape of one synthetic workload (names follow the paper: L layers, top-k)."""
    name: str
    hidden: int          # H
    ffn: int             # F
    n_experts: int       # E
    top_k: int           # k
    n_layers: int = 1    # L
    n_slots: int = 0     # S; 0 = all experts resident in HBM
    dtype: str = "bf16"  # 'f32' | 'bf16'
    n_tokens: int = 1    # T
    glue: int = 0        # 1: x <- rmsnorm(x + y) between stacked layers
    router_bias: bool = False
    seed: int = 0
    w_std: float = 0.02

    @property
    def expert_elems(self) -> int:
        return 3 * self.hidden * self.ffn

    @property
    def expert_bytes(self) -> int:
        return self.expert_elems * itemsize(self.dtype)

    def small(self, **kw) -> "MoEConfig":
        return replace(self, **kw)


# The five benchmark configurations (order as in the benchmark description).
CONFIGS = {
    1: MoEConfig("cfg1-f32-h512", 512, 1024, 8, 2, dtype="f32", n_tokens=16),
    2: MoEConfig("cfg2-mixtral-layer-resident", 4096, 14336, 8, 2, dtype="bf16", n_tokens=256),
    3: MoEConfig("cfg3-mixtral-32L-cacheless", 4096, 14336, 8, 2, n_layers=32, n_slots=4,
                 dtype="bf16", n_tokens=128, glue=1),
    4: MoEConfig("cfg4-mixtral-prefill-512", 4096, 14336, 8, 2, dtype="bf16", n_tokens=512,
                 router_bias=True),
    5: MoEConfig("cfg5-finegrained-24L-cacheless", 2048, 1408, 64, 6, n_layers=24, n_slots=12,
                 dtype="bf16", n_tokens=128, glue=1),
}

# tensor-id scheme: kind in the low bits, then expert, then layer
_KIND_X, _KIND_ROUTER, _KIND_BIAS, _KIND_EXPERT = 0, 1, 2, 3


def _tid(kind: int, layer: int = 0, expert: int = 0) -> int:
    return (layer << 24) | (expert << 4) | kind


def tokens(cfg: MoEConfig, n: int | None = None, first: int = 0) -> np.ndarray:
    """Stored activations x[T, H] ~ N(0, 1) (tokens first .. first+n-1)."""
    n = cfg.n_tokens if n is None else n
    a = normal(cfg.seed, _tid(_KIND_X), n * cfg.hidden, 1.0, offset=first * cfg.hidden)
    return store(a, cfg.dtype).reshape(n, cfg.hidden)


def router_weight(cfg: MoEConfig, layer: int = 0) -> np.ndarray:
    """Stored router matrix Wg[E, H] ~ N(0, w_std^2)."""
    a = normal(cfg.seed, _tid(_KIND_ROUTER, layer), cfg.n_experts * cfg.hidden, cfg.w_std)
    return store(a, cfg.dtype).reshape(cfg.n_experts, cfg.hidden)


def router_bias(cfg: MoEConfig, layer: int = 0) -> np.ndarray | None:
    """fp32 router bias b[E] ~ N(0, 1) for the skewed prefill workload, else None."""
    if not cfg.router_bias:
        return None
    return normal(cfg.seed, _tid(_KIND_BIAS, layer), cfg.n_experts, 1.0)


def expert_weights(cfg: MoEConfig, layer: int, expert: int, out: np.ndarray | None = None,
                   threads: int | None = None) -> np.ndarray:
    """One expert as a flat stored buffer  W1[F,H] | W3[F,H] | W2[H,F]  ~ N(0, w_std^2).

    `out` may be a preallocated flat array of the stored dtype (for example a
    view of pinned host memory) and is filled in place.
    """
    n = cfg.expert_elems
    a = normal(cfg.seed, _tid(_KIND_EXPERT, layer, expert), n, cfg.w_std, threads=threads)
    s = store(a, cfg.dtype)
    if out is not None:
        assert out.shape == (n,) and out.dtype == s.dtype
        out[:] = s
        return out
    return s


def split_expert(cfg: MoEConfig, flat: np.ndarray):
    """Views (W1[F,H], W3[F,H], W2[H,F]) into a flat expert buffer."""
    hf = cfg.hidden * cfg.ffn
    return (flat[:hf].reshape(cfg.ffn, cfg.hidden),
            flat[hf:2 * hf].reshape(cfg.ffn, cfg.hidden),
            flat[2 * hf:].reshape(cfg.hidden, cfg.ffn))


def layer_weights(cfg: MoEConfig, layer: int = 0):
    """(Wg, b, [expert flat buffers]) of one layer."""
    return (router_weight(cfg, layer), router_bias(cfg, layer),
            [expert_weights(cfg, layer, e) for e in range(cfg.n_experts)])
