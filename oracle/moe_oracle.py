"""CPU oracle for the cacheless MoE decode layer  --  TEST INFRASTRUCTURE ONLY.

Plain NumPy, float64, no blocking / fusion / reordering.  It is the definition
the HIP path is checked against; it shares no code with that path and must
never be imported by the product (only tests, the smoke check and the
benchmark's cpu_baseline leg may call it).

What the paper fixes: on-demand loading and eviction move bytes, they do not
change the mathematics (Section 1: full precision and all expert activations
are kept; Section 4.4: answer quality equals the fully cached model).  So the
oracle is the plain top-k MoE layer the paper points to (Section 3.1: the
gating network is the usual one of MoE models and is not spelled out; top-2
policy; Section 4.1: Mixtral-8x7B, i.e. SwiGLU experts w1/w3/w2 and a softmax
gate renormalised over the k selected experts).  The paper never prints these formulas; the reading
taken here, per step:

  1. logit[e] = b[e] + sum_h Wg[e,h] x[h]        float64, then rounded once to fp32
  2. idx      = the k largest fp32 logits, ordered (logit descending, index ascending)
  3. g_i      = exp(l_i - l_0) / sum_j exp(l_j - l_0)   over the k kept (== softmax over all E,
                renormalised over the kept ones)
  4. FFN_e(x) = W2_e ( silu(W1_e x) * (W3_e x) ),  silu(a) = a / (1 + exp(-a))
  5. y        = sum_{i<k} g_i FFN_{idx_i}(x)     i ascending, no intermediate rounding
  6. stacked layers only (stand-in for the main node's non-expert work between
     layers): y is rounded to the storage dtype, z = x + y,
     x_next = z / sqrt(mean(z^2) + 1e-6), rounded to the storage dtype.

The routing decision (an integer) is taken on fp32 logits on both sides: the
model in the paper is fp32 (Fig. 3 caption) and the kernel rounds its logit to
fp32 before comparing.

Inputs are the *stored* buffers (fp32 arrays, or uint16 arrays holding bf16 bit
patterns); they are widened exactly to float64 here.

Pins (tests/test_oracle_*.py): brute-force subset enumeration, gate sums to 1,
shift invariance, closed-form softmax case, dense all-experts equivalence,
k=E / k=1 / identical experts / x=0 / zero-router special cases, scalar
hand case, SiLU identities, pure-Python triple loops on tiny shapes, expert
relabelling, unit rms after the glue, both glue branches of the stack re-chained by hand, the
layer with a supplied selection against an independent dense sum.  Absolute layer outputs are not printed
anywhere in the paper: beyond those invariants they are parity unpinned.
"""
from __future__ import annotations

import numpy as np

GLUE_EPS = 1e-6


# --------------------------------------------------------------------------
# storage <-> float64
# --------------------------------------------------------------------------
def widen(a: np.ndarray) -> np.ndarray:
    """Stored buffer -> float64, exactly.  uint16 is read as bf16 bit patterns."""
    a = np.asarray(a)
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    if a.dtype in (np.float32, np.float64):
        return a.astype(np.float64, copy=False)   # float64 input is returned as it is (never written to)
    raise TypeError(f"unsupported storage dtype {a.dtype}")


def round_to_storage(v: np.ndarray, dtype: str) -> np.ndarray:
    """float64 -> stored representation ('f32': float32 array, 'bf16': uint16 bits), RNE.

    bf16 is rounded directly from float64 (one rounding): the float64 value is
    compared with the two neighbouring bf16 values, ties go to the even mantissa.
    """
    v = np.asarray(v, dtype=np.float64)
    if dtype == "f32":
        return v.astype(np.float32)
    if dtype != "bf16":
        raise ValueError(dtype)
    # truncate toward zero in the bf16 grid, then decide on the remainder
    f32_trunc = v.astype(np.float32)
    bits = f32_trunc.view(np.uint32)
    # astype may round up past v; step back to the fp32 value with |.| <= |v|
    too_big = np.abs(f32_trunc.astype(np.float64)) > np.abs(v)
    bits = np.where(too_big, bits - np.uint32(1), bits)
    lo_bits = bits & np.uint32(0xFFFF0000)                     # bf16 neighbour toward zero
    hi_bits = lo_bits + np.uint32(0x00010000)                  # next bf16 away from zero
    lo = lo_bits.view(np.float32).astype(np.float64)
    hi = hi_bits.view(np.float32).astype(np.float64)
    d_lo = np.abs(v - lo)
    d_hi = np.abs(hi - v)
    lo_even = ((lo_bits >> np.uint32(16)) & np.uint32(1)) == 0
    pick_hi = (d_hi < d_lo) | ((d_hi == d_lo) & ~lo_even)
    out = np.where(pick_hi, hi_bits, lo_bits)
    return (out >> np.uint32(16)).astype(np.uint16)


# --------------------------------------------------------------------------
# step 1-3: router and gate
# --------------------------------------------------------------------------
def router_logits(Wg, b, x) -> np.ndarray:
    """Step 1.  fp32 logits [E] = round_fp32( b + Wg x ) with a float64 sum."""
    s = widen(Wg) @ widen(x)
    if b is not None:
        s = s + widen(b)
    return s.astype(np.float32)


def topk_select(logits: np.ndarray, k: int) -> np.ndarray:
    """Step 2.  Indices of the k largest logits; order: logit descending, index ascending.

    +0.0 and -0.0 compare equal (a tie).  NaN logits are an error.
    """
    logits = np.asarray(logits)
    E = logits.shape[0]
    if not 1 <= k <= E:
        raise ValueError("need 1 <= k <= E")
    if np.isnan(logits).any():
        raise ValueError("NaN logit")
    order = sorted(range(E), key=lambda e: (-float(logits[e]), e))
    return np.array(order[:k], dtype=np.int32)


def gate_weights(logits: np.ndarray, idx: np.ndarray) -> np.ndarray:
    """Step 3.  Softmax over the kept logits, relative to the largest (idx[0])."""
    l = np.asarray(logits, dtype=np.float64)[idx]
    u = np.exp(l - l[0])
    return u / u.sum()


def route(Wg, b, x, k):
    """Steps 1-3 for one token: (idx int32[k], g float64[k], logits fp32[E])."""
    logits = router_logits(Wg, b, x)
    idx = topk_select(logits, k)
    return idx, gate_weights(logits, idx), logits


def routing_margin_ulps(logits: np.ndarray, k: int) -> float:
    """Smallest gap that fixes the routing result, in fp32 ulps of the larger logit.

    The gaps that matter are those between consecutive entries of the sorted
    top-(k+1) list: inside the top-k they fix the output order, the last one
    fixes membership.  0 means an exact tie (resolved by index).
    """
    l = np.sort(np.asarray(logits, dtype=np.float32).astype(np.float64))[::-1]
    top = l[:min(k + 1, l.shape[0])]
    if top.shape[0] < 2:
        return float("inf")
    gaps = top[:-1] - top[1:]
    ulp = np.spacing(np.maximum(np.abs(top[:-1]), np.abs(top[1:])).astype(np.float32)).astype(np.float64)
    return float(np.min(gaps / ulp))


# --------------------------------------------------------------------------
# step 4-5: experts and combine
# --------------------------------------------------------------------------
def silu(a: np.ndarray) -> np.ndarray:
    return a / (1.0 + np.exp(-a))


def expert_hidden(W1, W3, x) -> np.ndarray:
    """h = silu(W1 x) * (W3 x), float64 [F]."""
    xv = widen(x)
    return silu(widen(W1) @ xv) * (widen(W3) @ xv)


def expert_ffn(W1, W3, W2, x) -> np.ndarray:
    """Step 4.  FFN_e(x) in float64 [H]."""
    return widen(W2) @ expert_hidden(W1, W3, x)


def split_expert(flat: np.ndarray, H: int, F: int):
    """(W1[F,H], W3[F,H], W2[H,F]) views of a flat expert buffer W1|W3|W2."""
    hf = H * F
    return (flat[:hf].reshape(F, H), flat[hf:2 * hf].reshape(F, H), flat[2 * hf:3 * hf].reshape(H, F))


def moe_layer(x, Wg, b, experts, k: int):
    """Steps 1-5 for one token.

    experts: sequence of E flat buffers (W1|W3|W2) or of (W1, W3, W2) tuples.
    Returns (y float64[H], idx int32[k], g float64[k]).
    """
    H = np.asarray(x).shape[0]
    idx, g, _ = route(Wg, b, x, k)
    y = np.zeros(H, dtype=np.float64)
    for i in range(k):
        ew = experts[int(idx[i])]
        if not isinstance(ew, tuple):
            F = np.asarray(ew).shape[0] // (3 * H)
            ew = split_expert(np.asarray(ew), H, F)
        y = y + g[i] * expert_ffn(ew[0], ew[1], ew[2], x)
    return y, idx, g


def moe_layer_given_idx(x, Wg, b, experts, idx):
    """Steps 1 and 3-5 for one token with the selection (step 2) supplied by the caller.

    idx: the experts to use, in output order (idx[0] is the reference of the gate's exponent).
    Used by tests to continue a stacked comparison past a layer where two logits tie to within
    rounding and the kernel's own input made the other, equally valid, choice.  With
    idx = topk_select(router_logits(...)) it is moe_layer.  Returns (y float64[H], g float64[k]).
    """
    H = np.asarray(x).shape[0]
    idx = np.asarray(idx, dtype=np.int32)
    g = gate_weights(router_logits(Wg, b, x), idx)
    y = np.zeros(H, dtype=np.float64)
    for i in range(idx.shape[0]):
        ew = experts[int(idx[i])]
        if not isinstance(ew, tuple):
            F = np.asarray(ew).shape[0] // (3 * H)
            ew = split_expert(np.asarray(ew), H, F)
        y = y + g[i] * expert_ffn(ew[0], ew[1], ew[2], x)
    return y, g


def moe_layer_tokens(X, Wg, b, experts, k: int):
    """The layer applied to each row of X[T,H] independently (decode tokens or a prefill batch)."""
    X = np.asarray(X)
    T, H = X.shape
    Y = np.zeros((T, H), dtype=np.float64)
    IDX = np.zeros((T, k), dtype=np.int32)
    G = np.zeros((T, k), dtype=np.float64)
    for t in range(T):
        Y[t], IDX[t], G[t] = moe_layer(X[t], Wg, b, experts, k)
    return Y, IDX, G


# --------------------------------------------------------------------------
# step 6: stack glue and the stacked decode
# --------------------------------------------------------------------------
def glue_rmsnorm(x, y) -> np.ndarray:
    """z = x + y ; z / sqrt(mean(z^2) + eps), float64.  x, y are stored buffers or float64."""
    z = widen(x) + widen(y)
    return z / np.sqrt(np.mean(z * z) + GLUE_EPS)


def stack_decode(x, layers, k: int, dtype: str, glue: int = 1):
    """One token through L stacked layers.

    layers: sequence of (Wg, b, experts).  Returns (x_out stored [H], idx int32[L,k],
    xs: list of the stored input of every layer followed by the final state).
    glue=1: x <- store(rmsnorm(x + store(y))); glue=0: x <- store(y).
    """
    x = np.asarray(x)
    L = len(layers)
    IDX = np.zeros((L, k), dtype=np.int32)
    xs = [x]
    for l, (Wg, b, experts) in enumerate(layers):
        y, IDX[l], _ = moe_layer(x, Wg, b, experts, k)
        y_st = round_to_storage(y, dtype)
        x = round_to_storage(glue_rmsnorm(x, y_st), dtype) if glue else y_st
        xs.append(x)
    return x, IDX, xs


# --------------------------------------------------------------------------
# bookkeeping the paper states in prose / equations
# --------------------------------------------------------------------------
def expert_bytes(H: int, F: int, bytes_per_param: int) -> int:
    """Bytes of one SwiGLU expert (w1, w3: F x H; w2: H x F)."""
    return 3 * H * F * bytes_per_param


def embedding_bytes(H: int, bytes_per_param: int) -> int:
    """Bytes of one token's embedding as exchanged per layer (Section 4.2: about 16 KB)."""
    return H * bytes_per_param


def cacheless_loads_per_token(L: int, k: int) -> int:
    """No expert survives its use (Sections 1, 2), so every activation is a load."""
    return L * k


def recall(c: np.ndarray, A: np.ndarray, k: int) -> float:
    """Overall recall (Section 3.2, second recall equation).

    c[q, n, l] = number of correctly predicted experts, A[q, n] in {0,1} = token exists.
    """
    c = np.asarray(c, dtype=np.float64)
    A = np.asarray(A, dtype=np.float64)
    L = c.shape[2]
    return float((c * A[:, :, None]).sum() / (k * L * A.sum()))


def recall_per_token(c: np.ndarray, A: np.ndarray, k: int) -> np.ndarray:
    """recall(n) for every output-token index n (Section 3.2, first recall equation)."""
    c = np.asarray(c, dtype=np.float64)
    A = np.asarray(A, dtype=np.float64)
    L = c.shape[2]
    return (c * A[:, :, None]).sum(axis=(0, 2)) / (k * L * A.sum(axis=0))


def correct_predictions(pred_idx: np.ndarray, true_idx: np.ndarray) -> int:
    """|predicted set  intersect  activated set| for one token-layer."""
    return len(set(int(v) for v in pred_idx) & set(int(v) for v in true_idx))


def t_maxload(n_groups: int, t_M: float, t_W: float) -> float:
    """Longest expert load that causes no stall (Section 3.1, load-window equation).

    The printed equation uses G (group size, 2) but its worked example for the
    four-group testbed gives 4 t^M + 3 t^W, which only fits with G read as the
    number of groups; that reading is taken.
    """
    return n_groups * t_M + (n_groups - 1) * t_W
