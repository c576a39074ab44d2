"""Quantisers of the shadow-model emulation: pins of oracle/sep_oracle.py (CPU).  The product's
quantiser runs on the GPU and is compared with this oracle bit for bit in tests/test_gpu_sep.py."""
import numpy as np
import pytest

from oracle import moe_oracle as O
from oracle import sep_oracle as S
from paper_2512_03927_amd import synth

rng = np.random.default_rng(5)


def test_int8_rows_error_bound_grid_exactness_idempotence():
    W = rng.normal(0, 0.02, size=(7, 96))
    W[3] = 0.0                                            # an all-zero row stays zero, scale 0
    q, s = S.quantize_rows_int8(W)
    assert q.dtype == np.int8 and s.shape == (7,) and s[3] == 0 and (q[3] == 0).all()
    Wd = S.dequantize_rows(q, s)
    assert (np.abs(W - Wd) <= s[:, None] / 2 + 1e-18).all()
    assert np.abs(q).max() == 127                        # the largest element of a row maps to +-127
    for r in (0, 1, 2, 4):
        assert abs(Wd[r, np.argmax(np.abs(W[r]))]) == pytest.approx(np.abs(W[r]).max(), rel=1e-15)
    q2, s2 = S.quantize_rows_int8(Wd)                    # idempotent
    assert np.array_equal(q2, q) and np.allclose(s2, s, rtol=1e-15)
    qn, sn = S.quantize_rows_int8(-W)                    # odd symmetry
    assert np.array_equal(qn, -q) and np.array_equal(sn, s)


def test_int8_hand_worked_row_and_half_to_even():
    # scale = 127/127 = 1: values on .5 round to the even neighbour
    W = np.array([[127.0, 0.5, 1.5, 2.5, -0.5, -1.5, 63.49, -126.51]])
    q, s = S.quantize_rows_int8(W)
    assert s[0] == 1.0
    assert q[0].tolist() == [127, 0, 2, 2, 0, -2, 63, -127]


def test_int4_groups():
    W = rng.normal(0, 1.0, size=(3, 128))
    q, s = S.quantize_groups_int4(W, 64)
    assert s.shape == (3, 2) and np.abs(q).max() == 7 and np.abs(q).max(axis=1).min() == 7
    Wd = S.dequantize_groups(q, s, 64)
    assert (np.abs(W - Wd).reshape(3, 2, 64) <= s[:, :, None] / 2 + 1e-15).all()
    q2, _ = S.quantize_groups_int4(Wd, 64)
    assert np.array_equal(q2, q)
    with pytest.raises(ValueError):
        S.quantize_groups_int4(np.zeros((2, 100)), 64)
    # a hand-worked group: scale 7/7 = 1
    g = np.zeros((1, 64)); g[0, :5] = [7.0, -3.5, 2.5, 0.49, -6.51]
    q, s = S.quantize_groups_int4(g, 64)
    assert s[0, 0] == 1.0 and q[0, :5].tolist() == [7, -4, 2, 0, -7]


def test_fp16_rounding_hand_worked_values():
    """Binary16: 10 fraction bits, ties to even, subnormals of 2^-24, largest finite value 65504."""
    cases = [
        (1.0, 0x3C00, 1.0),
        (1.0 + 2.0 ** -11, 0x3C00, 1.0),                       # halfway between 1 and 1 + 2^-10: even fraction
        (1.0 + 3 * 2.0 ** -11, 0x3C02, 1.0 + 2.0 ** -9),       # halfway between fractions 1 and 2: even is 2
        (1.0 + 2.0 ** -11 + 2.0 ** -30, 0x3C01, 1.0 + 2.0 ** -10),   # just above a midpoint rounds up
        (1.0 / 3.0, 0x3555, 0.333251953125),
        (-0.02, 0xA51F, -0.0200042724609375),
        (2.0 ** -24, 0x0001, 2.0 ** -24),                      # smallest subnormal
        (2.0 ** -25, 0x0000, 0.0),                             # halfway to it: ties to even (zero)
        (3 * 2.0 ** -25, 0x0002, 2.0 ** -23),                  # halfway between subnormals 1 and 2: even
        (65504.0, 0x7BFF, 65504.0),
        (1e6, 0x7BFF, 65504.0), (-1e6, 0xFBFF, -65504.0),      # clipped, never infinite
        (0.0, 0x0000, 0.0),
    ]
    W = np.array([[c[0] for c in cases]])
    bits, vals = S.round_fp16(W)
    assert bits.dtype == np.uint16
    for j, (_, b, v) in enumerate(cases):
        assert bits[0, j] == b and vals[0, j] == v, (j, hex(bits[0, j]), vals[0, j])
    # relative error bound of a normal value: half a unit in the last place, 2^-11
    X = rng.normal(0, 0.02, size=4096)
    X = X[np.abs(X) > 2.0 ** -14]
    assert (np.abs(S.round_fp16(X)[1] - X) <= np.abs(X) * 2.0 ** -11).all()
    assert np.array_equal(S.round_fp16(S.round_fp16(X)[1])[1], S.round_fp16(X)[1])    # idempotent
    assert np.array_equal(S.round_fp16(-X)[1], -S.round_fp16(X)[1])                   # odd


def test_shadow_matrix_kinds():
    W = synth.normal(1, 3, 48 * 128, 0.02).reshape(48, 128).astype(np.float64)
    W[5] = 0
    assert np.array_equal(S.shadow_matrix(W, "bf16"), W)
    assert np.array_equal(S.shadow_matrix(W, "fp16"), S.round_fp16(W)[1])
    q, sc = S.quantize_rows_int8(W)
    assert np.array_equal(S.shadow_matrix(W, "int8"), q.astype(np.float64) * sc[:, None])
    q4, s4 = S.quantize_groups_int4(W)
    assert np.array_equal(S.shadow_matrix(W, "int4"), S.dequantize_groups(q4, s4))
    step = np.abs(W).max(axis=1, keepdims=True) / 127
    assert (np.abs(W - S.shadow_matrix(W, "int8")) <= step / 2 + 1e-18).all()
    with pytest.raises(ValueError):
        S.shadow_matrix(W, "int3")


def _oracle_shadow_layers(cfg, layers, kind):
    """Shadow copy of a stack through the oracle's quantisers, stored back in cfg's dtype."""
    out = []
    for (Wg, b, experts) in layers:
        ex = []
        for flat in experts:
            parts = [S.shadow_matrix(O.widen(W), kind) for W in O.split_expert(flat, cfg.hidden, cfg.ffn)]
            ex.append(O.round_to_storage(np.concatenate([p.ravel() for p in parts]), cfg.dtype))
        out.append((O.round_to_storage(S.shadow_matrix(O.widen(Wg), kind), cfg.dtype), b, ex))
    return out


def test_oracle_shadow_routing_recall_decreases_with_coarser_quantisation():
    """On the CPU oracle alone: routing of an int8 / int4 copy against the full stack (aligned,
    one token per trial).  Coarser quantisation cannot be better on average; the identical copy is perfect."""
    cfg = synth.MoEConfig("t", 64, 64, 8, 2, n_layers=4, dtype="f32", n_tokens=24, glue=1, seed=9)
    layers = [synth.layer_weights(cfg, l) for l in range(cfg.n_layers)]
    X = synth.tokens(cfg)
    rec = {}
    for kind in ("bf16", "fp16", "int8", "int4"):
        sh_layers = _oracle_shadow_layers(cfg, layers, kind)
        c = np.zeros((1, cfg.n_tokens, cfg.n_layers))
        for t in range(cfg.n_tokens):
            _, idx_m, _ = O.stack_decode(X[t], layers, cfg.top_k, "f32")
            _, idx_s, _ = O.stack_decode(X[t], sh_layers, cfg.top_k, "f32")
            c[0, t] = [O.correct_predictions(idx_s[l], idx_m[l]) for l in range(cfg.n_layers)]
        rec[kind] = O.recall(c, np.ones((1, cfg.n_tokens)), cfg.top_k)
    assert rec["bf16"] == 1.0
    assert rec["fp16"] >= rec["int8"] >= rec["int4"] > cfg.top_k / cfg.n_experts
