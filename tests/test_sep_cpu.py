"""Quantisers of the shadow-model emulation: oracle pins, and product == oracle bit for bit (CPU)."""
import numpy as np
import pytest

from oracle import moe_oracle as O
from oracle import sep_oracle as S
from paper_2512_03927_amd import shadow, synth

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


@pytest.mark.parametrize("kind", ["bf16", "int8", "int4"])
def test_product_quantiser_equals_oracle_bit_for_bit(kind):
    W = synth.normal(1, 3, 48 * 128, 0.02).reshape(48, 128)
    W[5] = 0
    got = shadow.quantize_dequantize(W, kind)
    want = S.shadow_matrix(W.astype(np.float64), kind)
    assert np.array_equal(got, want)


def test_shadow_layers_keep_layout_and_bf16_copy_is_identical():
    cfg = synth.MoEConfig("t", 64, 128, 4, 2, n_layers=2, dtype="bf16")
    layers = [synth.layer_weights(cfg, l) for l in range(2)]
    same = shadow.shadow_layers(cfg, layers, "bf16")
    for (a, _, ea), (b, _, eb) in zip(layers, same):
        assert np.array_equal(a, b) and all(np.array_equal(x, y) for x, y in zip(ea, eb))
    q8 = shadow.shadow_layers(cfg, layers, "int8")
    assert q8[0][2][1].shape == layers[0][2][1].shape and q8[0][2][1].dtype == np.uint16
    # the int8 copy differs, but by less than half a quantisation step plus one bf16 rounding
    W1 = O.widen(layers[0][2][1])[:64 * 128].reshape(128, 64)
    W1s = O.widen(q8[0][2][1])[:64 * 128].reshape(128, 64)
    step = np.abs(W1).max(axis=1, keepdims=True) / 127
    assert (np.abs(W1 - W1s) <= step / 2 + np.abs(W1) * 2.0 ** -8).all() and not np.array_equal(W1, W1s)


def test_oracle_shadow_routing_recall_decreases_with_coarser_quantisation():
    """On the CPU oracle alone: routing of an int8 / int4 copy against the full stack (aligned,
    one token per trial).  Coarser quantisation cannot be better on average; the identical copy is perfect."""
    cfg = synth.MoEConfig("t", 64, 64, 8, 2, n_layers=4, dtype="f32", n_tokens=24, glue=1, seed=9)
    layers = [synth.layer_weights(cfg, l) for l in range(cfg.n_layers)]
    X = synth.tokens(cfg)
    rec = {}
    for kind in ("bf16", "int8", "int4"):
        sh_layers = shadow.shadow_layers(cfg, layers, kind)
        c = np.zeros((1, cfg.n_tokens, cfg.n_layers))
        for t in range(cfg.n_tokens):
            _, idx_m, _ = O.stack_decode(X[t], layers, cfg.top_k, "f32")
            _, idx_s, _ = O.stack_decode(X[t], sh_layers, cfg.top_k, "f32")
            c[0, t] = [O.correct_predictions(idx_s[l], idx_m[l]) for l in range(cfg.n_layers)]
        rec[kind] = O.recall(c, np.ones((1, cfg.n_tokens)), cfg.top_k)
    assert rec["bf16"] == 1.0
    assert rec["int8"] >= rec["int4"] > cfg.top_k / cfg.n_experts
