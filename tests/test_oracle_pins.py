"""Pins for the CPU oracle: things the paper and the mathematics fix.

Each test is chosen so that one plausible mistake in oracle/moe_oracle.py (a
dropped term, a wrong sign or index, a transposed operand, a swapped matrix)
fails it.  None of them calls the HIP path.
"""
import itertools
import json
import math
import os

import numpy as np
import pytest
import scipy.special

from oracle import moe_oracle as O

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_facts.json")))
rng = np.random.default_rng(1234)


def _rand_layer(H, F, E, seed=0, std=0.5):
    r = np.random.default_rng(seed)
    Wg = r.normal(0, std, (E, H))
    experts = [(r.normal(0, std, (F, H)), r.normal(0, std, (F, H)), r.normal(0, std, (H, F)))
               for _ in range(E)]
    return Wg, experts


# ------------------------------------------------------------------ top-k
@pytest.mark.parametrize("E,k", [(3, 1), (4, 2), (5, 3), (8, 2), (8, 3), (6, 6)])
def test_topk_matches_brute_force_subsets(E, k):
    """The chosen set maximises the logit sum; among maximisers it is the
    lexicographically smallest index tuple (lowest index wins ties)."""
    r = np.random.default_rng(E * 100 + k)
    for trial in range(60):
        # small integer logits: ties are frequent
        logits = r.integers(-2, 3, size=E).astype(np.float32)
        if trial % 3 == 0:
            logits = r.normal(size=E).astype(np.float32)
        best = None
        for sub in itertools.combinations(range(E), k):
            s = float(sum(float(logits[e]) for e in sub))
            key = (-s, sub)
            if best is None or key < best:
                best = key
        idx = O.topk_select(logits, k)
        assert tuple(sorted(int(i) for i in idx)) == best[1]
        # order inside the result: logit descending, equal logits by index ascending
        for a, b in zip(idx[:-1], idx[1:]):
            assert (logits[a] > logits[b]) or (logits[a] == logits[b] and a < b)


def test_topk_signed_zero_is_a_tie_and_nan_is_an_error():
    assert list(O.topk_select(np.array([-0.0, 0.0, -1.0], np.float32), 2)) == [0, 1]
    assert list(O.topk_select(np.array([0.0, -0.0, -1.0], np.float32), 1)) == [0]
    with pytest.raises(ValueError):
        O.topk_select(np.array([0.0, np.nan], np.float32), 1)
    with pytest.raises(ValueError):
        O.topk_select(np.zeros(4, np.float32), 5)


def test_duplicated_router_rows_tie_break_lowest_index():
    H, E, k = 16, 6, 3
    r = np.random.default_rng(7)
    Wg = r.normal(size=(E, H)).astype(np.float32)
    Wg[4] = Wg[1]          # rows 1 and 4 give bit-identical logits
    Wg[5] = Wg[1]
    for _ in range(20):
        x = r.normal(size=H).astype(np.float32)
        idx, g, logits = O.route(Wg, None, x, k)
        assert logits[1] == logits[4] == logits[5]
        pos = {int(e): i for i, e in enumerate(idx)}
        for lo, hi in ((1, 4), (4, 5), (1, 5)):
            if hi in pos:
                assert lo in pos and pos[lo] < pos[hi]


def test_zero_router_gives_first_k_and_uniform_gate():
    H, E, k = 8, 8, 2
    idx, g, _ = O.route(np.zeros((E, H), np.float32), None, rng.normal(size=H).astype(np.float32), k)
    assert list(idx) == [0, 1]
    assert np.allclose(g, 0.5, atol=0, rtol=0)


# ------------------------------------------------------------------ gate
def test_gate_closed_form_ln_case():
    """logits (0, ln 2, ln 3): softmax = (1/6, 2/6, 3/6); top-2 = experts (2, 1), g = (3/5, 2/5)."""
    logits = np.array([0.0, math.log(2.0), math.log(3.0)], dtype=np.float32)
    idx = O.topk_select(logits, 2)
    assert list(idx) == [2, 1]
    g = O.gate_weights(logits, idx)
    assert np.allclose(g, [0.6, 0.4], atol=1e-7)


def test_gate_sums_to_one_shift_invariant_and_equals_renormalised_full_softmax():
    for E, k in [(8, 2), (64, 6), (5, 5), (9, 1)]:
        for _ in range(25):
            logits = rng.normal(0, 3, size=E).astype(np.float32)
            idx = O.topk_select(logits, k)
            g = O.gate_weights(logits, idx)
            assert abs(g.sum() - 1.0) < 1e-12
            assert (g > 0).all() and (np.diff(g) <= 0).all()
            # library softmax over all E experts, renormalised on the kept ones
            p = scipy.special.softmax(logits.astype(np.float64))
            assert np.allclose(g, p[idx] / p[idx].sum(), rtol=1e-12)
            # shift by a power of two keeps fp32 differences exact
            shifted = (logits.astype(np.float64) + 4.0)
            idx2 = O.topk_select(shifted, k)
            assert list(idx2) == list(idx)
            assert np.allclose(O.gate_weights(shifted, idx2), g, rtol=1e-9)


def test_k_equals_E_is_full_softmax_and_k1_is_argmax_with_unit_gate():
    logits = rng.normal(size=7).astype(np.float32)
    idx = O.topk_select(logits, 7)
    g = O.gate_weights(logits, idx)
    full = scipy.special.softmax(logits.astype(np.float64))
    assert np.allclose(g, full[idx], rtol=1e-12)
    idx1 = O.topk_select(logits, 1)
    assert int(idx1[0]) == int(np.argmax(logits))
    assert O.gate_weights(logits, idx1)[0] == 1.0


# ------------------------------------------------------------------ SiLU / FFN
def test_silu_identities():
    assert O.silu(np.array([0.0]))[0] == 0.0
    assert math.isclose(O.silu(np.array([math.log(3.0)]))[0], 0.75 * math.log(3.0), rel_tol=1e-15)
    a = rng.normal(0, 3, size=100)
    assert np.allclose(O.silu(-a), O.silu(a) - a, atol=1e-14)      # silu(-a) = silu(a) - a
    assert np.allclose(O.silu(a), a * scipy.special.expit(a), rtol=1e-13)


def test_ffn_scalar_hand_case_distinguishes_w1_from_w3():
    """H = F = 1: y = w2 * silu(w1 x) * (w3 x).  x=1, w1=ln 3, w3=2, w2=5 -> 5 * (3/4 ln 3) * 2."""
    y = O.expert_ffn(np.array([[math.log(3.0)]]), np.array([[2.0]]), np.array([[5.0]]), np.array([1.0]))
    assert math.isclose(y[0], 7.5 * math.log(3.0), rel_tol=1e-15)
    y0 = O.expert_ffn(np.zeros((3, 2)), rng.normal(size=(3, 2)), rng.normal(size=(2, 3)), rng.normal(size=2))
    assert (y0 == 0).all()                                           # W1 = 0 -> silu(0) = 0


def test_ffn_and_router_against_pure_python_loops():
    """Independent triple loops on tiny non-square shapes (a transposed operand cannot pass)."""
    H, F, E = 3, 5, 4
    r = np.random.default_rng(5)
    W1, W3, W2 = r.normal(size=(F, H)), r.normal(size=(F, H)), r.normal(size=(H, F))
    x = r.normal(size=H)
    h = []
    for j in range(F):
        a = sum(W1[j][c] * x[c] for c in range(H))
        b = sum(W3[j][c] * x[c] for c in range(H))
        h.append(a / (1.0 + math.exp(-a)) * b)
    y = [sum(W2[i][j] * h[j] for j in range(F)) for i in range(H)]
    assert np.allclose(O.expert_ffn(W1, W3, W2, x), y, rtol=1e-13)
    assert np.allclose(O.expert_hidden(W1, W3, x), h, rtol=1e-13)
    Wg, b = r.normal(size=(E, H)), r.normal(size=E).astype(np.float32)
    ref = [np.float32(float(b[e]) + sum(Wg[e][c] * x[c] for c in range(H))) for e in range(E)]
    assert np.array_equal(O.router_logits(Wg, b, x), np.array(ref, np.float32))
    assert np.array_equal(O.router_logits(Wg, None, x),
                          np.array([np.float32(sum(Wg[e][c] * x[c] for c in range(H))) for e in range(E)]))


def test_split_expert_layout_is_w1_w3_w2():
    H, F = 2, 3
    flat = np.arange(3 * H * F, dtype=np.float32)
    W1, W3, W2 = O.split_expert(flat, H, F)
    assert W1.shape == (F, H) and W3.shape == (F, H) and W2.shape == (H, F)
    assert W1[0, 0] == 0 and W1[1, 0] == H and W3[0, 0] == H * F and W2[0, 0] == 2 * H * F
    assert W2[1, 0] == 2 * H * F + F


# ------------------------------------------------------------------ whole layer
def _dense_layer(x, Wg, b, experts, k):
    """All E experts with the gate zeroed outside the selected set."""
    logits = O.router_logits(Wg, b, x).astype(np.float64)
    p = scipy.special.softmax(logits)
    keep = np.zeros_like(p)
    order = np.lexsort((np.arange(len(p)), -logits))[:k]
    keep[order] = p[order]
    keep /= keep.sum()
    return sum(keep[e] * O.expert_ffn(*experts[e], x) for e in range(len(experts)))


@pytest.mark.parametrize("H,F,E,k", [(8, 12, 4, 2), (6, 10, 8, 3), (5, 7, 3, 1), (4, 6, 5, 5)])
def test_sparse_layer_equals_dense_all_experts_with_zeroed_gates(H, F, E, k):
    Wg, experts = _rand_layer(H, F, E, seed=H + F)
    b = np.random.default_rng(3).normal(size=E).astype(np.float32)
    for t in range(8):
        x = np.random.default_rng(t).normal(size=H)
        y, idx, g = O.moe_layer(x, Wg, b, experts, k)
        assert np.allclose(y, _dense_layer(x, Wg, b, experts, k), rtol=1e-12, atol=1e-13)
        assert abs(g.sum() - 1) < 1e-12


def test_layer_special_cases():
    H, F, E, k = 6, 9, 5, 2
    Wg, experts = _rand_layer(H, F, E, seed=11)
    x = np.random.default_rng(2).normal(size=H)
    # identical experts: y = FFN(x) whatever the routing (gates sum to 1)
    same = [experts[0]] * E
    y, _, _ = O.moe_layer(x, Wg, None, same, k)
    assert np.allclose(y, O.expert_ffn(*experts[0], x), rtol=1e-12)
    # k = 1: y = FFN_argmax(x) exactly
    y1, idx1, g1 = O.moe_layer(x, Wg, None, experts, 1)
    assert g1[0] == 1.0
    assert np.array_equal(y1, O.expert_ffn(*experts[int(np.argmax(O.router_logits(Wg, None, x)))], x))
    # x = 0 -> y = 0
    y0, idx0, g0 = O.moe_layer(np.zeros(H), Wg, None, experts, k)
    assert (y0 == 0).all() and list(idx0) == [0, 1]
    # relabelling experts permutes idx and leaves y (no ties here)
    perm = np.array([3, 0, 4, 1, 2])                         # new position p holds old expert perm[p]
    y_a, idx_a, g_a = O.moe_layer(x, Wg, None, experts, k)
    y_b, idx_b, g_b = O.moe_layer(x, Wg[perm], None, [experts[p] for p in perm], k)
    assert np.allclose(y_a, y_b, rtol=1e-13)
    assert [int(perm[i]) for i in idx_b] == [int(i) for i in idx_a]
    assert np.allclose(g_a, g_b)


def test_flat_expert_buffers_and_tuple_experts_agree():
    H, F, E, k = 4, 6, 3, 2
    Wg, experts = _rand_layer(H, F, E, seed=21)
    flats = [np.concatenate([w.ravel() for w in ex]) for ex in experts]
    x = np.random.default_rng(8).normal(size=H)
    ya, ia, _ = O.moe_layer(x, Wg, None, experts, k)
    yb, ib, _ = O.moe_layer(x, Wg, None, flats, k)
    assert np.array_equal(ya, yb) and np.array_equal(ia, ib)
    Y, IDX, G = O.moe_layer_tokens(np.stack([x, 2 * x]), Wg, None, flats, k)
    assert np.array_equal(Y[0], ya) and IDX.shape == (2, k)


# ------------------------------------------------------------------ stack glue
def test_glue_has_unit_rms_and_stack_feeds_layers_in_order():
    H, F, E, k, L = 16, 24, 4, 2, 3
    layers = []
    for l in range(L):
        Wg, experts = _rand_layer(H, F, E, seed=100 + l, std=0.3)
        layers.append((Wg.astype(np.float32), None,
                       [tuple(w.astype(np.float32) for w in ex) for ex in experts]))
    x0 = np.random.default_rng(0).normal(size=H).astype(np.float32)
    xo, IDX, xs = O.stack_decode(x0, layers, k, "f32", glue=1)
    assert len(xs) == L + 1 and IDX.shape == (L, k)
    for x in xs[1:]:
        assert abs(np.sqrt(np.mean(O.widen(x) ** 2)) - 1.0) < 1e-3
    # layer l really sees the output of layer l-1: recompute by hand
    x = x0
    for l in range(L):
        y, idx, _ = O.moe_layer(x, *layers[l], k)
        assert np.array_equal(idx, IDX[l])
        z = x.astype(np.float64) + y.astype(np.float32).astype(np.float64)
        x = (z / np.sqrt((z ** 2).mean() + 1e-6)).astype(np.float32)
        assert np.array_equal(x, xs[l + 1])
    z = O.glue_rmsnorm(np.array([3.0, -4.0]), np.array([0.0, 0.0]))
    assert np.allclose(z, np.array([3.0, -4.0]) / math.sqrt(12.5 + 1e-6), rtol=1e-15)


def test_stack_without_glue_chains_the_stored_layer_output():
    """glue = 0: layer l+1 sees store(y_l), nothing else.  Pinned three ways: a scalar stack worked
    by hand, an independent re-chaining on random layers, and bf16 storage rounding between layers."""
    # one expert, H = F = 1: FFN(x) = w2 * silu(w1 x) * (w3 x); two layers chained by hand
    def ffn1(w1, w3, w2, x):
        a = w1 * x
        return w2 * (a / (1.0 + math.exp(-a))) * (w3 * x)
    l0 = (np.array([[0.3]]), None, [(np.array([[1.5]]), np.array([[-0.7]]), np.array([[2.0]]))])
    l1 = (np.array([[0.1]]), None, [(np.array([[0.4]]), np.array([[1.1]]), np.array([[-3.0]]))])
    x0 = np.array([0.8], np.float32)
    y0 = np.float32(ffn1(1.5, -0.7, 2.0, float(x0[0])))                 # stored as fp32 between layers
    y1 = np.float32(ffn1(0.4, 1.1, -3.0, float(y0)))
    xo, IDX, xs = O.stack_decode(x0, [l0, l1], 1, "f32", glue=0)
    assert abs(float(xs[1][0]) - float(y0)) <= 1e-7 * abs(float(y0)) and abs(float(xo[0]) - float(y1)) <= 2e-7 * abs(float(y1))
    assert len(xs) == 3 and np.array_equal(xs[2], xo) and (IDX == 0).all()
    # random layers: re-chain by hand; no residual, no normalisation
    H, F, E, k, L = 12, 20, 5, 2, 3
    layers = []
    for l in range(L):
        Wg, experts = _rand_layer(H, F, E, seed=300 + l, std=0.6)
        layers.append((Wg.astype(np.float32), None, [tuple(w.astype(np.float32) for w in ex) for ex in experts]))
    x0 = np.random.default_rng(5).normal(size=H).astype(np.float32)
    xo, IDX, xs = O.stack_decode(x0, layers, k, "f32", glue=0)
    x = x0
    for l in range(L):
        y, idx, _ = O.moe_layer(x, *layers[l], k)
        assert np.array_equal(idx, IDX[l])
        x = y.astype(np.float32)
        assert np.array_equal(x, xs[l + 1])
    assert np.array_equal(xo, x)
    # the two branches differ (a residual + norm would change the result)
    assert not np.allclose(O.widen(O.stack_decode(x0, layers, k, "f32", glue=1)[0]), O.widen(xo))
    # bf16 storage between layers
    xb = O.round_to_storage(x0.astype(np.float64), "bf16")
    xo_b, _, xs_b = O.stack_decode(xb, layers[:2], k, "bf16", glue=0)
    y, _, _ = O.moe_layer(xb, *layers[0], k)
    assert np.array_equal(xs_b[1], O.round_to_storage(y, "bf16")) and xs_b[1].dtype == np.uint16
    y2, _, _ = O.moe_layer(xs_b[1], *layers[1], k)
    assert np.array_equal(xo_b, O.round_to_storage(y2, "bf16"))


def test_layer_with_supplied_selection():
    """moe_layer_given_idx: with the router's own selection it is moe_layer; with any other
    selection it is the dense sum over all experts with a softmax renormalised on that set (computed
    here with a library softmax and explicit loops), in the order given."""
    H, F, E, k = 7, 9, 6, 3
    Wg, experts = _rand_layer(H, F, E, seed=77)
    b = np.random.default_rng(4).normal(size=E).astype(np.float32)
    for t in range(6):
        x = np.random.default_rng(40 + t).normal(size=H)
        y_ref, idx, g_ref = O.moe_layer(x, Wg, b, experts, k)
        y, g = O.moe_layer_given_idx(x, Wg, b, experts, idx)
        assert np.array_equal(y, y_ref) and np.array_equal(g, g_ref)
        other = np.random.default_rng(t).permutation(E)[:k]
        y2, g2 = O.moe_layer_given_idx(x, Wg, b, experts, other)
        p = scipy.special.softmax(O.router_logits(Wg, b, x).astype(np.float64))
        keep = np.zeros(E)
        keep[other] = p[other]
        keep /= keep.sum()
        dense = np.zeros(H)
        for e in range(E):
            W1, W3, W2 = experts[e]
            h = [sum(W1[j, i] * x[i] for i in range(H)) for j in range(F)]
            u = [sum(W3[j, i] * x[i] for i in range(H)) for j in range(F)]
            hv = [h[j] / (1.0 + math.exp(-h[j])) * u[j] for j in range(F)]
            dense += keep[e] * np.array([sum(W2[r, j] * hv[j] for j in range(F)) for r in range(H)])
        assert np.allclose(y2, dense, rtol=1e-11, atol=1e-13)
        assert np.allclose(g2, keep[other], rtol=1e-12) and abs(g2.sum() - 1) < 1e-12


# ------------------------------------------------------------------ storage rounding
def test_bf16_rounding_matches_library_and_handles_ties_to_even():
    torch = pytest.importorskip("torch")
    a = np.random.default_rng(0).normal(0, 10, size=20000).astype(np.float32)
    a[:6] = [0.0, -0.0, 1.0, -1.0, 3.0e-39, 65504.0]
    want = torch.from_numpy(a).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = O.round_to_storage(a.astype(np.float64), "bf16")
    assert np.array_equal(got, want)
    # exact round trip of every stored value
    assert np.array_equal(O.round_to_storage(O.widen(got), "bf16"), got)
    # midpoints between bf16 neighbours (not representable in... fp32 can hold them): ties to even
    one = 1.0
    ulp = 2.0 ** -7                                       # bf16 spacing in [1, 2)
    assert O.widen(O.round_to_storage(np.array([one + ulp / 2]), "bf16"))[0] == 1.0            # even below
    assert O.widen(O.round_to_storage(np.array([one + ulp + ulp / 2]), "bf16"))[0] == 1.0 + 2 * ulp
    # a float64 just above the midpoint must round up even though fp32 would hide the excess
    v = one + ulp / 2 + 2.0 ** -40
    assert O.widen(O.round_to_storage(np.array([v]), "bf16"))[0] == 1.0 + ulp
    assert O.widen(O.round_to_storage(np.array([-v]), "bf16"))[0] == -(1.0 + ulp)
    assert O.round_to_storage(np.array([0.1]), "f32").dtype == np.float32


def test_widen_reads_bf16_bits_exactly():
    bits = np.array([0x3F80, 0xBF80, 0x4049, 0x0000, 0x8000], dtype=np.uint16)
    assert list(O.widen(bits)) == [1.0, -1.0, 3.140625, 0.0, -0.0]
    with pytest.raises(TypeError):
        O.widen(np.array([1, 2], dtype=np.int32))


# ------------------------------------------------------------------ margins
def test_routing_margin():
    assert O.routing_margin_ulps(np.array([1.0, 1.0, 0.0], np.float32), 1) == 0.0
    one_up = np.nextafter(np.float32(1.0), np.float32(2.0))
    assert O.routing_margin_ulps(np.array([one_up, 1.0, 0.0], np.float32), 1) == 1.0
    # gap below the cut does not matter, gap at the cut and inside the top-k does
    m = O.routing_margin_ulps(np.array([4.0, 2.0, 1.0, 1.0], np.float32), 2)
    assert m > 1e6


# ------------------------------------------------------------------ the paper's printed numbers
def test_byte_sizes_the_paper_prints():
    mx = GOLD["mixtral"]
    assert O.embedding_bytes(mx["hidden"], 4) == GOLD["embedding_bytes_per_token_layer"]["value"]
    one = O.expert_bytes(mx["hidden"], mx["ffn"], 4)
    assert one == 704_643_072 and one < GOLD["worker_gpu_bytes_upper"]["value"]
    total_gb = one * mx["n_experts"] * mx["n_layers"] / 1e9
    assert abs(total_gb - GOLD["full_model_gpu_gb"]["value"]) < 1.0          # 180.4 GB of experts
    assert O.expert_bytes(mx["hidden"], mx["ffn"], 2) == 352_321_536
    assert O.cacheless_loads_per_token(32, 2) == 64


def test_recall_definitions_and_random_prefetch_rate():
    # hand-made arrays: Q=2 prompts, N=3 tokens, L=2 layers, k=2
    c = np.array([[[2, 1], [0, 2], [1, 1]],
                  [[2, 2], [1, 0], [9, 9]]])          # last token of prompt 2 does not exist
    A = np.array([[1, 1, 1], [1, 1, 0]])
    assert math.isclose(O.recall(c, A, 2), (3 + 2 + 2 + 4 + 1) / (2 * 2 * 5))
    assert np.allclose(O.recall_per_token(c, A, 2), [(3 + 4) / 8, (2 + 1) / 8, 2 / 4])
    # random prefetch of k of E experts: expected recall k / E (the paper quotes about 25% for 2 of 8)
    E, k, Q, N, L = 8, 2, 4, 200, 32
    r = np.random.default_rng(0)
    cc = np.zeros((Q, N, L))
    for q in range(Q):
        for n in range(N):
            for l in range(L):
                cc[q, n, l] = O.correct_predictions(r.permutation(E)[:k], r.permutation(E)[:k])
    got = O.recall(cc, np.ones((Q, N)), k)
    assert abs(got - GOLD["random_prefetch_recall"]["value"]) < 0.01
    assert O.correct_predictions(np.array([1, 2]), np.array([2, 1])) == 2


def test_load_window_matches_worked_example():
    ex = GOLD["maxload_example"]
    tM, tW = 1.7, 0.9
    assert math.isclose(O.t_maxload(ex["n_groups"], tM, tW), ex["coef_tM"] * tM + ex["coef_tW"] * tW)
