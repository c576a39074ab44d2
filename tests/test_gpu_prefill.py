"""GPU parity of the prefill path (tokens grouped by expert, grouped GEMM on the matrix cores)
against the CPU oracle, which simply applies the layer definition to every token.

Tolerance: bf16, max-abs-err <= 2e-2 * max|y_ref| per token (the benchmark's bound); the bf16
prefill kernels round the SwiGLU intermediate to bf16 before the w2 GEMM, the oracle does not.
fp32 layers: max-abs-err <= 1e-4.
"""
import numpy as np
import pytest

from oracle import moe_oracle as O
from paper_2512_03927_amd import synth

pytestmark = pytest.mark.gpu
BF16_REL = 2e-2


@pytest.fixture(scope="module")
def H():
    from paper_2512_03927_amd import harness
    return harness


def _check_tokens(yn, Y, toks):
    worst = 0.0
    for t in toks:
        ref = Y[t]
        err = np.max(np.abs(O.widen(yn[t]) - ref))
        scale = np.max(np.abs(ref))
        assert err <= BF16_REL * scale, f"token {t}: err {err} scale {scale}"
        worst = max(worst, err / scale)
    return worst


@pytest.mark.parametrize("Hd,F,E,k,T,bias", [
    (256, 512, 4, 2, 600, True),     # groups of several M-tiles, ragged tails, skewed routing
    (320, 576, 8, 2, 16, False),     # smallest batch that takes the grouped path; some experts idle
    (128, 192, 8, 3, 257, True),     # k = 3, odd token count
    (2048, 1408, 64, 6, 48, False),  # fine-grained layer shape, most experts see 0-10 tokens
    (128, 192, 16, 4, 1500, True),   # 6000 token-slots: experts with 1-4 chunks each, about 30 chunks
])
def test_prefill_matches_oracle(H, Hd, F, E, k, T, bias):
    cfg = synth.MoEConfig("t", Hd, F, E, k, dtype="bf16", n_tokens=T, router_bias=bias, seed=21)
    Wg, b, experts = synth.layer_weights(cfg)
    X = synth.tokens(cfg)
    Y, IDX, G = O.moe_layer_tokens(X, Wg, b, experts, k)
    with H.MoEStack(cfg, [(Wg, b, experts)]) as st:
        x = H.to_device(X)
        idx, gate = st.route(0, x)
        assert np.array_equal(idx.cpu().numpy(), IDX)
        yn = H.from_device(st.ffn(0, idx, gate, x))                      # n_tokens >= 16 -> grouped GEMM
        _check_tokens(yn, Y, range(T))
        # a few tokens through the per-token GEMV path (token-slots do not outnumber the experts)
        n1 = max(1, E // k)
        y1 = H.from_device(st.ffn(0, idx[:n1].contiguous(), gate[:n1].contiguous(), x[:n1].contiguous()))
        _check_tokens(y1, Y, range(n1))
        # ... and a small batch that just crosses over to the grouped path
        n2 = n1 + 1
        y2 = H.from_device(st.ffn(0, idx[:n2].contiguous(), gate[:n2].contiguous(), x[:n2].contiguous()))
        _check_tokens(y2, Y, range(n2))
        assert np.array_equal(y2, yn[:n2])          # the grouped path does not depend on the batch around a token
    counts = np.bincount(IDX.ravel(), minlength=E)
    assert counts.sum() == T * k


def _random_prefill_cases(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        E = int(rng.integers(2, 33))
        out.append((64 * int(rng.integers(1, 13)), 64 * int(rng.integers(1, 13)), E, int(rng.integers(1, min(E, 4) + 1)),
                    int(rng.integers(17, 900)), bool(rng.integers(0, 2)), "bf16" if rng.random() < 0.6 else "f32"))
    return out


@pytest.mark.parametrize("Hd,F,E,k,T,bias,dtype", _random_prefill_cases(10, 7))
def test_prefill_random_shapes(H, Hd, F, E, k, T, bias, dtype):
    """Seeded random layer shapes, batch sizes and routing skews through the grouped GEMMs: chunk
    classes of every size, experts with no tokens, K splits, both element types."""
    cfg = synth.MoEConfig("t", Hd, F, E, k, dtype=dtype, n_tokens=T, router_bias=bias, seed=Hd + F + T)
    Wg, b, experts = synth.layer_weights(cfg)
    X = synth.tokens(cfg)
    Y, IDX, G = O.moe_layer_tokens(X, Wg, b, experts, k)
    with H.MoEStack(cfg, [(Wg, b, experts)]) as st:
        x = H.to_device(X)
        idx, gate = st.route(0, x)
        assert np.array_equal(idx.cpu().numpy(), IDX)
        yn = H.from_device(st.ffn(0, idx, gate, x))
        if dtype == "f32":
            assert np.max(np.abs(yn - Y)) <= 1e-4
        else:
            _check_tokens(yn, Y, range(T))


def test_prefill_unsupported_shape_falls_back_to_per_token_path(H):
    cfg = synth.MoEConfig("t", 264, 520, 4, 2, dtype="bf16", n_tokens=20, seed=22)   # not multiples of 64
    Wg, b, experts = synth.layer_weights(cfg)
    X = synth.tokens(cfg)
    Y, IDX, _ = O.moe_layer_tokens(X, Wg, b, experts, cfg.top_k)
    with H.MoEStack(cfg, [(Wg, b, experts)]) as st:
        x = H.to_device(X)
        idx, gate = st.route(0, x)
        _check_tokens(H.from_device(st.ffn(0, idx, gate, x)), Y, range(cfg.n_tokens))
    cfg32 = synth.MoEConfig("t", 136, 136, 4, 2, dtype="f32", n_tokens=18, seed=23)   # fp32, not multiples of 64
    Wg, b, experts = synth.layer_weights(cfg32)
    X = synth.tokens(cfg32)
    Y, _, _ = O.moe_layer_tokens(X, Wg, b, experts, 2)
    with H.MoEStack(cfg32, [(Wg, b, experts)]) as st:
        x = H.to_device(X)
        idx, gate = st.route(0, x)
        yn = H.from_device(st.ffn(0, idx, gate, x))
        assert np.max(np.abs(yn - Y)) <= 1e-4


@pytest.mark.parametrize("Hd,F,E,k,T,bias", [
    (256, 512, 4, 2, 600, True),     # chunks of up to 320 rows, ragged tails, skewed routing
    (128, 192, 8, 3, 257, True),     # k = 3, odd token count, K split of the w2 GEMM
    (512, 1024, 8, 2, 16, False),    # config 1's layer shape, smallest batch on the grouped path
    (64, 64, 16, 4, 1500, False),    # one K step per block, about 30 chunks
])
def test_fp32_prefill_matches_oracle(H, Hd, F, E, k, T, bias):
    """Full-precision layers take the grouped GEMMs too (fp32 matrix instructions, nothing rounded
    on the way): parity to the fp32 bound, and equal to the per-token GEMV path within it."""
    cfg = synth.MoEConfig("t", Hd, F, E, k, dtype="f32", n_tokens=T, router_bias=bias, seed=31)
    Wg, b, experts = synth.layer_weights(cfg)
    X = synth.tokens(cfg)
    Y, IDX, G = O.moe_layer_tokens(X, Wg, b, experts, k)
    with H.MoEStack(cfg, [(Wg, b, experts)]) as st:
        x = H.to_device(X)
        idx, gate = st.route(0, x)
        assert np.array_equal(idx.cpu().numpy(), IDX)
        yn = H.from_device(st.ffn(0, idx, gate, x))
        assert yn.dtype == np.float32
        assert np.max(np.abs(yn - Y)) <= 1e-4
        y1 = H.from_device(st.ffn(0, idx[:1].contiguous(), gate[:1].contiguous(), x[:1].contiguous()))   # GEMV path
        assert np.max(np.abs(y1[0] - yn[0])) <= 1e-4
        y_again = H.from_device(st.ffn(0, idx, gate, x))
        assert np.array_equal(y_again, yn)


def test_fp32_cacheless_prefill_from_host(H):
    """fp32 batches in cacheless mode stream each expert once, like bf16 ones."""
    cfg = synth.MoEConfig("t", 128, 256, 8, 2, n_layers=1, n_slots=3, dtype="f32", n_tokens=200, seed=33)
    Wg, b, experts = synth.layer_weights(cfg)
    X = synth.tokens(cfg)
    Y, IDX, _ = O.moe_layer_tokens(X, Wg, b, experts, cfg.top_k)
    with H.MoEStack(cfg, [(Wg, b, experts)]) as st:
        x = H.to_device(X)
        idx, gate = st.route(0, x)
        yn = H.from_device(st.ffn(0, idx, gate, x, idx_host=np.ascontiguousarray(IDX)))
        assert np.max(np.abs(yn - Y)) <= 1e-4


def test_prefill_all_tokens_to_one_expert_and_repeat_calls(H):
    """Degenerate routing: one expert gets every token (3 chunks of 320, 320 and 260 rows that share every
    weight tile), the others none; the call is repeatable (workspace reuse) and a smaller batch
    after a larger one is still right."""
    cfg = synth.MoEConfig("t", 128, 256, 4, 1, dtype="bf16", n_tokens=900, seed=24)
    Wg, _, experts = synth.layer_weights(cfg)
    b = np.array([0.0, 50.0, 0.0, 0.0], np.float32)          # expert 1 always wins
    X = synth.tokens(cfg)
    Y, IDX, _ = O.moe_layer_tokens(X, Wg, b, experts, 1)
    assert (IDX == 1).all()
    with H.MoEStack(cfg, [(Wg, b, experts)]) as st:
        x = H.to_device(X)
        idx, gate = st.route(0, x)
        y_a = H.from_device(st.ffn(0, idx, gate, x))
        y_b = H.from_device(st.ffn(0, idx, gate, x))
        assert np.array_equal(y_a, y_b)
        _check_tokens(y_a, Y, range(cfg.n_tokens))
        y_c = H.from_device(st.ffn(0, idx[:40].contiguous(), gate[:40].contiguous(), x[:40].contiguous()))
        assert np.array_equal(y_c, y_a[:40])


# Measured bound of the bf16 prefill path at full size (the SwiGLU intermediate is rounded to bf16
# before the w2 GEMM, the oracle rounds nothing): the largest error over all 512 tokens of config 4
# is printed by the test below and must stay under this, well inside the benchmark's 2e-2.
CFG4_BF16_PREFILL_REL = 8e-3


def test_cfg4_full_size_prefill_all_512_tokens(H, mixtral_layer, mixtral_experts_f64):
    """Config 4 as stated: Mixtral-shaped layer, 512 tokens, router bias N(0,1).  Routing and
    outputs are compared with the oracle for every token, through the batch call bench.py times."""
    cfg = synth.CONFIGS[4]
    _, (Wg, _, experts) = mixtral_layer                 # config 4's layer is config 2's plus a router bias
    b = synth.router_bias(cfg)
    X = synth.tokens(cfg)
    T, k = cfg.n_tokens, cfg.top_k
    IDX = np.stack([O.route(Wg, b, X[t], k)[0] for t in range(T)])
    counts = np.bincount(IDX.ravel(), minlength=cfg.n_experts)
    print("tokens per expert:", counts.tolist())
    assert counts.min() >= 1, "router skew starves an expert; not representative of a prefill batch"
    assert counts.max() > 128, "no expert spans more than one M-tile; the skew is too weak for this test"
    with H.MoEStack(cfg, [(Wg, b, experts)]) as st:
        x = H.to_device(X)
        idx, gate = st.route(0, x)
        assert np.array_equal(idx.cpu().numpy(), IDX)
        yn = H.from_device(st.ffn(0, idx, gate, x))
        # a decode token on the same handle takes the GEMV path and agrees to one bf16 rounding
        y1 = H.from_device(st.ffn(0, idx[7:8].contiguous(), gate[7:8].contiguous(), x[7:8].contiguous()))[0]
    worst = 0.0
    for t in range(T):
        y_ref, idx_ref, _ = O.moe_layer(X[t], Wg, b, mixtral_experts_f64, k)
        assert np.array_equal(idx_ref, IDX[t])
        err = float(np.max(np.abs(O.widen(yn[t]) - y_ref)) / np.max(np.abs(y_ref)))
        assert err <= BF16_REL, f"token {t}: {err}"
        worst = max(worst, err)
        if t == 7:
            assert np.max(np.abs(O.widen(y1) - y_ref)) <= 1.5 * 2.0 ** -8 * np.max(np.abs(y_ref))
    print("config 4: worst max-abs error over all 512 tokens = %.3e of max|y| (bf16 prefill path)" % worst)
    assert worst <= CFG4_BF16_PREFILL_REL


def test_cacheless_prefill_streams_each_expert_once_and_matches_resident(H):
    """Prefill with the experts in pinned host memory and only 2 HBM slots: each expert that got
    tokens is copied once, results are bit-identical to the resident prefill and match the oracle."""
    from paper_2512_03927_amd import binding as B
    cfg = synth.MoEConfig("t", 256, 512, 8, 2, dtype="bf16", n_tokens=300, router_bias=True, seed=31)
    Wg, b, experts = synth.layer_weights(cfg)
    X = synth.tokens(cfg)
    Y, IDX, _ = O.moe_layer_tokens(X, Wg, b, experts, cfg.top_k)
    with H.MoEStack(cfg, [(Wg, b, experts)]) as res:
        x = H.to_device(X)
        idx, gate = res.route(0, x)
        y_res = H.from_device(res.ffn(0, idx, gate, x))
    for n_slots, idx_host in ((2, None), (3, np.ascontiguousarray(IDX))):
        ccfg = cfg.small(n_slots=n_slots)
        with H.MoEStack(ccfg, [(Wg, b, experts)]) as st:
            x = H.to_device(X)
            idx, gate = st.route(0, x)
            assert np.array_equal(idx.cpu().numpy(), IDX)
            y = H.from_device(st.ffn(0, idx, gate, x, idx_host=idx_host, evict_after=1))
            assert np.array_equal(y, y_res)
            _check_tokens(y, Y, range(0, cfg.n_tokens, 7))
            # everything was evicted: a second call loads again and gives the same bits
            y2 = H.from_device(st.ffn(0, idx, gate, x, idx_host=idx_host, evict_after=1))
            assert np.array_equal(y2, y_res)
            # a decode token on the same handle still works afterwards
            yt, idx_t, stats = st.decode(x[5])
            assert np.array_equal(idx_t[0], IDX[5]) and stats.loads == cfg.top_k
            # a batch of a few tokens streams only the experts those tokens chose
            y4 = H.from_device(st.ffn(0, idx[:4].contiguous(), gate[:4].contiguous(), x[:4].contiguous(),
                                      idx_host=None if idx_host is None else np.ascontiguousarray(idx_host[:4]),
                                      evict_after=1))
            assert np.array_equal(y4, y_res[:4])
