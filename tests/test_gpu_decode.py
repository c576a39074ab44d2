"""GPU parity: the HIP path (through the C-ABI) against the CPU oracle, element by element.

Tolerances (from the benchmark description): routing indices bit-exact (ties: lowest
index first); fp32 outputs max-abs-err <= 1e-4; bf16 outputs max-abs-err <= 2e-2 * max|y_ref|
per token.  Gate weights: <= 1e-6 absolute (fp32 exp and division against float64).
"""
import numpy as np
import pytest

from oracle import moe_oracle as O
from paper_2512_03927_amd import synth

pytestmark = pytest.mark.gpu

FP32_ATOL = 1e-4
BF16_REL = 2e-2
GATE_ATOL = 1e-6


@pytest.fixture(scope="module")
def H():
    from paper_2512_03927_amd import harness
    return harness


def check_y(y_gpu_stored, y_ref64, dtype, batch=False):
    y = O.widen(y_gpu_stored)
    err = np.max(np.abs(y - y_ref64))
    if dtype == "f32":
        assert err <= FP32_ATOL, f"fp32 max abs err {err}"
    else:
        scale = np.max(np.abs(y_ref64))
        assert err <= BF16_REL * scale, f"bf16 err {err} vs scale {scale}"
        # tighter, informative bound for the GEMV path: one bf16 rounding of a value computed in
        # fp32 (a batch may take the grouped GEMMs, which round the SwiGLU intermediate to bf16)
        if not batch:
            assert err <= 2.0 ** -8 * scale * 1.5 + 1e-30


def oracle_tokens(cfg, X, Wg, b, experts):
    return O.moe_layer_tokens(X, Wg, b, experts, cfg.top_k)


# ---------------------------------------------------------------- config 1 (fp32) as stated
def test_cfg1_fp32_route_and_ffn_all_16_tokens(H):
    cfg = synth.CONFIGS[1]
    Wg, b, experts = synth.layer_weights(cfg)
    X = synth.tokens(cfg)
    Y, IDX, G = oracle_tokens(cfg, X, Wg, b, experts)
    with H.MoEStack(cfg, [(Wg, b, experts)]) as st:
        x = H.to_device(X)
        idx, gate = st.route(0, x)
        assert np.array_equal(idx.cpu().numpy(), IDX)
        assert np.max(np.abs(gate.cpu().numpy().astype(np.float64) - G)) <= GATE_ATOL
        y = st.ffn(0, idx, gate, x)
        yn = H.from_device(y)
        for t in range(cfg.n_tokens):
            check_y(yn[t], Y[t], "f32")
        # the fused per-token entry point gives the same bits as route + ffn on that token (the
        # batch of 16 above went through the grouped GEMMs, whose sums run in another order)
        for t in (0, 7, 15):
            yt, idx_t, stats = st.decode(x[t])
            assert np.array_equal(idx_t[0], IDX[t])
            y1 = st.ffn(0, idx[t:t + 1].contiguous(), gate[t:t + 1].contiguous(), x[t:t + 1].contiguous())
            assert np.array_equal(H.from_device(yt), H.from_device(y1)[0])
            check_y(H.from_device(yt), Y[t], "f32")
            assert stats.loads == 0 and stats.h2d_bytes == 0
    margins = [O.routing_margin_ulps(O.router_logits(Wg, b, X[t]), cfg.top_k) for t in range(cfg.n_tokens)]
    assert min(margins) > 0


# ---------------------------------------------------------------- shapes spanning tiles + ragged tails
SHAPES = [
    # H, F, E, k, dtype
    (520, 1048, 8, 2, "bf16"),      # ragged tails in both GEMVs (chunk = 512 elements)
    (264, 520, 5, 3, "f32"),        # fp32 chunk = 256
    (1024, 2816, 16, 4, "bf16"),
    (8, 8, 2, 1, "bf16"),           # smallest legal shape, k = 1 (gate == 1)
    (2048, 1408, 64, 6, "bf16"),    # fine-grained layer shape (config 5)
    (64, 72, 8, 8, "f32"),          # k = E = max top-k
    (4104, 264, 4, 2, "f32"),       # H beyond the register-resident w1/w3 kernel -> LDS-staged fallback
    (64, 32776, 3, 2, "f32"),       # F beyond the register-resident w2 kernel -> LDS-staged fallback
    (8200, 72, 4, 2, "bf16"),       # bf16 H just past 16 chunks -> fallback
    (4096, 14336, 8, 2, "bf16"),    # the Mixtral layer shape (configs 2-4)
    (64, 64, 1024, 8, "bf16"),      # the most experts and the largest top-k the library takes
    (64, 64, 1, 1, "f32"),          # a single expert
    (256, 8192, 4, 2, "bf16"),      # w2 rows of 16 chunks: four column slices x two expert groups per block
    (4096, 256, 4, 2, "f32"),       # fp32 rows of 16 register chunks (16 waves per CU in the w1/w3 GEMV)
    (6144, 64, 4, 2, "bf16"),       # bf16 rows of 12 register chunks
    (40960, 8, 2, 1, "f32"),        # the longest hidden vector the library takes (160 KB of LDS in the fallback)
    (8, 40960, 3, 2, "bf16"),       # the longest ffn vector
]


@pytest.mark.parametrize("Hd,F,E,k,dtype", SHAPES)
def test_layer_parity_shapes(H, Hd, F, E, k, dtype):
    cfg = synth.MoEConfig("t", Hd, F, E, k, dtype=dtype, n_tokens=5 if Hd * F < (1 << 24) else 2,
                          router_bias=(E == 5), seed=3)
    Wg, b, experts = synth.layer_weights(cfg)
    X = synth.tokens(cfg)
    Y, IDX, G = oracle_tokens(cfg, X, Wg, b, experts)
    with H.MoEStack(cfg, [(Wg, b, experts)]) as st:
        x = H.to_device(X)
        idx, gate = st.route(0, x)
        assert np.array_equal(idx.cpu().numpy(), IDX)
        assert np.max(np.abs(gate.cpu().numpy().astype(np.float64) - G)) <= GATE_ATOL
        assert np.allclose(gate.cpu().numpy().sum(axis=1), 1.0, atol=1e-6)
        # token by token: always the GEMV kernels
        for t in range(cfg.n_tokens):
            y1 = st.ffn(0, idx[t:t + 1].contiguous(), gate[t:t + 1].contiguous(), x[t:t + 1].contiguous())
            check_y(H.from_device(y1)[0], Y[t], dtype)
        # the batch in one call (grouped GEMMs when the token-slots outnumber the experts and the
        # shape allows them, else the same GEMVs)
        yn = H.from_device(st.ffn(0, idx, gate, x))
        for t in range(cfg.n_tokens):
            check_y(yn[t], Y[t], dtype, batch=True)


def _random_shapes(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        E = int(rng.integers(1, 25))
        out.append((8 * int(rng.integers(1, 257)), 8 * int(rng.integers(1, 257)), E,
                    int(rng.integers(1, min(E, 4) + 1)), "bf16" if rng.random() < 0.6 else "f32"))
    return out


@pytest.mark.parametrize("Hd,F,E,k,dtype", _random_shapes(12, 2024))
def test_layer_parity_random_small_shapes(H, Hd, F, E, k, dtype):
    """Seeded random shapes (hidden and ffn any multiple of 8 up to 2048, 1-24 experts): ragged
    chunks, odd wave counts and every launch-policy branch the fixed list may miss; token by token
    (GEMVs), as a batch (grouped GEMMs where the shape allows them) and from pinned host memory."""
    cfg = synth.MoEConfig("t", Hd, F, E, k, dtype=dtype, n_tokens=3, router_bias=bool(E % 2), seed=Hd + F)
    Wg, b, experts = synth.layer_weights(cfg)
    X = synth.tokens(cfg)
    Y, IDX, G = oracle_tokens(cfg, X, Wg, b, experts)
    with H.MoEStack(cfg, [(Wg, b, experts)]) as st, \
            H.MoEStack(cfg, [(Wg, b, experts)], experts_in_host_memory=True) as st_host:
        x = H.to_device(X)
        idx, gate = st.route(0, x)
        assert np.array_equal(idx.cpu().numpy(), IDX)
        assert np.max(np.abs(gate.cpu().numpy().astype(np.float64) - G)) <= GATE_ATOL
        for t in range(cfg.n_tokens):
            args = (idx[t:t + 1].contiguous(), gate[t:t + 1].contiguous(), x[t:t + 1].contiguous())
            y1 = H.from_device(st.ffn(0, *args))[0]
            check_y(y1, Y[t], dtype)
            assert np.array_equal(H.from_device(st_host.ffn(0, *args))[0], y1)   # same bits read in place
        yn = H.from_device(st.ffn(0, idx, gate, x))
        for t in range(cfg.n_tokens):
            check_y(yn[t], Y[t], dtype, batch=True)


# ---------------------------------------------------------------- routing edge cases
@pytest.mark.parametrize("E", [12, 40])   # 40 experts: few-token calls take the multi-block router
def test_routing_ties_zero_router_and_bias(H, E):
    cfg = synth.MoEConfig("t", 256, 64, E, 4, dtype="bf16", n_tokens=40, seed=5)
    Wg, _, experts = synth.layer_weights(cfg)
    Wg = Wg.copy()
    Wg[7] = Wg[2]
    Wg[10] = Wg[2]           # three bit-identical rows -> exact ties, lowest index first
    Wg[4] = 0                # a zero row: logit exactly 0 (+0.0 / -0.0 both possible with bias)
    X = synth.tokens(cfg)
    b = np.zeros(cfg.n_experts, np.float32)
    b[4] = -0.0
    for bias in (None, b):
        with H.MoEStack(cfg, [(Wg, bias, experts)]) as st:
            xd = H.to_device(X)
            idx, gate = st.route(0, xd)
            idx, gate = idx.cpu().numpy(), gate.cpu().numpy()
            # few tokens at a time go through the router variant that spreads a token's experts
            # over several blocks: same bits, also when called repeatedly
            for lo, hi in ((0, 16), (16, 19), (19, 20), (0, 16)):
                i2, g2 = st.route(0, xd[lo:hi].contiguous())
                assert np.array_equal(i2.cpu().numpy(), idx[lo:hi])
                assert np.array_equal(g2.cpu().numpy(), gate[lo:hi])
        hit = 0
        for t in range(cfg.n_tokens):
            ri, rg, _ = O.route(Wg, bias, X[t], cfg.top_k)
            assert np.array_equal(idx[t], ri)
            assert np.max(np.abs(gate[t] - rg)) <= GATE_ATOL
            pos = {int(e): i for i, e in enumerate(idx[t])}
            if 7 in pos:
                hit += 1
                assert 2 in pos and pos[2] < pos[7]
        assert hit > 0, "the tie case never reached the top-k; change the seed of this test"
    # all-zero router: idx = 0..k-1, g = 1/k exactly
    Z = np.zeros_like(Wg)
    with H.MoEStack(cfg, [(Z, None, experts)]) as st:
        for n in (cfg.n_tokens, 3):
            idx, gate = st.route(0, H.to_device(X[:n]))
            assert (idx.cpu().numpy() == np.arange(cfg.top_k)).all()
            assert (gate.cpu().numpy() == np.float32(1.0 / cfg.top_k)).all()
        # x = 0 -> y = 0 exactly
        x0 = st.empty_x(1).zero_()
        i0, g0 = st.route(0, x0)
        assert (H.from_device(st.ffn(0, i0, g0, x0)) == 0).all()


def test_idx_that_is_no_expert_id_selects_nothing(H):
    """idx comes from the caller's device memory.  An entry outside [0, E) must not be used as a
    table index: on the per-token path that rank is left out of the sum, as on the grouped path."""
    import torch
    cfg = synth.MoEConfig("t", 264, 520, 6, 3, dtype="bf16", n_tokens=2, seed=9)
    Wg, b, experts = synth.layer_weights(cfg)
    X = synth.tokens(cfg)
    with H.MoEStack(cfg, [(Wg, b, experts)]) as st:
        x = H.to_device(X)
        idx, gate = st.route(0, x)
        assert x.shape[0] * cfg.top_k <= cfg.n_experts           # per-token GEMV path
        bad = idx.clone()
        bad[0, 1] = 1 << 20
        bad[1, 0] = -7
        yb = H.from_device(st.ffn(0, bad, gate, x))
        ids, g = idx.cpu().numpy(), gate.cpu().numpy().astype(np.float64)
        for t, skip in ((0, 1), (1, 0)):
            ref = np.zeros(cfg.hidden)
            for i in range(cfg.top_k):
                if i != skip:
                    ref += g[t, i] * O.expert_ffn(*O.split_expert(experts[ids[t, i]], cfg.hidden, cfg.ffn), X[t])
            check_y(yb[t], ref, "bf16")
        y_ok = H.from_device(st.ffn(0, idx, gate, x))             # and the handle is fine afterwards
        Y, _, _ = oracle_tokens(cfg, X, Wg, b, experts)
        check_y(y_ok[0], Y[0], "bf16")


def test_multi_block_router_is_repeatable(H):
    """The router variant that spreads a token's experts over several blocks relies on a ticket
    counter that every launch leaves at zero: many launches in a row, with varying token counts,
    keep giving the bits of the one-block-per-token variant (which batches of more than 16 tokens
    take), and so does a launch that follows other work on the stream."""
    import torch
    cfg = synth.MoEConfig("t", 512, 64, 96, 6, dtype="bf16", n_tokens=48, seed=6)
    Wg, _, experts = synth.layer_weights(cfg)
    X = synth.tokens(cfg)
    with H.MoEStack(cfg, [(Wg, None, experts)]) as st:
        xd = H.to_device(X)
        idx_ref, gate_ref = st.route(0, xd)                      # 48 tokens: one block per token
        idx_ref, gate_ref = idx_ref.cpu(), gate_ref.cpu()
        r = np.random.default_rng(1)
        outs = []
        for it in range(300):
            n = int(r.integers(1, 17))
            lo = int(r.integers(0, cfg.n_tokens - n + 1))
            outs.append((lo, n, st.route(0, xd[lo:lo + n].contiguous())))
            if it % 50 == 49:
                st.ffn(0, outs[-1][2][0], outs[-1][2][1], xd[lo:lo + n].contiguous())
        torch.cuda.synchronize()
        for lo, n, (i2, g2) in outs:
            assert torch.equal(i2.cpu(), idx_ref[lo:lo + n]) and torch.equal(g2.cpu(), gate_ref[lo:lo + n])


def test_identical_experts_make_routing_irrelevant(H):
    cfg = synth.MoEConfig("t", 128, 256, 6, 3, dtype="f32", n_tokens=3, seed=8)
    Wg, _, experts = synth.layer_weights(cfg)
    same = [experts[0]] * cfg.n_experts
    X = synth.tokens(cfg)
    with H.MoEStack(cfg, [(Wg, None, same)]) as st:
        x = H.to_device(X)
        idx, gate = st.route(0, x)
        yn = H.from_device(st.ffn(0, idx, gate, x))
    for t in range(3):
        ref = O.expert_ffn(*O.split_expert(experts[0], cfg.hidden, cfg.ffn), X[t])
        assert np.max(np.abs(yn[t] - ref)) <= FP32_ATOL


# ---------------------------------------------------------------- cacheless stacks
def _stack_layers(cfg):
    return [synth.layer_weights(cfg, l) for l in range(cfg.n_layers)]


@pytest.mark.parametrize("dtype,Hd,F,E,k,L,S", [("bf16", 256, 512, 8, 2, 6, 4), ("f32", 128, 264, 8, 2, 4, 2),
                                                 ("bf16", 256, 264, 16, 3, 5, 7)])
def test_cacheless_stack_free_running_and_teacher_forced(H, dtype, Hd, F, E, k, L, S):
    cfg = synth.MoEConfig("t", Hd, F, E, k, n_layers=L, n_slots=S, dtype=dtype, n_tokens=4, glue=1, seed=11)
    layers = _stack_layers(cfg)
    X = synth.tokens(cfg)
    with H.MoEStack(cfg, layers) as st:
        assert st.handle is not None
        from paper_2512_03927_amd import binding as B
        assert B.odmoe_slot_pool_bytes(st.handle) == S * cfg.expert_bytes
        for t in range(cfg.n_tokens):
            x_ref, IDX, xs = O.stack_decode(X[t], layers, k, dtype, glue=1)
            y, idx, stats = st.decode(H.to_device(X[t]))
            assert np.array_equal(idx, IDX)                       # free-running routing, every layer
            assert stats.loads == L * k and stats.reloads == 0    # every activation is a load
            assert stats.h2d_bytes == L * k * cfg.expert_bytes
            got = O.widen(H.from_device(y))
            tol = FP32_ATOL if dtype == "f32" else BF16_REL * np.max(np.abs(O.widen(x_ref)))
            assert np.max(np.abs(got - O.widen(x_ref))) <= tol
            # teacher-forced: layer l on the oracle's input to layer l, via the fine-grained calls
            for l in range(L):
                xl = H.to_device(xs[l].reshape(1, -1))
                idx_d, gate_d = st.route(l, xl)
                ids = idx_d.cpu().numpy()[0]
                assert np.array_equal(ids, IDX[l])
                for e in ids:
                    B.odmoe_expert_load_async(st.handle, l, int(e))
                yl = st.ffn(l, idx_d, gate_d, xl, idx_host=np.ascontiguousarray(ids), evict_after=1)
                y_ref, _, _ = O.moe_layer(xs[l], *layers[l], k)
                check_y(H.from_device(yl)[0], y_ref, dtype)


def test_hints_change_timing_only(H):
    cfg = synth.MoEConfig("t", 256, 512, 8, 2, n_layers=8, n_slots=4, dtype="bf16", n_tokens=2, glue=1, seed=13)
    layers = _stack_layers(cfg)
    X = synth.tokens(cfg)
    L, k, E = cfg.n_layers, cfg.top_k, cfg.n_experts
    with H.MoEStack(cfg, layers) as st:
        for t in range(cfg.n_tokens):
            x = H.to_device(X[t])
            y0, idx0, s0 = st.decode(x)
            base = H.from_device(y0)
            # perfect hints
            y1, idx1, s1 = st.decode(x, pred=idx0)
            assert np.array_equal(H.from_device(y1), base) and np.array_equal(idx1, idx0)
            assert s1.loads == L * k and s1.reloads == 0 and s1.hint_hits == L * k
            # every hint wrong
            wrong = np.stack([[e for e in range(E) if e not in idx0[l]][:k] for l in range(L)]).astype(np.int32)
            y2, idx2, s2 = st.decode(x, pred=wrong)
            assert np.array_equal(H.from_device(y2), base) and np.array_equal(idx2, idx0)
            assert s2.reloads == L * k and s2.hint_hits == 0 and s2.loads == 2 * L * k
            # mixed / unusable hints
            mix = idx0.copy()
            mix[1] = wrong[1]
            mix[2, 0] = -5
            mix[5] = mix[5][::-1]
            y3, idx3, s3 = st.decode(x, pred=mix)
            assert np.array_equal(H.from_device(y3), base) and np.array_equal(idx3, idx0)
            assert s3.reloads == k + 1 and s3.hint_hits == L * k - (k + 1)
            # timed variant fills the time fields
            y4, _, s4 = st.decode(x, pred=idx0, timed=True)
            assert np.array_equal(H.from_device(y4), base)
            assert s4.t_step_ms > 0 and s4.t_ffn_up_ms > 0 and s4.t_ffn_down_ms > 0 and s4.t_load_ms > 0
            assert s4.t_route_ms > 0 and s4.t_glue_ms > 0
        # the copy-only replay moves the same bytes, leaves every slot free, and the stack still
        # gives the same output afterwards (the slots it overwrote held no expert)
        from paper_2512_03927_amd import binding as B
        ms = B.odmoe_time_expert_loads(st.handle, 2)
        assert ms > 0
        y5, idx5, s5 = st.decode(x)
        assert np.array_equal(H.from_device(y5), base) and s5.loads == L * k
    with H.MoEStack(cfg.small(n_slots=0), layers) as st_res:
        with pytest.raises(RuntimeError):
            B.odmoe_time_expert_loads(st_res.handle, 1)          # resident mode has no loads


def test_experts_read_in_place_from_pinned_host_memory(H):
    """n_slots = 0 with expert pointers into pinned host memory: the kernels read the weights over
    the host link; output and routing equal the slot pool's bit for bit, and match the oracle."""
    cfg = synth.MoEConfig("t", 256, 512, 8, 2, n_layers=6, n_slots=4, dtype="bf16", n_tokens=3, glue=1, seed=29)
    layers = _stack_layers(cfg)
    X = synth.tokens(cfg)
    with H.MoEStack(cfg, layers) as st_pool, \
            H.MoEStack(cfg.small(n_slots=0), layers, experts_in_host_memory=True) as st_host:
        for t in range(cfg.n_tokens):
            x = H.to_device(X[t])
            y0, idx0, s0 = st_pool.decode(x)
            y1, idx1, s1 = st_host.decode(x)
            assert np.array_equal(H.from_device(y0), H.from_device(y1)) and np.array_equal(idx0, idx1)
            assert s1.loads == 0 and s1.h2d_bytes == 0          # nothing was copied
        x_ref, ids_ref, _ = O.stack_decode(X[0], layers, cfg.top_k, "bf16", glue=1)
        y, idx, _ = st_host.decode(H.to_device(X[0]))
        assert np.array_equal(idx, ids_ref)
        assert np.max(np.abs(O.widen(H.from_device(y)) - O.widen(x_ref))) <= BF16_REL * np.max(np.abs(O.widen(x_ref)))
        # a small batch through the grouped GEMMs reads the host-resident weights too
        xb = H.to_device(X)
        idx_d, gate_d = st_host.route(0, xb)
        yb = H.from_device(st_host.ffn(0, idx_d, gate_d, xb))
        for t in range(cfg.n_tokens):
            y_ref, _, _ = O.moe_layer(X[t], *layers[0], cfg.top_k)
            check_y(yb[t], y_ref, "bf16", batch=True)


def test_caller_supplied_copy_stream_gives_the_same_tokens(H):
    """With a copy stream borrowed from the caller every expert copy goes through that one stream
    (the library's own four-stream rotation is off): same output, same load count."""
    import torch
    cfg = synth.MoEConfig("t", 256, 512, 8, 2, n_layers=6, n_slots=4, dtype="bf16", n_tokens=3, glue=1, seed=19)
    layers = _stack_layers(cfg)
    X = synth.tokens(cfg)
    cs = torch.cuda.Stream()
    with H.MoEStack(cfg, layers) as st_own, H.MoEStack(cfg, layers, copy_stream=cs) as st_ext:
        for t in range(cfg.n_tokens):
            x = H.to_device(X[t])
            y0, idx0, s0 = st_own.decode(x)
            y1, idx1, s1 = st_ext.decode(x)
            assert np.array_equal(H.from_device(y0), H.from_device(y1)) and np.array_equal(idx0, idx1)
            assert s0.loads == s1.loads == cfg.n_layers * cfg.top_k
            y2, _, s2 = st_ext.decode(x, pred=idx0)
            assert np.array_equal(H.from_device(y2), H.from_device(y0)) and s2.hint_hits == s2.loads


def test_hint_recall_is_what_was_planted(H):
    """Hints corrupted at a chosen rate: the output never changes, and the confirmed fraction
    (the paper's recall, Section 3.2) is exactly the fraction of hints left intact."""
    from paper_2512_03927_amd import binding as B
    cfg = synth.MoEConfig("t", 128, 256, 8, 2, n_layers=16, n_slots=4, dtype="bf16", n_tokens=3, glue=1, seed=17)
    layers = _stack_layers(cfg)
    X = synth.tokens(cfg)
    L, k, E = cfg.n_layers, cfg.top_k, cfg.n_experts
    r = np.random.default_rng(0)
    with H.MoEStack(cfg, layers) as st:
        assert B.odmoe_slot_groups(st.handle) == 2
        for t in range(cfg.n_tokens):
            x = H.to_device(X[t])
            y0, idx0, _ = st.decode(x)
            for rate in (0.0, 0.25, 0.75):
                pred = idx0.copy()
                n_bad = 0
                for l in range(L):
                    for i in range(k):
                        if r.random() < rate:
                            pred[l, i] = [e for e in range(E) if e not in idx0[l] and e not in pred[l]][0]
                            n_bad += 1
                y, idx, s = st.decode(x, pred=pred)
                assert np.array_equal(H.from_device(y), H.from_device(y0)) and np.array_equal(idx, idx0)
                assert s.hint_hits == L * k - n_bad and s.reloads == n_bad
                assert s.loads == L * k + n_bad
                recall = O.recall(np.array([[[O.correct_predictions(pred[l], idx0[l]) for l in range(L)]]]),
                                  np.ones((1, 1)), k)
                assert abs(recall - s.hint_hits / (L * k)) < 1e-12


def test_error_paths(H):
    from paper_2512_03927_amd import binding as B
    cfg = synth.MoEConfig("t", 64, 64, 4, 2, n_layers=2, n_slots=2, dtype="f32", n_tokens=1, glue=1)
    layers = _stack_layers(cfg)
    with H.MoEStack(cfg, layers) as st:
        x = H.to_device(synth.tokens(cfg))
        idx, gate = st.route(0, x)
        ids = idx.cpu().numpy()[0]
        with pytest.raises(B.OdmoeError) as ei:                   # nothing loaded yet
            st.ffn(0, idx, gate, x, idx_host=ids)
        assert ei.value.code == B.ODMOE_ESTATE
        s0 = B.odmoe_expert_load_async(st.handle, 0, 0)
        assert B.odmoe_expert_load_async(st.handle, 0, 0) == s0     # already loading: same slot
        B.odmoe_expert_load_async(st.handle, 0, 1)
        with pytest.raises(B.OdmoeError) as ei:
            B.odmoe_expert_load_async(st.handle, 0, 2)
        assert ei.value.code == B.ODMOE_EBUSY
        B.odmoe_expert_evict(st.handle, 0, 0)
        with pytest.raises(B.OdmoeError) as ei:
            B.odmoe_expert_evict(st.handle, 0, 0)
        assert ei.value.code == B.ODMOE_ESTATE
        B.odmoe_expert_evict(st.handle, 0, 1)
        for bad in ((5, 0), (0, 9), (-1, 0)):
            with pytest.raises(B.OdmoeError) as ei:
                B.odmoe_expert_load_async(st.handle, *bad)
            assert ei.value.code == B.ODMOE_EINVAL
        with pytest.raises(B.OdmoeError):
            st.route(7, x)
        # without idx_host the library reads idx back itself
        for e in ids:
            B.odmoe_expert_load_async(st.handle, 0, int(e))
        y = st.ffn(0, idx, gate, x, idx_host=None)
        y_ref, _, _ = O.moe_layer(synth.tokens(cfg)[0], *layers[0], cfg.top_k)
        check_y(H.from_device(y)[0], y_ref, "f32")
        # empty batch is a no-op
        B.odmoe_route_topk(st.handle, 0, x, 0, idx, gate)
    rcfg = synth.MoEConfig("t", 64, 64, 4, 2, dtype="f32")
    # expert buffers in plain (pageable) host memory: refused at init, in either mode
    import torch
    Wg_r, _, experts_r = synth.layer_weights(rcfg)
    router_dev = H.to_device(Wg_r)
    for n_slots in (0, 2):
        c = B.odmoe_config(64, 64, 4, 2, 1, n_slots, B.ODMOE_F32, 0)
        with pytest.raises(B.OdmoeError) as ei:
            B.odmoe_layer_init(c, [router_dev], None, [np.ascontiguousarray(e) for e in experts_r],
                               torch.cuda.current_stream().cuda_stream, None)
        assert ei.value.code == B.ODMOE_EINVAL
    c = B.odmoe_config(64, 64, 4, 2, 1, 0, B.ODMOE_F32, 0)
    with pytest.raises(B.OdmoeError) as ei:                      # router weights in plain host memory
        B.odmoe_layer_init(c, [np.ascontiguousarray(Wg_r)], None, [H.to_device(e) for e in experts_r],
                           torch.cuda.current_stream().cuda_stream, None)
    assert ei.value.code == B.ODMOE_EINVAL
    # device buffers where the slot pool expects pinned host memory
    c = B.odmoe_config(64, 64, 4, 2, 1, 2, B.ODMOE_F32, 0)
    with pytest.raises(B.OdmoeError) as ei:
        B.odmoe_layer_init(c, [router_dev], None, [H.to_device(e) for e in experts_r],
                           torch.cuda.current_stream().cuda_stream, None)
    assert ei.value.code == B.ODMOE_EINVAL
    with H.MoEStack(rcfg) as st:
        with pytest.raises(B.OdmoeError) as ei:
            B.odmoe_expert_load_async(st.handle, 0, 0)
        assert ei.value.code == B.ODMOE_EINVAL


def test_resident_decode_step_can_be_captured_in_a_graph(H):
    """Resident mode with nothing to report enqueues kernels only (no allocation, no fill by the
    runtime, no host wait), so a decode step can be recorded into a HIP graph on the handle's
    compute stream.  Every replay, with eager steps and synchronisations in between and the input
    buffer rewritten in place, gives the bits of the eager step."""
    import torch
    cfg = synth.MoEConfig("t", 256, 512, 40, 4, n_layers=5, n_slots=0, dtype="bf16", n_tokens=4, glue=1, seed=23)
    layers = _stack_layers(cfg)
    X = synth.tokens(cfg)
    from paper_2512_03927_amd import binding as B
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        with H.MoEStack(cfg, layers) as st:                  # the handle's compute stream is `side`
            x = H.to_device(X[0])
            y_eager, y_graph = torch.empty_like(x), torch.empty_like(x)
            B.odmoe_decode_step(st.handle, x, y_eager, None, None, None)
            side.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                B.odmoe_decode_step(st.handle, x, y_graph, None, None, None)
            for t in range(cfg.n_tokens):
                x.copy_(H.to_device(X[t]))
                B.odmoe_decode_step(st.handle, x, y_eager, None, None, None)
                side.synchronize()
                y_graph.zero_()
                g.replay()
                side.synchronize()
                assert torch.equal(y_eager, y_graph), f"replay {t}"
                assert float(y_graph.float().abs().max()) > 0
            del g


def test_glue_zero_chains_y(H):
    cfg = synth.MoEConfig("t", 128, 128, 4, 2, n_layers=3, n_slots=0, dtype="f32", n_tokens=1, glue=0, w_std=0.1)
    layers = _stack_layers(cfg)
    X = synth.tokens(cfg)
    x_ref, IDX, _ = O.stack_decode(X[0], layers, cfg.top_k, "f32", glue=0)
    with H.MoEStack(cfg, layers) as st:
        y, idx, _ = st.decode(H.to_device(X[0]))
        assert np.array_equal(idx, IDX)
        assert np.max(np.abs(H.from_device(y) - x_ref)) <= FP32_ATOL
