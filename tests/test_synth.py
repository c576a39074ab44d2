"""The seeded input generator: reproducible, sliceable, right distribution and storage."""
import numpy as np
import pytest

from paper_2512_03927_amd import synth


def test_counter_based_slices_and_threads_agree():
    full = synth.normal(0, 5, 10001, 0.02, threads=1)
    for off, n in [(0, 10001), (1, 999), (2, 1), (4097, 3000), (10000, 1)]:
        part = synth.normal(0, 5, n, 0.02, offset=off, threads=1)
        assert np.array_equal(part, full[off:off + n])
    big1 = synth.normal(3, 9, (1 << 22) + 7, threads=1)
    big4 = synth.normal(3, 9, (1 << 22) + 7, threads=4)
    assert np.array_equal(big1, big4)
    assert not np.array_equal(synth.normal(0, 5, 64), synth.normal(1, 5, 64))
    assert not np.array_equal(synth.normal(0, 5, 64), synth.normal(0, 6, 64))
    assert synth.normal(0, 1, 0).shape == (0,)


def test_distribution_moments():
    a = synth.normal(0, 77, 2_000_000, 0.02).astype(np.float64)
    assert abs(a.mean()) < 1e-4 and abs(a.std() - 0.02) < 1e-4
    z = a / 0.02
    assert abs((z ** 3).mean()) < 0.02 and abs((z ** 4).mean() - 3.0) < 0.05
    assert np.isfinite(a).all()
    # neighbouring elements (the two outputs of one pair) are uncorrelated
    assert abs(np.corrcoef(z[0::2], z[1::2])[0, 1]) < 5e-3


def test_bf16_storage_matches_library_rounding():
    torch = pytest.importorskip("torch")
    a = synth.normal(0, 3, 50000, 5.0)
    want = torch.from_numpy(a).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(synth.f32_to_bf16_bits(a), want)
    back = synth.bf16_bits_to_f32(want)
    assert np.array_equal(back, torch.from_numpy(a).to(torch.bfloat16).float().numpy())


def test_config_table_matches_benchmark_shapes():
    c = synth.CONFIGS
    assert c[1].expert_bytes == 6_291_456 and c[1].dtype == "f32"
    assert c[2].expert_bytes == 352_321_536 and c[3].n_slots == 4 and c[3].n_layers == 32
    assert c[5].expert_bytes == 17_301_504 and c[5].top_k == 6 and c[5].n_experts == 64
    assert c[4].router_bias and c[4].n_tokens == 512


def test_layer_buffers_shapes_and_split():
    cfg = synth.CONFIGS[1].small(hidden=16, ffn=24, n_experts=3)
    Wg, b, ex = synth.layer_weights(cfg)
    assert Wg.shape == (3, 16) and b is None and len(ex) == 3 and ex[0].shape == (3 * 16 * 24,)
    W1, W3, W2 = synth.split_expert(cfg, ex[1])
    assert W1.shape == (24, 16) and W2.shape == (16, 24)
    assert W3[0, 0] == ex[1][16 * 24]
    x = synth.tokens(cfg, 5)
    assert np.array_equal(synth.tokens(cfg, 2, first=3), x[3:5])
    cb = cfg.small(dtype="bf16", router_bias=True)
    assert synth.tokens(cb, 2).dtype == np.uint16 and synth.router_bias(cb).dtype == np.float32
    out = np.empty(cb.expert_elems, np.uint16)
    synth.expert_weights(cb, 0, 2, out=out)
    assert np.array_equal(out, synth.expert_weights(cb, 0, 2))
