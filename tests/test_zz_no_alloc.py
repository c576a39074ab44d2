"""The entry point that allocates nothing (odmoe_expert_ffn_static) against odmoe_expert_ffn.

Two calls in a row on the same GPU, the second with a smaller input (fewer tokens of a smaller
layer), so the second call runs over whatever the first left in the library's static scratch:
both must give the bits of the handle-based per-token path, and match the CPU oracle.
"""
import numpy as np
import pytest

from oracle import moe_oracle as O
from paper_2512_03927_amd import synth

pytestmark = pytest.mark.gpu


def _case(H, B, torch, Hd, F, E, k, T, dtype, seed):
    cfg = synth.MoEConfig("t", Hd, F, E, k, dtype=dtype, n_tokens=T, seed=seed)
    Wg, b, experts = synth.layer_weights(cfg)
    X = synth.tokens(cfg)
    Y, IDX, G = O.moe_layer_tokens(X, Wg, b, experts, k)
    with H.MoEStack(cfg, [(Wg, b, experts)]) as st:
        x = H.to_device(X)
        idx, gate = st.route(0, x)
        assert np.array_equal(idx.cpu().numpy(), IDX)
        assert T * k <= E and T < 16                      # the handle takes its per-token path
        y_handle = st.ffn(0, idx, gate, x)
        # the same expert buffers, addressed through a caller-made device table
        experts_dev = st._keep[2][0]
        table = torch.tensor([e.data_ptr() for e in experts_dev], dtype=torch.int64, device="cuda:0")
        c = B.odmoe_config(Hd, F, E, k, 1, 0, B.ODMOE_F32 if dtype == "f32" else B.ODMOE_BF16, 0)
        y_static = torch.zeros_like(x)
        B.odmoe_expert_ffn_static(c, table, idx, gate, x, T, y_static, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        a, r = H.from_device(y_static), H.from_device(y_handle)
    assert np.array_equal(a, r), f"static entry point differs from odmoe_expert_ffn ({Hd}x{F})"
    for t in range(T):
        err = np.max(np.abs(O.widen(a[t]) - Y[t]))
        assert err <= (1e-4 if dtype == "f32" else 2e-2 * np.max(np.abs(Y[t])))


def test_static_entry_point_two_calls_second_smaller():
    import torch
    from paper_2512_03927_amd import binding as B
    from paper_2512_03927_amd import harness as H
    _case(H, B, torch, 520, 1048, 8, 2, 4, "bf16", 51)      # ragged tails, 4 tokens
    _case(H, B, torch, 264, 520, 8, 2, 2, "bf16", 52)       # smaller layer, fewer tokens
    _case(H, B, torch, 128, 264, 6, 3, 2, "f32", 53)        # fp32, k = 3
    # shapes beyond the static scratch are refused before anything is enqueued
    c = B.odmoe_config(64, 40960, 8, 8, 1, 0, B.ODMOE_BF16, 0)
    with pytest.raises(B.OdmoeError) as ei:
        B.odmoe_expert_ffn_static(c, 1, 1, 1, 1, 1, 1, None)
    assert ei.value.code == B.ODMOE_EINVAL and "static scratch" in str(ei.value)
    c = B.odmoe_config(64, 64, 8, 2, 1, 2, B.ODMOE_BF16, 0)
    with pytest.raises(B.OdmoeError) as ei:
        B.odmoe_expert_ffn_static(c, 1, 1, 1, 1, 1, 1, None)
    assert ei.value.code == B.ODMOE_EINVAL
