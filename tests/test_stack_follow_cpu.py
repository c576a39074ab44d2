"""The stack-comparison helpers of the GPU tests, exercised on the CPU with the oracle standing in
for the GPU's per-layer step: they must accept an exact trajectory, follow a supplied selection,
and reject a wrong routing or a wrong state."""
import numpy as np
import pytest

from oracle import moe_oracle as O
from paper_2512_03927_amd import synth

from stack_follow import follow_stack, on_gpu_trajectory


def _stack(dtype="bf16", L=5):
    cfg = synth.MoEConfig("t", 64, 128, 8, 2, n_layers=L, dtype=dtype, glue=1, seed=3)
    return cfg, [synth.layer_weights(cfg, l) for l in range(L)], synth.tokens(cfg)[0]


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_exact_trajectory_is_accepted_and_reproduced(dtype):
    cfg, layers, x0 = _stack(dtype)
    x_ref, IDX, xs = O.stack_decode(x0, layers, 2, dtype, glue=1)

    def step(l, x):
        xn, idx, _ = O.stack_decode(x, [layers[l]], 2, dtype, glue=1)
        return xn, idx[0]

    x_end, states, idx, worst = on_gpu_trajectory(x0, layers, 2, dtype, step, 2e-2 if dtype == "bf16" else 1e-4)
    assert np.array_equal(x_end, x_ref) and np.array_equal(idx, IDX) and worst == 0.0
    assert all(np.array_equal(a, b) for a, b in zip(states, xs))
    x_f, swaps, st = follow_stack(x0, layers, 2, dtype, IDX)
    assert np.array_equal(x_f, x_ref) and swaps == [] and len(st) == len(layers) + 1


def test_wrong_routing_or_state_is_rejected_and_a_supplied_selection_is_followed():
    cfg, layers, x0 = _stack()
    _, IDX, _ = O.stack_decode(x0, layers, 2, "bf16", glue=1)

    def wrong_idx(l, x):
        xn, idx, _ = O.stack_decode(x, [layers[l]], 2, "bf16", glue=1)
        return xn, (idx[0][::-1].copy() if l == 2 else idx[0])      # layer 2 reports the other order

    with pytest.raises(AssertionError, match="layer 2"):
        on_gpu_trajectory(x0, layers, 2, "bf16", wrong_idx, 2e-2)

    def wrong_state(l, x):
        xn, idx, _ = O.stack_decode(x, [layers[l]], 2, "bf16", glue=1)
        if l == 3:
            xn = xn.copy()
            xn[5] ^= np.uint16(0x0400)                                # a large error in one element
        return xn, idx[0]

    with pytest.raises(AssertionError, match="layer 3"):
        on_gpu_trajectory(x0, layers, 2, "bf16", wrong_state, 2e-2)

    other = IDX.copy()
    other[1] = [e for e in range(8) if e not in IDX[1]][:2]         # another selection at layer 1
    x_f, swaps, states = follow_stack(x0, layers, 2, "bf16", other)
    assert swaps[0] == 1
    # the state after layer 1 is that layer evaluated by hand with the supplied selection
    Wg, b, ex = layers[1]
    y, _ = O.moe_layer_given_idx(states[1], Wg, b, ex, other[1])
    x2 = O.round_to_storage(O.glue_rmsnorm(states[1], O.round_to_storage(y, "bf16")), "bf16")
    assert np.array_equal(states[2], x2) and np.array_equal(states[-1], x_f)
