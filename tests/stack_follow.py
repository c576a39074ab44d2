"""Comparison of a decoded stack of many layers with the CPU oracle, layer by layer, with no
tolerance on the routing and no path that ends without an element-wise check.

The GPU feeds every layer its own stored output.  Its stored state differs from the oracle's in
the last bit of a few elements (both round nearly the same real number to the storage dtype), and
the layer map is far from a contraction here (with N(0, 0.02) weights the expert output is larger
than the residual it is added to), so over tens of layers the two free-running trajectories drift
apart by more than one rounding, and router logits that are close can come out in the other
order.  Both orders are valid results of the method on the respective inputs.  So:

  on_gpu_trajectory   every layer is checked on the input the GPU actually had: the oracle, given
                      the GPU's stored input to layer l, must select exactly the GPU's experts
                      (bit-exact, no near-tie allowance) and reproduce the GPU's stored output of
                      that layer within the one-layer tolerance.  The chain of single-layer GPU
                      steps must equal the stack call's output bit for bit.
  follow_stack        the oracle runs free from the same first input; where its selection differs
                      from the GPU's it continues with the GPU's selection (that selection was
                      shown valid by on_gpu_trajectory); the distance between the two final states
                      is returned for the caller to report and bound.
"""
import numpy as np

from oracle import moe_oracle as O



def on_gpu_trajectory(x0, layers, k: int, dtype: str, gpu_layer_step, rel_tol: float, glue: int = 1):
    """Walks the GPU's own trajectory.  gpu_layer_step(l, x_stored) -> (x_next stored, idx[k]) runs
    layer l alone on the GPU (one token through a one-layer stack).  For every layer the oracle is
    evaluated on the same stored input: routing must be equal, the next state within
    rel_tol * max|ref| (f32: absolute rel_tol).  Returns (final state, list of states, idx[L,k],
    worst error seen)."""
    x = np.asarray(x0)
    xs, IDX, worst = [x], [], 0.0
    for l, (Wg, b, experts) in enumerate(layers):
        x_gpu, idx_gpu = gpu_layer_step(l, x)
        y, idx_o, _ = O.moe_layer(x, Wg, b, experts, k)
        assert np.array_equal(np.asarray(idx_gpu, np.int32), idx_o), \
            f"layer {l}: on its own input the GPU chose {idx_gpu}, the oracle {idx_o}"
        y_st = O.round_to_storage(y, dtype)
        ref = O.widen(O.round_to_storage(O.glue_rmsnorm(x, y_st), dtype) if glue else y_st)
        err = float(np.max(np.abs(O.widen(x_gpu) - ref)))
        scale = float(np.max(np.abs(ref))) if dtype == "bf16" else 1.0
        assert err <= rel_tol * scale, f"layer {l}: error {err} of scale {scale}"
        worst = max(worst, err / scale)
        x = np.asarray(x_gpu)
        xs.append(x)
        IDX.append(np.asarray(idx_gpu, np.int32))
    return x, xs, np.stack(IDX), worst


def follow_stack(x0, layers, k: int, dtype: str, idx_gpu, glue: int = 1):
    """Free-running oracle that takes the GPU's selection wherever its own differs.

    Returns (x_final stored, swaps: layers where the selections differed, states: stored input of
    every layer and the final state)."""
    x = np.asarray(x0)
    swaps, states = [], [x]
    for l, (Wg, b, experts) in enumerate(layers):
        idx_o = O.topk_select(O.router_logits(Wg, b, x), k)
        idx_g = np.asarray(idx_gpu[l], dtype=np.int32)
        if np.array_equal(idx_o, idx_g):
            y, _, _ = O.moe_layer(x, Wg, b, experts, k)
        else:
            swaps.append(l)
            y, _ = O.moe_layer_given_idx(x, Wg, b, experts, idx_g)
        y_st = O.round_to_storage(y, dtype)
        x = O.round_to_storage(O.glue_rmsnorm(x, y_st), dtype) if glue else y_st
        states.append(x)
    return x, swaps, states
