"""Emulated SEP predictor on the GPU: a quantised shadow stack supplies the expert hints.

What must hold whatever the weights: hints never change the full stack's output; an identical
copy predicts perfectly; the confirmed fraction equals the recall of Section 3.2 computed by the
oracle from the two index lists; a coarser copy is not better; without alignment recall decays.
"""
import numpy as np
import pytest

from oracle import moe_oracle as O
from paper_2512_03927_amd import shadow, synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def H():
    from paper_2512_03927_amd import harness
    return harness


def test_shadow_stack_hints(H):
    cfg = synth.MoEConfig("t", 256, 512, 8, 2, n_layers=8, n_slots=4, dtype="bf16", n_tokens=1, glue=1, seed=41)
    layers = [synth.layer_weights(cfg, l) for l in range(cfg.n_layers)]
    x0 = H.to_device(synth.tokens(cfg)[0])
    n_iter = 24
    L, k = cfg.n_layers, cfg.top_k
    res_cfg = cfg.small(n_slots=0)
    with H.MoEStack(cfg, layers) as main:
        # reference chain without any hints
        x, base = x0, []
        for _ in range(n_iter):
            x, idx, _ = main.decode(x)
            base.append((H.from_device(x).copy(), idx.copy()))
        rec = {}
        for kind in ("bf16", "int8", "int4"):
            with H.MoEStack(res_cfg, shadow.shadow_layers(cfg, layers, kind)) as sh:
                for aligned in (True, False):
                    r, x_end = shadow.emulate(main, sh, x0, n_iter, aligned)
                    rec[(kind, aligned)] = r
                    # hints change timing only: the main chain ends in the same bits
                    assert np.array_equal(H.from_device(x_end), base[-1][0])
                if kind == "int4":
                    # alignment period: period 1 is the aligned run, a period longer than the run
                    # is the free-running one, and iterations right after a realignment equal the
                    # aligned run's (same input, same weights)
                    assert shadow.emulate(main, sh, x0, n_iter, True, 1)[0] == rec[(kind, True)]
                    assert shadow.emulate(main, sh, x0, n_iter, True, n_iter + 1)[0] == rec[(kind, False)]
                    r4 = shadow.emulate(main, sh, x0, n_iter, True, 4)[0]
                    assert r4[0::4] == rec[(kind, True)][0::4]
                    rec[(kind, 4)] = r4
                # recall bookkeeping against the oracle's definition, first iteration, aligned
                _, idx_s, _ = sh.decode(x0)
                _, idx_m, st = main.decode(x0, pred=idx_s)
                c = np.array([[[O.correct_predictions(idx_s[l], idx_m[l]) for l in range(L)]]])
                assert abs(O.recall(c, np.ones((1, 1)), k) - st.hint_hits / (L * k)) < 1e-12
                assert st.reloads == L * k - st.hint_hits
    assert all(v == 1.0 for v in rec[("bf16", True)]) and all(v == 1.0 for v in rec[("bf16", False)])
    m = {key: float(np.mean(v)) for key, v in rec.items()}
    print("mean recall:", {f"{k_}-{a}": round(v, 3) for (k_, a), v in m.items()})
    assert m[("int8", True)] >= m[("int4", True)] > k / cfg.n_experts
    assert m[("int8", True)] > 0.8
    # without alignment the copy drifts: late iterations are worse than with alignment
    late = slice(n_iter // 2, None)
    assert np.mean(rec[("int4", False)][late]) < np.mean(rec[("int4", True)][late])
    assert rec[("int4", False)][0] == rec[("int4", True)][0]          # first iteration starts aligned
