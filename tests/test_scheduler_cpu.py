"""Slot pool + decode scheduler driven on the CPU (no copy engine, no GPU).

What the paper fixes (Sections 1, 3.1): no expert survives its use, so a cacheless token
issues exactly L*k loads (+ reloads after wrong predictions); a wrong prediction only costs
a reload; never more than S experts are in HBM.
"""
import ctypes as C
import os

import numpy as np
import pytest

PKG = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2512_03927_amd")
LOAD, DROP, RELEASE = 0, 1, 2


@pytest.fixture(scope="module")
def sim():
    path = os.path.join(PKG, "libodmoe_hostsim.so")
    if not os.path.exists(path):
        pytest.fail("libodmoe_hostsim.so is not built: run python -m paper_2512_03927_amd.build")
    lib = C.CDLL(path)
    lib.odmoe_sim_new.restype = C.c_void_p
    lib.odmoe_sim_new.argtypes = [C.c_int] * 4
    for n in ("odmoe_sim_del", "odmoe_sim_begin", "odmoe_sim_before_route", "odmoe_sim_after_route",
              "odmoe_sim_after_compute", "odmoe_sim_counters", "odmoe_sim_n_free", "odmoe_sim_pool_acquire",
              "odmoe_sim_pool_find", "odmoe_sim_pool_release", "odmoe_sim_pool_release_all"):
        getattr(lib, n).argtypes = None
    return lib


def _p(a):
    return a.ctypes.data_as(C.c_void_p)


def run_token(lib, L, E, k, S, actual, pred=None):
    """Drives one token; returns (actions, counters) and checks the invariants on the way."""
    h = C.c_void_p(lib.odmoe_sim_new(L, E, k, S))
    buf = np.zeros(4 * 4 * (L * k + S + 8), dtype=np.int32)
    predp = None if pred is None else _p(pred)
    lib.odmoe_sim_begin(h, predp)
    resident = {}          # slot -> (layer, expert)
    log = []

    def apply(n):
        assert n >= 0
        for a in buf[:4 * n].reshape(n, 4):
            kind, layer, expert, slot = (int(v) for v in a)
            log.append((kind, layer, expert, slot))
            if kind == LOAD:
                assert slot not in resident, "load into an occupied slot"
                assert (layer, expert) not in resident.values(), "expert loaded twice"
                resident[slot] = (layer, expert)
            else:
                assert resident.pop(slot) == (layer, expert)
            assert len(resident) <= S
        assert lib.odmoe_sim_n_free(h) + len(resident) == S      # after the whole batch

    for l in range(L):
        apply(lib.odmoe_sim_before_route(h, l, _p(buf), len(buf)))
        slots = np.full(k, -1, dtype=np.int32)
        apply(lib.odmoe_sim_after_route(h, l, _p(actual[l]), _p(slots), _p(buf), len(buf)))
        for i in range(k):                       # every chosen expert is in the slot reported for it
            assert resident[int(slots[i])] == (l, int(actual[l, i]))
        assert all(lay >= l for (lay, _) in resident.values()), "an expert outlived its layer"
        assert sum(1 for (lay, _) in resident.values() if lay == l) == k, "unused expert of this layer kept"
        apply(lib.odmoe_sim_after_compute(h, l, _p(actual[l]), _p(buf), len(buf)))
        assert all(lay > l for (lay, _) in resident.values()), "expert not evicted after use"
    assert not resident and lib.odmoe_sim_n_free(h) == S
    loads, reloads, hits = C.c_uint64(), C.c_uint64(), C.c_uint64()
    lib.odmoe_sim_counters(h, C.byref(loads), C.byref(reloads), C.byref(hits))
    lib.odmoe_sim_del(h)
    return log, (loads.value, reloads.value, hits.value)


def _routes(L, E, k, seed):
    r = np.random.default_rng(seed)
    return np.stack([r.permutation(E)[:k] for _ in range(L)]).astype(np.int32)


@pytest.mark.parametrize("L,E,k,S", [(32, 8, 2, 4), (24, 64, 6, 12), (5, 8, 2, 2), (7, 8, 3, 7), (1, 4, 4, 4)])
def test_no_hints_every_activation_is_a_load(sim, L, E, k, S):
    actual = _routes(L, E, k, 0)
    log, (loads, reloads, hits) = run_token(sim, L, E, k, S, actual)
    assert loads == L * k and reloads == 0 and hits == 0
    assert sum(1 for a in log if a[0] == LOAD) == L * k
    assert sum(1 for a in log if a[0] == RELEASE) == L * k
    # the same expert chosen by consecutive layers (or tokens) is still loaded again: no cache
    same = np.tile(np.arange(k, dtype=np.int32), (L, 1))
    _, (loads2, _, _) = run_token(sim, L, E, k, S, same)
    assert loads2 == L * k


@pytest.mark.parametrize("L,E,k,S", [(32, 8, 2, 4), (24, 64, 6, 12), (9, 8, 2, 5), (6, 8, 2, 2)])
def test_perfect_hints_prefetch_ahead_and_never_reload(sim, L, E, k, S):
    actual = _routes(L, E, k, 1)
    log, (loads, reloads, hits) = run_token(sim, L, E, k, S, actual, pred=actual.copy())
    assert loads == L * k and reloads == 0 and hits == L * k
    # look-ahead: when layer 0 is routed, floor(S/k) layers' experts are already on their way
    first_route = [i for i, a in enumerate(log) if a[0] == RELEASE][0]
    ahead_layers = {a[1] for a in log[:first_route] if a[0] == LOAD}
    assert ahead_layers == set(range(min(L, S // k)))


def test_wrong_hints_cost_reloads_only(sim):
    L, E, k, S = 16, 8, 2, 4
    actual = _routes(L, E, k, 2)
    pred = actual.copy()
    pred[3] = [(actual[3, 0] + 1) % E if (actual[3, 0] + 1) % E not in actual[3] else (actual[3, 0] + 2) % E,
               actual[3, 1]]                                   # one of two wrong in layer 3
    wrong7 = [e for e in range(E) if e not in actual[7]][:2]
    pred[7] = wrong7                                           # both wrong in layer 7
    pred[9] = [-1, 99]                                         # unusable hints
    pred[11] = [actual[11, 1], actual[11, 0]]                  # right set, other order
    log, (loads, reloads, hits) = run_token(sim, L, E, k, S, actual, pred=pred)
    assert reloads == 1 + 2 + 2
    assert hits == L * k - 5
    assert loads == L * k + 1 + 2                              # the unusable hints were never loaded
    assert sum(1 for a in log if a[0] == DROP) == 3


def test_random_hints_hit_rate_is_k_over_E(sim):
    """Random prefetching confirms about k/E of the activations (the paper quotes about 25% for 2 of 8)."""
    L, E, k, S = 32, 8, 2, 4
    hits_total = 0
    n_tok = 60
    for t in range(n_tok):
        actual = _routes(L, E, k, 100 + t)
        pred = _routes(L, E, k, 9000 + t)
        _, (loads, reloads, hits) = run_token(sim, L, E, k, S, actual, pred=pred)
        assert loads == L * k + reloads and hits + reloads == L * k
        hits_total += hits
    assert abs(hits_total / (n_tok * L * k) - k / E) < 0.03


def test_slot_pool_fifo_and_errors(sim):
    h = C.c_void_p(sim.odmoe_sim_new(1, 8, 2, 3))
    assert [sim.odmoe_sim_pool_acquire(h, 0, e) for e in range(4)] == [0, 1, 2, -1]
    assert sim.odmoe_sim_pool_find(h, 0, 1) == 1 and sim.odmoe_sim_pool_find(h, 1, 1) == -1
    assert sim.odmoe_sim_pool_release(h, 1) == 0 and sim.odmoe_sim_pool_release(h, 1) == -1
    assert sim.odmoe_sim_pool_release(h, 0) == 0
    # oldest-released slot is reused first
    assert sim.odmoe_sim_pool_acquire(h, 0, 5) == 1 and sim.odmoe_sim_pool_acquire(h, 0, 6) == 0
    assert sim.odmoe_sim_pool_release(h, 7) == -1
    sim.odmoe_sim_del(h)


def test_recovery_after_a_token_that_failed_part_way(sim):
    """What the library does when a decode step fails between layers: every slot is given back,
    whatever held it (hinted experts of later layers, the failing layer's own), and the next token
    runs as on a fresh handle."""
    L, E, k, S = 8, 8, 2, 6
    actual = _routes(L, E, k, 5)
    h = C.c_void_p(sim.odmoe_sim_new(L, E, k, S))
    buf = np.zeros(4 * 64, dtype=np.int32)
    sim.odmoe_sim_begin(h, _p(actual))
    assert sim.odmoe_sim_before_route(h, 0, _p(buf), len(buf)) == S       # three layers' experts hinted ahead
    slots = np.full(k, -1, dtype=np.int32)
    sim.odmoe_sim_after_route(h, 0, _p(actual[0]), _p(slots), _p(buf), len(buf))
    assert sim.odmoe_sim_n_free(h) == 0                                    # ... the token "fails" here
    sim.odmoe_sim_pool_release_all(h)
    assert sim.odmoe_sim_n_free(h) == S
    assert all(sim.odmoe_sim_pool_find(h, l, int(e)) == -1 for l in range(L) for e in range(E))
    sim.odmoe_sim_pool_release_all(h)                                      # idempotent
    assert sim.odmoe_sim_n_free(h) == S
    # the next token on the same pool behaves as on a fresh one
    sim.odmoe_sim_begin(h, None)
    for l in range(L):
        assert sim.odmoe_sim_before_route(h, l, _p(buf), len(buf)) == 0
        assert sim.odmoe_sim_after_route(h, l, _p(actual[l]), _p(slots), _p(buf), len(buf)) == k
        assert sim.odmoe_sim_after_compute(h, l, _p(actual[l]), _p(buf), len(buf)) == k
    loads, reloads, hits = C.c_uint64(), C.c_uint64(), C.c_uint64()
    sim.odmoe_sim_counters(h, C.byref(loads), C.byref(reloads), C.byref(hits))
    assert (loads.value, reloads.value, hits.value) == (L * k, 0, 0) and sim.odmoe_sim_n_free(h) == S
    sim.odmoe_sim_del(h)


def test_any_hints_keep_the_invariants():
    """Property test: whatever the hints hold (right, wrong, duplicated, out of range), the
    invariants checked in run_token hold, every load is either used or dropped, and nothing is
    counted twice."""
    from hypothesis import given, settings, strategies as st

    path = os.path.join(PKG, "libodmoe_hostsim.so")
    lib = C.CDLL(path)
    lib.odmoe_sim_new.restype = C.c_void_p
    lib.odmoe_sim_new.argtypes = [C.c_int] * 4

    @st.composite
    def case(draw):
        E = draw(st.integers(1, 12))
        k = draw(st.integers(1, min(E, 4)))
        S = draw(st.integers(k, 4 * k))
        L = draw(st.integers(1, 9))
        seed = draw(st.integers(0, 2 ** 31 - 1))
        mode = draw(st.sampled_from(["perfect", "noisy", "garbage"]))
        return L, E, k, S, seed, mode

    @settings(max_examples=300, deadline=None)
    @given(case())
    def check(c):
        L, E, k, S, seed, mode = c
        r = np.random.default_rng(seed)
        actual = np.stack([r.permutation(E)[:k] for _ in range(L)]).astype(np.int32)
        pred = actual.copy()
        if mode == "noisy":
            mask = r.random(pred.shape) < 0.4
            pred[mask] = r.integers(0, E, size=int(mask.sum()))          # may duplicate within a layer
        elif mode == "garbage":
            pred = r.integers(-3, E + 3, size=pred.shape).astype(np.int32)
        log, (loads, reloads, hits) = run_token(lib, L, E, k, S, actual, np.ascontiguousarray(pred))
        drops = sum(1 for a in log if a[0] == DROP)
        releases = sum(1 for a in log if a[0] == RELEASE)
        assert releases == L * k and loads - drops == L * k
        assert hits + reloads <= L * k and reloads <= loads
        if mode == "perfect":
            assert drops == 0 and reloads == 0 and loads == L * k
            if S >= 2 * k:
                assert hits == L * k

    check()
