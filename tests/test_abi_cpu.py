"""The C-ABI library builds, loads and exports everything include/odmoe.h declares (no GPU calls)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADERS = sorted(os.path.join(ROOT, "include", f) for f in os.listdir(os.path.join(ROOT, "include")) if f.endswith(".h"))


def _declared():
    src = "\n".join(open(h).read() for h in HEADERS)
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(odmoe_[a-z_]+)\s*\(", src)))


def test_header_declares_the_five_calls():
    names = _declared()
    for n in ("odmoe_layer_init", "odmoe_route_topk", "odmoe_expert_load_async", "odmoe_expert_ffn",
              "odmoe_decode_step"):
        assert n in names


def test_library_exports_every_declared_symbol():
    from paper_2512_03927_amd import binding as B
    if not os.path.exists(B.LIB_PATH):
        pytest.fail("libodmoe.so is not built: run python -m paper_2512_03927_amd.build")
    lib = B.lib()
    for name in _declared():
        assert hasattr(lib, name), f"{name} is declared in odmoe.h but not exported"
    assert sorted(B.EXPORTS) == _declared()
    assert b"gfx950" in lib.odmoe_version()


def test_struct_layouts_match_header():
    from paper_2512_03927_amd import binding as B
    assert ctypes.sizeof(B.odmoe_config) == 36
    assert ctypes.sizeof(B.odmoe_stats) == 56
    assert B.odmoe_stats.h2d_bytes.offset == 24


def test_argument_errors_need_no_gpu():
    """Validation happens before anything is enqueued, so these return EINVAL on a CPU-only box."""
    from paper_2512_03927_amd import binding as B
    lib = B.lib()
    out = ctypes.c_void_p()
    bad = B.odmoe_config(hidden=100, ffn=64, n_experts=4, top_k=2, n_layers=1, n_slots=0, dtype=0, glue=0,
                         expert_quant=0)
    assert lib.odmoe_layer_init(ctypes.byref(bad), None, None, None, None, None, ctypes.byref(out)) == B.ODMOE_EINVAL
    assert "multiples of 8" in B.odmoe_last_error()
    for kw in (dict(top_k=9), dict(top_k=5), dict(n_slots=1), dict(dtype=7), dict(n_experts=0), dict(n_layers=0),
               dict(glue=2), dict(ffn=1 << 20), dict(expert_quant=3), dict(expert_quant=2, ffn=96), dict(expert_quant=1, hidden=72),
               dict(expert_quant=1, hidden=16384)):
        base = dict(hidden=64, ffn=64, n_experts=4, top_k=2, n_layers=1, n_slots=0, dtype=0, glue=0, expert_quant=0)
        base.update(kw)
        c = B.odmoe_config(**base)
        assert lib.odmoe_layer_init(ctypes.byref(c), None, None, None, None, None, ctypes.byref(out)) == B.ODMOE_EINVAL
        assert out.value is None
    assert lib.odmoe_route_topk(None, 0, None, 1, None, None) == B.ODMOE_EINVAL
    assert lib.odmoe_decode_step(None, None, None, None, None, None) == B.ODMOE_EINVAL
    assert lib.odmoe_layer_destroy(None) == B.ODMOE_OK
    # expert buffer sizes: stored dtype, and int8 codes plus one fp32 scale per weight row
    c = B.odmoe_config(4096, 14336, 8, 2, 1, 0, B.ODMOE_BF16, 0, B.ODMOE_Q_NONE)
    assert B.odmoe_expert_bytes(c) == 3 * 4096 * 14336 * 2 == 352321536
    c.expert_quant = B.ODMOE_Q_INT8_ROW
    assert B.odmoe_expert_bytes(c) == 3 * 4096 * 14336 + 4 * (2 * 14336 + 4096)
    c.expert_quant = B.ODMOE_Q_INT4_G64
    assert B.odmoe_expert_bytes(c) == 3 * 4096 * 14336 // 2 + 4 * (3 * 4096 * 14336 // 64)
    c.expert_quant = B.ODMOE_Q_F16                     # binary16 experts: fp32 layers only
    assert B.odmoe_expert_bytes(c) == 0 and "fp32" in B.odmoe_last_error()
    c.dtype = B.ODMOE_F32
    assert B.odmoe_expert_bytes(c) == 3 * 4096 * 14336 * 2
    c.expert_quant = 4
    assert B.odmoe_expert_bytes(c) == 0
    assert B.odmoe_expert_bytes(bad) == 0
    assert lib.odmoe_quantize(1, 0, 4, 64, 3, None, 1, None, None) == B.ODMOE_EINVAL        # binary16 has no scales
    assert lib.odmoe_quantize(None, 1, 4, 64, 1, None, None, None, None) == B.ODMOE_EINVAL
    assert lib.odmoe_quantize(1, 1, 4, 100, 2, None, None, None, None) == B.ODMOE_EINVAL     # 4-bit groups of 64
    assert lib.odmoe_quantize(1, 1, 4, 64, 7, None, None, None, None) == B.ODMOE_EINVAL


def test_load_window_matches_oracle_and_worked_example():
    """Host-only arithmetic of the library against the oracle's reading of the load-window equation."""
    from oracle import moe_oracle as O
    from paper_2512_03927_amd import binding as B
    for ng, tm, tw in [(4, 1.7, 0.9), (2, 0.01, 0.12), (1, 3.0, 5.0), (6, 0.0, 1.0)]:
        assert abs(B.odmoe_load_window_ms(ng, tm, tw) - O.t_maxload(ng, tm, tw)) < 1e-12
    assert abs(B.odmoe_load_window_ms(4, 1.0, 1.0) - 7.0) < 1e-12        # 4 t^M + 3 t^W
    assert B.odmoe_load_window_ms(0, 1.0, 1.0) == 0.0
    assert B.odmoe_slot_groups(None) == 0


def test_bench_refuses_more_than_one_gpu():
    """The benchmark measures one GPU; asking for more exits with a message (no GPU is touched)."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in (r.stderr + r.stdout)
