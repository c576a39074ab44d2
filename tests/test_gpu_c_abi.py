"""The C ABI without Python in between: a plain C program (paper_2512_03927_amd/csrc/c_abi_demo.c,
built by `python -m paper_2512_03927_amd.build`) links libodmoe.so, builds a cacheless stack from a
file of synthetic weights, decodes one token with and without hints, and writes the result; this
test writes the file, runs the program and checks its output against the CPU oracle."""
import os
import struct
import subprocess

import numpy as np
import pytest

from oracle import moe_oracle as O
from paper_2512_03927_amd import synth

pytestmark = pytest.mark.gpu

PKG = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2512_03927_amd")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_c_program_decodes_a_cacheless_stack(tmp_path, dtype):
    exe = os.path.join(PKG, "c_abi_demo")
    if not os.path.exists(exe):
        pytest.fail(f"{exe} is missing: build it with `python -m paper_2512_03927_amd.build`")
    cfg = synth.MoEConfig("t", 128, 192, 8, 2, n_layers=4, n_slots=4, dtype=dtype, n_tokens=1, glue=1, seed=29)
    layers = [synth.layer_weights(cfg, l) for l in range(cfg.n_layers)]
    x = synth.tokens(cfg)[0]
    inp, out = tmp_path / "in.bin", tmp_path / "out.bin"
    with open(inp, "wb") as f:
        f.write(struct.pack("<8i", cfg.hidden, cfg.ffn, cfg.n_experts, cfg.top_k, cfg.n_layers, cfg.n_slots,
                            0 if dtype == "f32" else 1, cfg.glue))
        for (Wg, _, experts) in layers:
            f.write(np.ascontiguousarray(Wg).tobytes())
            for e in experts:
                f.write(np.ascontiguousarray(e).tobytes())
        f.write(np.ascontiguousarray(x).tobytes())
    r = subprocess.run([exe, str(inp), str(out)], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stderr
    raw = open(out, "rb").read()
    es = 4 if dtype == "f32" else 2
    y = np.frombuffer(raw[:cfg.hidden * es], dtype=np.float32 if dtype == "f32" else np.uint16)
    off = cfg.hidden * es
    idx = np.frombuffer(raw[off:off + 4 * cfg.n_layers * cfg.top_k], dtype=np.int32).reshape(cfg.n_layers, cfg.top_k)
    loads, hits = struct.unpack("<2Q", raw[off + 4 * cfg.n_layers * cfg.top_k:])
    x_ref, IDX, _ = O.stack_decode(x, [(Wg, None, ex) for (Wg, _, ex) in layers], cfg.top_k, dtype, glue=1)
    assert np.array_equal(idx, IDX)
    assert loads == hits == cfg.n_layers * cfg.top_k
    err = np.max(np.abs(O.widen(y) - O.widen(x_ref)))
    tol = 1e-4 if dtype == "f32" else 2e-2 * np.max(np.abs(O.widen(x_ref)))
    assert err <= tol, err
