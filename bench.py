#!/usr/bin/env python3
"""Benchmark of the cacheless MoE decode layer on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

Workload (default): the single Mixtral-shaped MoE layer in bf16 with all 8 experts
resident in HBM, batch-1 decode of 256 synthetic tokens, one token at a time.  One
"step" = the 256 tokens of that batch, each through router GEMV -> top-2 gate -> w1/w3
GEMV + SiLU -> w2 GEMV + weighted combine.  `value` = tokens/s with weights and
activations already in HBM when the timed region starts.

Also reported on the same JSON line:
  roofline      the dominant kernel (w1/w3 GEMV + SiLU) against the HBM peak, timed with
                HIP events on the compute stream in a second pass over the same tokens
                (the kernel launched back to back for all 256 tokens between two events)
  cacheless     the 32-layer cacheless stack (experts in pinned host memory, 4 HBM slots):
                H2D expert-load GB/s, tokens/s, step / max(compute, load)
  sep_emulation the quantised shadow model's side: int8 experts on the same layer (tokens/s,
                GEMV GB/s) and the recall an int8 / 4-bit copy gives as the predictor
  cpu_baseline  the float64 NumPy oracle on a bounded sample of the same tokens
"""
from __future__ import annotations

import argparse
import contextlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E bandwidth
PCIE5_X16_GBPS = 64.0           # host link, raw per direction


def log(*a):
    print(*a, file=sys.stderr, flush=True)


# hidden, ffn, experts held resident here (not the model's count where that is large), top_k, dtype
SWEEP_SHAPES = [
    (4096, 14336, 8, 2, "bf16"),    # Mixtral-8x7B layer (benchmark config 2)
    (4096, 14336, 8, 2, "f32"),     # the same in fp32 (the paper's full precision)
    (6144, 16384, 8, 2, "bf16"),
    (8192, 8192, 8, 2, "bf16"),
    (7168, 2048, 32, 8, "bf16"),    # many small experts on a wide hidden state
    (5120, 1536, 32, 6, "bf16"),
    (3072, 8192, 16, 2, "bf16"),
    (2048, 8192, 8, 2, "bf16"),
    (2048, 1408, 64, 6, "bf16"),    # fine-grained layer (benchmark config 5)
    (2048, 1408, 64, 6, "f32"),
    (2048, 768, 128, 8, "bf16"),
    (1024, 4096, 16, 2, "bf16"),
    (1024, 4096, 16, 2, "f32"),
]


def shape_sweep(sel) -> int:
    """Decode-kernel timings over a range of MoE layer shapes: for each one a synthetic layer is made
    resident and the router, w1/w3 GEMV and w2 GEMV are timed with HIP events (each kernel launched
    back to back for 32 tokens); GB/s = algorithmic bytes of the k chosen experts over the kernel
    time.  The launch policies of the two GEMVs were chosen from this table."""
    from paper_2512_03927_amd import binding as B
    from paper_2512_03927_amd import harness, synth
    n_tok = 32
    for si in (sel or range(len(SWEEP_SHAPES))):
        hd, f, e, k, dt = SWEEP_SHAPES[si]
        cfg = synth.MoEConfig(f"sweep{si}", hd, f, e, k, dtype=dt, n_tokens=n_tok, seed=100 + si)
        layer = synth.layer_weights(cfg, 0)
        with harness.MoEStack(cfg, [layer]) as st:
            x = harness.to_device(synth.tokens(cfg, n_tok))
            # the GPU idled while the host generated the layer: about 60 ms of the same kernels bring
            # it back to its working clocks before anything is recorded
            warm_us = 0.0
            while warm_us < 60e3:
                r, u, d = B.odmoe_time_decode_kernels(st.handle, 0, x, n_tok, 4)
                warm_us += (r + u + d) * n_tok * 4
            best = None
            for _ in range(3):
                r, u, d = B.odmoe_time_decode_kernels(st.handle, 0, x, n_tok, 4)
                if best is None or u + d < best[1] + best[2]:
                    best = (r, u, d)
        r, u, d = best
        es = 4 if dt == "f32" else 2
        up_b, down_b = k * 2 * hd * f * es, k * hd * f * es
        print(f"{dt:4s} H{hd:<5d} F{f:<6d} E{e:<4d} k{k}: route {r:6.2f} us | w1/w3 {u:7.2f} us "
              f"{up_b / u / 1e3:5.0f} GB/s | w2 {d:7.2f} us {down_b / d / 1e3:5.0f} GB/s", flush=True)
        del layer
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--tokens", type=int, default=None, help="tokens per step (default: the workload's 256)")
    ap.add_argument("--cacheless-tokens", type=int, default=32,
                    help="tokens of the 32-layer cacheless stack to time (0 = skip; the workload states 128)")
    ap.add_argument("--arena-layers", type=int, default=8,
                    help="unique layers in the pinned host arena of the 32-layer stack (layer l uses l mod U)")
    ap.add_argument("--shape-sweep", nargs="*", type=int, default=None, metavar="I",
                    help="instead of the benchmark: time the decode kernels over a list of MoE layer shapes "
                         "(all of them, or the given positions) and print one line per shape")
    ap.add_argument("--cpu-tokens", type=int, default=40, help="tokens the CPU oracle is timed on (0 = skip)")
    ap.add_argument("--prefill-iters", type=int, default=5, help="timed prefill calls of 512 tokens (0 = skip)")
    ap.add_argument("--probe-mib", type=int, default=672,
                    help="size of the plain read/copy probe that measures the HBM and host-link ceilings (0 = skip)")
    ap.add_argument("--sep-iters", type=int, default=32,
                    help="emulated decode iterations with a quantised shadow stack supplying hints (0 = skip)")
    ap.add_argument("--int8-passes", type=int, default=3,
                    help="timed passes over the tokens with the layer's experts held as int8 / 4-bit codes (0 = skip)")
    ap.add_argument("--no-prefill-from-host", action="store_true",
                    help="skip the prefill run that streams the experts from host memory")
    ap.add_argument("--no-kernel-pass", action="store_true", help="skip the HIP-event pass (for profilers)")
    ap.add_argument("--fp32-tokens", type=int, default=64,
                    help="tokens of the same layer held in fp32, the paper's full precision (0 = skip)")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on ONE GPU only (no sharding, no collectives); "
            f"--gpus {args.gpus} is not supported.")
        return 2

    import numpy as np
    import torch
    from paper_2512_03927_amd import binding as B
    from paper_2512_03927_amd import harness, synth

    if not torch.cuda.is_available():
        log("bench.py: no GPU visible")
        return 3
    B.lib()  # fails loudly if the HIP library is not built
    if args.shape_sweep is not None:
        return shape_sweep(args.shape_sweep)
    mem_total_gb = mem_avail_gb = None
    try:
        mi = dict(l.split(":") for l in open("/proc/meminfo").read().splitlines() if ":" in l)
        mem_total_gb = int(mi["MemTotal"].split()[0]) / 1e6
        mem_avail_gb = int(mi["MemAvailable"].split()[0]) / 1e6
        log(f"[bench] host memory: {mem_total_gb:.0f} GB total, {mem_avail_gb:.0f} GB available")
    except Exception:
        pass

    cfg = synth.CONFIGS[2]
    T = args.tokens or cfg.n_tokens
    t0 = time.time()
    layer = synth.layer_weights(cfg, 0)
    X_np = synth.tokens(cfg, T)
    log(f"[bench] generated {cfg.name}: 8 experts x {cfg.expert_bytes / 1e6:.1f} MB in {time.time() - t0:.1f} s")

    # ---- measured ceilings: a plain streaming read of HBM, a plain pinned host->HBM copy
    ceilings = None
    if args.probe_mib > 0:
        nb = args.probe_mib << 20
        src = torch.empty(4 * nb, dtype=torch.uint8, device="cuda:0").fill_(1)     # 4 windows, rotated
        dst = torch.empty(nb, dtype=torch.uint8, device="cuda:0")
        cur = torch.cuda.current_stream().cuda_stream
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        res = {}
        for mode, name in ((1, "hbm_read_GBps"), (0, "hbm_copy_GBps")):
            for w in range(2):
                B.odmoe_probe_hbm(dst, src[w * nb:], nb, mode, cur)
            torch.cuda.synchronize()
            ev0.record()
            for w in range(8):
                B.odmoe_probe_hbm(dst, src[(w % 4) * nb:], nb, mode, cur)
            ev1.record()
            torch.cuda.synchronize()
            res[name] = round(nb * 8 / (ev0.elapsed_time(ev1) * 1e-3) / 1e9 * (2 if mode == 0 else 1), 1)
        host = torch.empty(nb, dtype=torch.uint8, pin_memory=True)
        dst.copy_(host, non_blocking=True)
        torch.cuda.synchronize()
        ev0.record()
        for _ in range(4):
            dst.copy_(host, non_blocking=True)
        ev1.record()
        torch.cuda.synchronize()
        res["h2d_pinned_GBps"] = round(nb * 4 / (ev0.elapsed_time(ev1) * 1e-3) / 1e9, 2)
        res["probe_MiB"] = args.probe_mib
        ceilings = res
        del src, dst, host
        log(f"[bench] measured ceilings: {ceilings}")

    stack = harness.MoEStack(cfg, [layer])
    X = harness.to_device(X_np)
    Y = torch.empty_like(X)
    h = stack.handle

    def step():
        for t in range(T):
            B.odmoe_decode_step(h, X[t], Y[t], None, None, None)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start
    ms_per_step = elapsed / args.steps * 1e3
    tokens_per_s = T * args.steps / elapsed
    log(f"[bench] {args.steps} steps x {T} tokens: {ms_per_step:.3f} ms/step, {tokens_per_s:.1f} tokens/s")

    # ---- second pass over the same steps with HIP events around each kernel (compute stream)
    up_bytes = cfg.top_k * 2 * cfg.hidden * cfg.ffn * 2      # w1 + w3 of the k experts, bf16
    down_bytes = cfg.top_k * cfg.hidden * cfg.ffn * 2        # w2 of the k experts
    roofline = None
    gemv_gbps = None
    route_ms_resident = 0.006
    if not args.no_kernel_pass:
        # each kernel launched back to back for the same 256 tokens, HIP events around each pass
        route_us, up_us, down_us = B.odmoe_time_decode_kernels(h, 0, X, T, max(1, min(args.steps, 4)))
        up_ms, down_ms, route_ms = up_us * 1e-3, down_us * 1e-3, route_us * 1e-3
        route_ms_resident = route_ms
        achieved = up_bytes / (up_ms * 1e-3) / 1e9
        gemv_gbps = (up_bytes + down_bytes) / ((up_ms + down_ms) * 1e-3) / 1e9
        traffic = traffic_src = None
        tpath = os.path.join(ROOT, "profiles", "hbm_traffic_cfg2.json")
        if os.path.exists(tpath):               # a stored figure: counters cannot be read from inside this process
            tj = json.load(open(tpath))
            traffic = tj.get("ffn_up_kernel_bytes_per_launch")
            traffic_src = "stored: profiles/hbm_traffic_cfg2.json (rocprofv3 --pmc FETCH_SIZE, scaled by the read probe" + \
                          (f"; taken at commit {tj['commit']})" if tj.get("commit") else ")")
        roofline = {"bound": "hbm", "kernel": "ffn_up_reg_kernel<unsigned short, 8, true> (w1/w3 GEMV + SiLU, bf16)",
                    "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                    "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic, "traffic_source": traffic_src,
                    "algorithmic_bytes_per_launch": up_bytes, "avg_launch_us": round(up_ms * 1e3, 2),
                    "ffn_down_us": round(down_ms * 1e3, 2), "route_us": round(route_ms * 1e3, 2),
                    "ffn_down_GBps": round(down_bytes / (down_ms * 1e-3) / 1e9, 1)}
        log(f"[bench] kernels: up {up_ms * 1e3:.1f} us ({achieved:.0f} GB/s), down {down_ms * 1e3:.1f} us, "
            f"route {route_ms * 1e3:.1f} us")
    Y_keep = harness.from_device(Y[:max(4, args.cpu_tokens)]).copy()
    stack.close()

    # ---- prefill: 512 tokens in one call, skewed routing, grouped GEMM on the matrix cores
    prefill = None
    if args.prefill_iters > 0:
        c4 = synth.CONFIGS[4]
        Wg4, _, experts4 = layer
        b4 = synth.router_bias(c4)
        X4 = harness.to_device(synth.tokens(c4))
        with harness.MoEStack(c4, [(Wg4, b4, experts4)]) as st4:
            idx4, gate4 = st4.route(0, X4)
            Y4 = torch.empty_like(X4)
            counts = np.bincount(idx4.cpu().numpy().ravel(), minlength=c4.n_experts)

            def prefill_once():
                B.odmoe_route_topk(st4.handle, 0, X4, c4.n_tokens, idx4, gate4)
                B.odmoe_expert_ffn(st4.handle, 0, idx4, gate4, None, X4, c4.n_tokens, Y4, 0)

            # warm-up: the GPU idled while the host made the inputs and takes some tens of milliseconds
            # of work to return to its working clocks (batches right after idling: 0.83, 0.75, 0.70 ms)
            for _ in range(80):
                prefill_once()
            torch.cuda.synchronize()
            batches = []
            for _ in range(3):                       # three timed batches of prefill_iters calls; the median counts
                ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                ev0.record()
                for _ in range(args.prefill_iters):
                    prefill_once()
                ev1.record()
                torch.cuda.synchronize()
                batches.append(ev0.elapsed_time(ev1) / args.prefill_iters)
            ms = float(np.median(batches))
        flops = 6.0 * c4.n_tokens * c4.top_k * c4.hidden * c4.ffn
        wbytes = float(np.count_nonzero(counts)) * c4.expert_bytes
        # per-expert bound: weights once from HBM vs that expert's GEMM flops on the matrix cores
        ideal_ms = sum(max(c4.expert_bytes / (HBM_PEAK_GBPS * 1e9),
                           6.0 * n * c4.hidden * c4.ffn / 2.5e15) for n in counts if n > 0) * 1e3
        prefill = {"workload": c4.name, "tokens": c4.n_tokens, "ms": round(ms, 4),
                   "tokens_per_s": round(c4.n_tokens / (ms * 1e-3), 1),
                   "tflops": round(flops / (ms * 1e-3) / 1e12, 1), "mfma_frac_of_2500": round(flops / (ms * 1e-3) / 2.5e15, 4),
                   "weight_GBps": round(wbytes / (ms * 1e-3) / 1e9, 1),
                   "roofline_ms_sum_max_hbm_mfma": round(ideal_ms, 4), "frac_of_roofline": round(ideal_ms / ms, 4),
                   "ms_batches": [round(b, 4) for b in batches], "tokens_per_expert": counts.tolist()}
        # the same batch with the experts in pinned host memory and 4 HBM slots (Section 3.3 on one GPU:
        # every expert is streamed in once; its GEMMs overlap the next expert's copy)
        c4h = c4.small(n_slots=4)
        if args.no_prefill_from_host:
            c4h = None
        with (harness.MoEStack(c4h, [(Wg4, b4, experts4)]) if c4h else contextlib.nullcontext()) as st4h:
          if c4h:
            idx4h, gate4h = st4h.route(0, X4)
            ih = idx4h.cpu().numpy()
            Y4h = torch.empty_like(X4)
            B.odmoe_expert_ffn(st4h.handle, 0, idx4h, gate4h, ih, X4, c4.n_tokens, Y4h, 1)
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            for _ in range(2):
                B.odmoe_expert_ffn(st4h.handle, 0, idx4h, gate4h, ih, X4, c4.n_tokens, Y4h, 1)
            torch.cuda.synchronize()
            ms_h = (time.perf_counter() - t1) / 2 * 1e3
            same = bool(torch.equal(Y4h, Y4))
            prefill["from_host"] = {"ms": round(ms_h, 3), "h2d_GBps": round(wbytes / (ms_h * 1e-3) / 1e9, 2),
                                    "n_slots": 4, "experts_loaded": int(np.count_nonzero(counts)),
                                    "bit_identical_to_resident": same}
        log(f"[bench] prefill: {prefill}")

    # ---- the same layer shape in fp32 (the paper's "full precision"): twice the bytes per token
    fp32 = None
    if args.fp32_tokens > 0:
        c32 = cfg.small(name="cfg2-shape-fp32-resident", dtype="f32")
        t0 = time.time()
        layer32 = synth.layer_weights(c32, 0)
        X32_np = synth.tokens(c32, args.fp32_tokens)
        log(f"[bench] generated {c32.name} in {time.time() - t0:.1f} s")
        with harness.MoEStack(c32, [layer32]) as st32:
            X32 = harness.to_device(X32_np)
            Y32 = torch.empty_like(X32)
            for t in range(max(8, 256)):                  # warm-up (the GPU idled during weight generation)
                B.odmoe_decode_step(st32.handle, X32[t % args.fp32_tokens], Y32[t % args.fp32_tokens], None, None, None)
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            for t in range(args.fp32_tokens):
                B.odmoe_decode_step(st32.handle, X32[t], Y32[t], None, None, None)
            torch.cuda.synchronize()
            el32 = time.perf_counter() - t1
            r_us, u_us, d_us = B.odmoe_time_decode_kernels(st32.handle, 0, X32, args.fp32_tokens, 2)
            # prefill of 512 tokens in fp32: grouped GEMMs on the fp32 matrix instructions
            pf32 = None
            if args.prefill_iters > 0:
                Tp = 512
                Xp_np = synth.tokens(c32, Tp)
                Xp = harness.to_device(Xp_np)
                idx_p, gate_p = st32.route(0, Xp)
                Yp = torch.empty_like(Xp)
                B.odmoe_expert_ffn(st32.handle, 0, idx_p, gate_p, None, Xp, Tp, Yp, 0)
                torch.cuda.synchronize()
                tp = []
                for _ in range(args.prefill_iters):
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record()
                    B.odmoe_expert_ffn(st32.handle, 0, idx_p, gate_p, None, Xp, Tp, Yp, 0)
                    e1.record()
                    torch.cuda.synchronize()
                    tp.append(e0.elapsed_time(e1))
                ms_p = float(np.median(tp))
                flop_p = 6.0 * c32.hidden * c32.ffn * Tp * c32.top_k
                pf32 = {"tokens": Tp, "ms": round(ms_p, 3), "TFLOPs": round(flop_p / ms_p / 1e9, 1),
                        "frac_of_fp32_matrix_peak_157.3": round(flop_p / ms_p / 1e9 / 157.3, 3)}
        # the same fp32 layer with its experts held in binary16 (the paper's FP16 shadow model of
        # Sections 1, 3.2: half the bytes per token)
        f16 = None
        if args.int8_passes > 0:
            from paper_2512_03927_amd import shadow
            with shadow.shadow_stack(c32, [layer32], "fp16") as sth:
                Xh = harness.to_device(X32_np)
                Yh = torch.empty_like(Xh)
                for t in range(256):
                    B.odmoe_decode_step(sth.handle, Xh[t % args.fp32_tokens], Yh[t % args.fp32_tokens], None, None, None)
                torch.cuda.synchronize()
                t1 = time.perf_counter()
                for t in range(args.fp32_tokens):
                    B.odmoe_decode_step(sth.handle, Xh[t], Yh[t], None, None, None)
                torch.cuda.synchronize()
                elh = time.perf_counter() - t1
                rh, uh, dh = B.odmoe_time_decode_kernels(sth.handle, 0, Xh, args.fp32_tokens, 2)
                ubh = c32.top_k * 2 * c32.hidden * c32.ffn * 2
                f16 = {"workload": c32.name + " with binary16 experts", "tokens_per_s": round(args.fp32_tokens / elh, 1),
                       "speedup_over_fp32": round(el32 / elh, 3), "bytes_vs_fp32": 0.5,
                       "ffn_up_us": round(uh, 2), "ffn_up_GBps": round(ubh / uh / 1e3, 1),
                       "ffn_up_frac_of_hbm_peak": round(ubh / uh / 1e3 / HBM_PEAK_GBPS, 4),
                       "ffn_down_us": round(dh, 2), "ffn_down_GBps": round(ubh / 2 / dh / 1e3, 1),
                       "ffn_down_frac_of_hbm_peak": round(ubh / 2 / dh / 1e3 / HBM_PEAK_GBPS, 4)}
                del Xh, Yh
        ub32 = c32.top_k * 2 * c32.hidden * c32.ffn * 4
        fp32 = {"workload": c32.name, "tokens": args.fp32_tokens,
                "tokens_per_s": round(args.fp32_tokens / el32, 1),
                "ffn_up_us": round(u_us, 2), "ffn_up_GBps": round(ub32 / u_us / 1e3, 1),
                "ffn_down_us": round(d_us, 2), "ffn_down_GBps": round(ub32 / 2 / d_us / 1e3, 1),
                "route_us": round(r_us, 2), "prefill": pf32, "binary16_experts": f16}
        del layer32
        log(f"[bench] fp32: {fp32}")

    # ---- cacheless stacks, short runs (host-link roofline)
    def run_cacheless(c, layers_u, n_tok, x_rows):
        t0 = time.time()
        stc = harness.MoEStack(c, layers_u, unique_layers=len(layers_u))
        log(f"[bench] {c.name}: pinned arena of {len(layers_u)} unique layer(s) ready in {time.time() - t0:.1f} s")
        xs = [harness.to_device(r) for r in x_rows]
        yc = torch.empty_like(xs[0])
        s = B.odmoe_stats()
        for _ in range(min(8, max(2, n_tok // 3))):                       # warm-up tokens (not timed)
            B.odmoe_decode_step(stc.handle, xs[0], yc, None, None, s)
        torch.cuda.synchronize()
        yc_first = yc.clone()
        t_start = time.perf_counter()
        loads = 0
        per_token = []
        t_prev = t_start
        for t in range(n_tok):
            B.odmoe_decode_step(stc.handle, xs[t % len(xs)], yc, None, None, s)
            loads += s.loads
            t_now = time.perf_counter()                                  # the step waits for every layer's ids
            per_token.append((t_now - t_prev) * 1e3)
            t_prev = t_now
        torch.cuda.synchronize()
        el = time.perf_counter() - t_start
        log(f"[bench] {c.name}: {n_tok} tokens without hints in {el:.1f} s")
        pt = np.sort(np.asarray(per_token))
        idx_used = np.zeros((c.n_layers, c.top_k), np.int32)
        B.odmoe_decode_step(stc.handle, xs[0], yc, None, idx_used, s)
        t1 = time.perf_counter()
        for t in range(n_tok):                                           # the same tokens with perfect hints
            B.odmoe_decode_step(stc.handle, xs[0], yc, idx_used, None, s)
        torch.cuda.synchronize()
        el_hint = time.perf_counter() - t1
        log(f"[bench] {c.name}: {n_tok} tokens with perfect hints in {el_hint:.1f} s")
        # hints corrupted at a chosen miss rate (fresh draws for every token): a wrong hint costs a
        # wasted copy plus a reload, so on a saturated link time grows with the miss rate (the
        # paper's predictors miss 0.06 % - 4.3 % of the activations, random prefetching 75 %,
        # Sections 3.2 and 4.2; rates below a few per cent need more hints than a short run holds
        # to be resolved and are left out).  The recall printed is the measured one.
        by_recall = {}
        rng = np.random.default_rng(0)
        for miss in (0.1, 0.75):
            n_r = max(4, n_tok // 4)
            hits = loads_r = 0
            preds = []
            for _ in range(n_r):
                pred = idx_used.copy()
                for l in range(c.n_layers):
                    wrong = [e for e in range(c.n_experts) if e not in idx_used[l]]
                    for i in range(c.top_k):
                        if rng.random() < miss and wrong:
                            pred[l, i] = wrong.pop(int(rng.integers(len(wrong))))
                preds.append(pred)
            torch.cuda.synchronize()
            t2 = time.perf_counter()
            for pred in preds:
                B.odmoe_decode_step(stc.handle, xs[0], yc, pred, None, s)
                hits += s.hint_hits
                loads_r += s.loads
            torch.cuda.synchronize()
            log(f"[bench] {c.name}: hints with miss rate {miss:g} done")
            by_recall[f"{miss:g}"] = {"hints": n_r * c.n_layers * c.top_k,
                                      "recall": round(hits / (n_r * c.n_layers * c.top_k), 4),
                                      "ms_per_token": round((time.perf_counter() - t2) / n_r * 1e3, 3),
                                      "copies_per_token": round(loads_r / n_r, 1)}
        s.t_step_ms = -1.0
        B.odmoe_decode_step(stc.handle, xs[0], yc, None, None, s)        # one timed token for the breakdown
        # the same bytes copied with no kernels in between (wall clock, all copy streams)
        load_ms = B.odmoe_time_expert_loads(stc.handle, max(2, n_tok // 5))
        kern_ms = s.t_ffn_up_ms + s.t_ffn_down_ms + s.t_glue_ms
        # the compute leg: the same stack with every expert resident in HBM (no copies, no host syncs)
        with harness.MoEStack(c.small(n_slots=0), layers_u, unique_layers=len(layers_u)) as str_:
            yr = torch.empty_like(xs[0])
            n_res = 16
            for _ in range(2):
                B.odmoe_decode_step(str_.handle, xs[0], yr, None, None, None)
            torch.cuda.synchronize()
            t2 = time.perf_counter()
            for t in range(n_res):
                B.odmoe_decode_step(str_.handle, xs[t % len(xs)], yr, None, None, None)
            torch.cuda.synchronize()
            comp_ms = (time.perf_counter() - t2) / n_res * 1e3
        # experts read in place: the same pinned buffers, no slot pool, no copies; the GEMV kernels
        # pull the activated experts' weights across the host link while they compute
        with harness.MoEStack(c.small(n_slots=0), layers_u, unique_layers=len(layers_u),
                              experts_in_host_memory=True, buffers_of=stc) as sth:
            yh = torch.empty_like(xs[0])
            B.odmoe_decode_step(sth.handle, xs[0], yh, None, None, None)
            torch.cuda.synchronize()
            same_bits = bool(torch.equal(yh, yc_first))
            n_inp = max(2, n_tok // 3)
            t2 = time.perf_counter()
            for t in range(n_inp):
                B.odmoe_decode_step(sth.handle, xs[t % len(xs)], yh, None, None, None)
            torch.cuda.synchronize()
            inplace_ms = (time.perf_counter() - t2) / n_inp * 1e3
        # the paper's predictor at this scale (Sections 1, 3.2): an int8 copy of the stack, resident in
        # HBM, decodes each token first; its routing is the prediction the cacheless stack starts its
        # copies from (the copy restarts from the full stack's input every iteration)
        shadow_pred = None
        if args.sep_iters > 0:
            from paper_2512_03927_amd import shadow
            t2 = time.time()
            with shadow.shadow_stack(c, layers_u, "int8") as shq:
                n_it = max(4, n_tok // 4)
                shadow.emulate(stc, shq, xs[0], 2, True)                  # warm-up
                rec, _, sh_ms, main_ms = shadow.emulate(stc, shq, xs[0], n_it, True)
                shadow_pred = {"shadow": "int8 experts, resident in HBM", "iterations": n_it,
                               "recall": round(float(np.mean(rec)), 4),
                               "shadow_ms_per_token": round(sh_ms / n_it, 3),
                               "main_ms_per_token": round(main_ms / n_it, 3),
                               "shadow_hbm_GB": round(len(layers_u) * c.n_experts * shq.expert_bytes / 1e9, 2)}
            log(f"[bench] {c.name}: int8 shadow predictor {shadow_pred} ({time.time() - t2:.1f} s)")
        step_ms = el / n_tok * 1e3
        # load-window check of the paper (Section 3.1): per layer, t^M = router + glue (the stand-in
        # for the main node's work), t^W = expert FFN, against the time to load one layer's k experts
        n_groups = B.odmoe_slot_groups(stc.handle)
        # (the timed router interval also contains the wait for this layer's copies: use the
        # resident-layer router time measured above for t^M)
        t_m = (route_ms_resident if c.hidden == cfg.hidden else 0.006) + s.t_glue_ms / c.n_layers
        t_w = (s.t_ffn_up_ms + s.t_ffn_down_ms) / c.n_layers
        t_load_layer = load_ms / c.n_layers
        window = B.odmoe_load_window_ms(n_groups, t_m, t_w)
        h2d = loads * c.expert_bytes / el / 1e9
        out = {"workload": c.name, "tokens": n_tok, "unique_layers": len(layers_u),
               "tokens_per_s": round(n_tok / el, 4), "ms_per_token": round(step_ms, 3),
               "ms_per_token_median_p10_p90": [round(float(np.median(pt)), 3),
                                               round(float(pt[int(0.1 * (len(pt) - 1))]), 3),
                                               round(float(pt[int(round(0.9 * (len(pt) - 1)))]), 3)],
               "h2d_GBps": round(h2d, 2), "h2d_frac_of_pcie5_x16": round(h2d / PCIE5_X16_GBPS, 4),
               "copy_only_ms_per_token": round(load_ms, 3), "kernel_ms_per_token": round(kern_ms, 3),
               "resident_stack_ms_per_token": round(comp_ms, 3),
               "step_over_max_compute_load": round(step_ms / max(load_ms, comp_ms), 4),
               "ms_per_token_with_perfect_hints": round(el_hint / n_tok * 1e3, 3),
               "experts_read_in_place": {"ms_per_token": round(inplace_ms, 3),
                                         "tokens_per_s": round(1e3 / inplace_ms, 4),
                                         "link_GBps": round(c.n_layers * c.top_k * c.expert_bytes / inplace_ms / 1e6, 2),
                                         "over_copy_only": round(inplace_ms / load_ms, 4),
                                         "hbm_expert_bytes": 0, "same_output_bits_as_slot_pool": same_bits},
               "by_hint_miss_rate": by_recall, "with_int8_shadow_predictor": shadow_pred,
               "load_window": {"n_groups": n_groups, "t_M_ms": round(t_m, 4), "t_W_ms": round(t_w, 4),
                               "t_maxload_ms": round(window, 4), "t_load_per_layer_ms": round(t_load_layer, 4),
                               "io_bottlenecked": bool(t_load_layer > window)},
               "hbm_slot_bytes": B.odmoe_slot_pool_bytes(stc.handle)}
        stc.close()
        log(f"[bench] cacheless: {out}")
        return out

    cacheless = None
    cacheless_fine = None
    if args.cacheless_tokens > 0:
        # Host arena of the 32-layer stack: U unique layers, layer l using the weights of layer l mod U.
        # The full arena (32 x 8 experts) is 90.2 GB; nothing is ever cached, so the bytes moved per
        # token do not depend on U.  U = 8 (22.5 GB pinned) unless the box is short of memory.
        c3 = synth.CONFIGS[3]
        U = max(1, min(args.arena_layers, c3.n_layers))
        if mem_avail_gb is not None:
            while U > 1 and 3 * U * c3.n_experts * c3.expert_bytes / 1e9 > 0.5 * mem_avail_gb:
                U //= 2              # stored copy + pinned copy (+ the resident-stack leg lives in HBM)
        t0 = time.time()
        layers3 = [layer] + [synth.layer_weights(c3, l) for l in range(1, U)]
        log(f"[bench] {c3.name}: {U} unique layers ({U * c3.n_experts * c3.expert_bytes / 1e9:.1f} GB) generated in "
            f"{time.time() - t0:.1f} s")
        cacheless = run_cacheless(c3, layers3, args.cacheless_tokens, [X_np[t] for t in range(4)])
        cacheless["host_arena"] = {"unique_layers": U, "pinned_GB": round(U * c3.n_experts * c3.expert_bytes / 1e9, 2),
                                   "full_arena_GB": round(c3.n_layers * c3.n_experts * c3.expert_bytes / 1e9, 1),
                                   "host_mem_total_GB": None if mem_total_gb is None else round(mem_total_gb),
                                   "why": "bytes per token do not depend on U (no expert is ever cached); "
                                          "U = 8 keeps weight generation and pinning to about a minute"}
        del layers3
        c5 = synth.CONFIGS[5]
        layers5 = [synth.layer_weights(c5, l) for l in range(2)]
        X5 = synth.tokens(c5, 4)
        cacheless_fine = run_cacheless(c5, layers5, 4 * args.cacheless_tokens, [X5[t] for t in range(4)])
        # sensitivity to the number of HBM slots (the paper does not state one for this shape):
        # S = k (no room to load ahead), 2k (the default), 4k
        sens = {}
        for S in (c5.top_k, 2 * c5.top_k, 4 * c5.top_k):
            with harness.MoEStack(c5.small(n_slots=S), layers5, unique_layers=2) as sts:
                x5 = harness.to_device(X5[0])
                y5 = torch.empty_like(x5)
                s5 = B.odmoe_stats()
                ids5 = np.zeros((c5.n_layers, c5.top_k), np.int32)
                B.odmoe_decode_step(sts.handle, x5, y5, None, ids5, s5)
                res = {}
                for name, pred in (("no_hints", None), ("perfect_hints", ids5)):
                    B.odmoe_decode_step(sts.handle, x5, y5, pred, None, s5)
                    torch.cuda.synchronize()
                    t3 = time.perf_counter()
                    n5 = max(4, args.cacheless_tokens)
                    for _ in range(n5):
                        B.odmoe_decode_step(sts.handle, x5, y5, pred, None, s5)
                    torch.cuda.synchronize()
                    res[name] = round((time.perf_counter() - t3) / n5 * 1e3, 3)
                sens[str(S)] = res
        cacheless_fine["ms_per_token_by_slot_count"] = sens
        log(f"[bench] slot sensitivity: {sens}")

    # ---- the shadow model's side (Sections 1, 3.2): int8 experts on the Mixtral-shaped layer (the cost
    # of the quantised copy), and the emulated predictor on a small stack (the recall it gives)
    sep = None
    if args.sep_iters > 0 or args.int8_passes > 0:
        from paper_2512_03927_amd import shadow
        sep = {}
    for qkind in (("int8", "int4") if args.int8_passes > 0 else ()):
        with shadow.shadow_stack(cfg, [layer], qkind) as q8:
            Xq = harness.to_device(X_np)
            Yq = torch.empty_like(Xq)
            for _ in range(2):
                for t in range(T):
                    B.odmoe_decode_step(q8.handle, Xq[t], Yq[t], None, None, None)
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            for _ in range(args.int8_passes):
                for t in range(T):
                    B.odmoe_decode_step(q8.handle, Xq[t], Yq[t], None, None, None)
            torch.cuda.synchronize()
            el8 = (time.perf_counter() - t1) / args.int8_passes
            r_us, u_us, d_us = (0.0, 1.0, 1.0) if args.no_kernel_pass else \
                B.odmoe_time_decode_kernels(q8.handle, 0, Xq, T, 2)
            hf = cfg.hidden * cfg.ffn
            if qkind == "int8":      # codes + one scale per row
                ub8, db8 = cfg.top_k * (2 * hf + 8 * cfg.ffn), cfg.top_k * (hf + 4 * cfg.hidden)
                what = "int8 experts (a scale per weight row)"
            else:                    # packed codes + one scale per group of 64
                ub8, db8 = cfg.top_k * (hf + 8 * hf // 64), cfg.top_k * (hf // 2 + 4 * hf // 64)
                what = "4-bit experts (a scale per group of 64)"
            sep[qkind + "_layer"] = {"workload": cfg.name + " with " + what, "tokens": T,
                                     "tokens_per_s": round(T / el8, 1),
                                     "speedup_over_bf16": round(T / el8 / tokens_per_s, 3),
                                     "expert_bytes": q8.expert_bytes,
                                     "bytes_vs_bf16": round(q8.expert_bytes / cfg.expert_bytes, 4),
                                     "ffn_up_us": round(u_us, 2), "ffn_up_GBps": round(ub8 / u_us / 1e3, 1),
                                     "ffn_up_frac_of_hbm_peak": round(ub8 / u_us / 1e3 / HBM_PEAK_GBPS, 4),
                                     "ffn_down_us": round(d_us, 2), "ffn_down_GBps": round(db8 / d_us / 1e3, 1),
                                     "ffn_down_frac_of_hbm_peak": round(db8 / d_us / 1e3 / HBM_PEAK_GBPS, 4),
                                     "route_us": round(r_us, 2)}
            if qkind == "int4":
                # bound by the conversion arithmetic, not the weight stream: about 2.4 vector
                # instructions per weight (mask, byte -> fp32, FMA) against 256 CUs x 64 lanes x 2.4 GHz
                ops = 2.4 * cfg.top_k * 3 * hf
                sep[qkind + "_layer"]["valu_frac_of_peak"] = round(ops / ((u_us + d_us) * 1e-6) / (256 * 64 * 2.4e9), 3)
            del Xq, Yq
        log(f"[bench] {qkind} experts: {sep[qkind + '_layer']}")
    if args.sep_iters > 0:
        cs = synth.MoEConfig("sep-h1024-f2048-e8-k2-16L", 1024, 2048, 8, 2, n_layers=16, n_slots=4,
                             dtype="bf16", n_tokens=1, glue=1, seed=7)
        layers_s = [synth.layer_weights(cs, l) for l in range(cs.n_layers)]
        xs0 = harness.to_device(synth.tokens(cs)[0])
        sep.update({"emulation_workload": cs.name, "iterations": args.sep_iters, "mean_recall": {}, "ms_per_token": {}})
        with harness.MoEStack(cs, layers_s) as main_s:
            for kind in ("bf16", "int8", "int4"):
                with shadow.shadow_stack(cs, layers_s, kind) as sh:
                    for aligned in (True, False):
                        r, _, sh_ms, main_ms = shadow.emulate(main_s, sh, xs0, args.sep_iters, aligned)
                        key = f"{kind}_{'aligned' if aligned else 'unaligned'}"
                        sep["mean_recall"][key] = round(float(np.mean(r)), 4)
                        sep["ms_per_token"][key] = {"shadow": round(sh_ms / args.sep_iters, 4),
                                                    "main_cacheless": round(main_ms / args.sep_iters, 4)}
        sep["random_prefetch_expectation"] = cs.top_k / cs.n_experts
        del layers_s
        # the paper's own setting: a full-precision (fp32) stack predicted by its FP16 / INT8 / 4-bit copies
        cf = cs.small(name="sep-h1024-f2048-e8-k2-16L-fp32", dtype="f32")
        layers_f = [synth.layer_weights(cf, l) for l in range(cf.n_layers)]
        xf0 = harness.to_device(synth.tokens(cf)[0])
        sep["fp32_main"] = {"emulation_workload": cf.name, "mean_recall": {}}
        with harness.MoEStack(cf, layers_f) as main_f:
            for kind in ("fp16", "int8", "int4"):
                with shadow.shadow_stack(cf, layers_f, kind) as sh:
                    for aligned in (True, False):
                        r, _, _, _ = shadow.emulate(main_f, sh, xf0, args.sep_iters, aligned)
                        sep["fp32_main"]["mean_recall"][f"{kind}_{'aligned' if aligned else 'unaligned'}"] = \
                            round(float(np.mean(r)), 4)
        del layers_f
        log(f"[bench] sep emulation: {sep}")

    # ---- CPU oracle on a bounded sample of the same workload
    cpu = None
    if args.cpu_tokens > 0:
        from oracle import moe_oracle as O
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            cores = os.cpu_count() or 1
        Wg, b, experts = layer
        t_start = time.perf_counter()
        worst = 0.0
        for t in range(args.cpu_tokens):
            y_ref, _, _ = O.moe_layer(X_np[t], Wg, b, experts, cfg.top_k)
            if t < Y_keep.shape[0]:
                worst = max(worst, float(np.max(np.abs(O.widen(Y_keep[t]) - y_ref)) / np.max(np.abs(y_ref))))
        el = time.perf_counter() - t_start
        cpu = {"value": round(args.cpu_tokens / el, 4), "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
               "sample": f"first {args.cpu_tokens} of the {T} tokens of {cfg.name} (float64 NumPy oracle)",
               "stored_weight_GBps": round(args.cpu_tokens / el * cfg.top_k * cfg.expert_bytes / 1e9, 2),
               "gpu_vs_oracle_max_rel_err": worst}
        log(f"[bench] cpu oracle: {cpu}")

    out = {
        "metric": "decode tokens/s per MoE layer stack", "value": round(tokens_per_s, 2), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": cfg.name, "hidden": cfg.hidden, "ffn": cfg.ffn, "n_experts": cfg.n_experts,
                   "top_k": cfg.top_k, "n_layers": 1, "tokens_per_step": T, "batch": 1,
                   "weights": "resident in HBM"},
        "expert_gemv_hbm_GBps": None if gemv_gbps is None else round(gemv_gbps, 1),
        "measured_ceilings": ceilings,
        "roofline": roofline, "full_precision_fp32": fp32, "cacheless": cacheless, "cacheless_fine_grained": cacheless_fine,
        "prefill": prefill, "sep_emulation": sep, "cpu_baseline": cpu,
    }
    print(json.dumps(out), flush=True)
    # explicit teardown: every handle above is closed; drop the remaining device / pinned tensors and
    # drain the device before the interpreter starts unloading libraries in its own order
    del X, Y, layer
    import gc
    gc.collect()
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    return 0


if __name__ == "__main__":
    sys.exit(main())
