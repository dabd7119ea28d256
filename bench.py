#!/usr/bin/env python3
"""Benchmark of the AnyBCQ bit-plane product on one MI355X.

Workload (the configuration the headline metric is quoted on): the seven linear
layers of one Llama-3-8B decoder block (q, k, v, o, gate, up, down), batch 1,
group 128, each run at precision p = 2, 3 and 4 -- 21 bcq_gemv calls per step.
Inputs are seeded and synthetic (synthetic_inputs.py) and resident in HBM before
the timed region.  To keep reads coming from HBM rather than the 256 MB last
level cache, successive steps rotate over distinct copies of the whole layer
set (>= 1 GiB in total).  Each step is one HIP-graph replay, so host launch
cost does not pace the GPU.

Prints ONE JSON line:
  value     effective HBM GB/s over the timed steps = algorithmic bytes / time,
            algorithmic bytes per call = m*n*p/8 (planes) + m*(n/128)*p*2
            (scales) + n*2 (x) + m*2 (y)
  roofline  the dominant kernel (plane_mfma_kernel<4> on a 14336x4096 layer):
            algorithmic bytes per launch / mean launch duration, measured with
            HIP events around back-to-back launches on the launch stream,
            against the 8 TB/s HBM peak
  cpu_baseline  the float64 oracle timed on the host cores on one copy of the
            same layer set (a reported baseline, not a target)
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
PRECISIONS = (2, 3, 4)
MIN_ROTATION_BYTES = 1 << 30


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--no-graph", action="store_true", help="launch from Python instead of replaying HIP graphs")
    ap.add_argument("--skip-cpu-baseline", action="store_true")
    ap.add_argument("--details", action="store_true", help="also time every (layer, p) kernel and an fp16 GEMV")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 256 MiB device copy a few times (a reference kernel of known traffic for counter runs)")
    ap.add_argument("--suite", choices=["decode", "mixed", "large", "phi4", "fused", "offset", "quant", "step", "issue", "generic"], default=None,
                    help="instead of the headline workload, time another workload family and print its table")
    return ap.parse_args()


KERNEL_SOURCE = os.path.join(ROOT, "paper_2510_10467_amd", "csrc", "bcq_plane_mfma.hip")
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "plane_mfma_llama3_8b_batch1.txt")


def kernel_source_sha256():
    import hashlib
    with open(KERNEL_SOURCE, "rb") as f:
        return hashlib.sha256(f.read()).hexdigest()


def profiled_traffic_bytes(p, m, n):
    """HBM bytes per launch of the dominant kernel from the committed counter summary (FETCH_SIZE + WRITE_SIZE,
    scaled by a plain copy).  The summary names the sha256 of the kernel source it was taken with; if the source has
    changed since, or the summary does not cover this kernel, the figure is None (never a stale number).
    Returns (bytes or None, note)."""
    want = (f"plane_mfma_kernel<{p},1,false>", f"{m}x{n}")
    try:
        text = open(TRAFFIC_PROFILE).read()
    except OSError:
        return None, "no counter summary under profiles/"
    stamp = [line.split()[-1] for line in text.splitlines() if line.startswith("kernel source sha256:")]
    if not stamp or stamp[0] != kernel_source_sha256():
        return None, "the kernel source has changed since the counter summary was taken"
    seen_counters = False
    for line in text.splitlines():
        seen_counters = seen_counters or line.startswith("HBM traffic counters")
        parts = line.split()
        if seen_counters and len(parts) >= 8 and parts[0] == want[0] and parts[1] == want[1]:
            return int(float(parts[-3]) * 1e6), "profiles/plane_mfma_llama3_8b_batch1.txt, same kernel source"
    return None, "the counter summary does not cover this kernel"


def run_suite(args, torch, bcq, syn, dev):
    """Other workload families: decode batches, per-request precision, Llama-3-70B shapes with large batches.

    Every entry is the mean time of back-to-back launches (one HIP graph) rotating over enough
    distinct weight copies to exceed the last-level cache; GB/s uses the algorithmic bytes."""
    gen = torch.Generator(device=dev)
    gen.manual_seed(syn.BASE_SEED)

    def device_layer(m, n):
        # same distributions as synthetic_inputs, drawn on the GPU to keep set-up short for the big shapes
        planes = torch.randint(-2 ** 31, 2 ** 31 - 1, (syn.P_MAX, m, n // 32), dtype=torch.int32, device=dev, generator=gen)
        scales = {}
        for p in (2, 3, 4):
            a1 = (torch.randn((m, n // syn.GROUP), device=dev, generator=gen) * 0.02).abs()
            rows = [a1]
            for _ in range(1, p):
                rows.append(rows[-1] * (0.4 + 0.2 * torch.rand((m, n // syn.GROUP), device=dev, generator=gen)))
            scales[p] = torch.stack(rows).half().contiguous()
        return planes, scales

    def timed_graph(fn, reps=10, warm=3):
        fn()
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            fn()
        for _ in range(warm):
            g.replay()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            g.replay()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    rows = []
    launches = 16

    def bench_shape(m, n, batches, precisions, mixed=False, offsets=False):
        copies = max(2, -(-MIN_ROTATION_BYTES // (m * n // 2)))
        copies = min(copies, 24)
        sets = [device_layer(m, n) for _ in range(copies)]
        for batch in batches:
            x = torch.randn((batch, n), device=dev, generator=gen).half()
            y = torch.empty((batch, m), dtype=torch.float16, device=dev)
            for p in precisions:
                # asymmetric scheme: one fp16 offset per (row, group), N(0, 0.01^2), one set per precision
                z = (torch.randn((m, n // syn.GROUP), device=dev, generator=gen) * 0.01).half() if offsets else None

                def burst():
                    for i in range(launches):
                        pl, sc = sets[i % copies]
                        bcq.bcq_gemv(pl, sc[p], p, x, y, offsets=z)
                us = timed_graph(burst) * 1e3 / launches
                by = syn.algorithmic_bytes(m, n, p, batch) + (m * (n // syn.GROUP) * 2 if offsets else 0)
                rows.append({"m": m, "n": n, "batch": batch, "p": p, "offsets": bool(offsets), "kernel": bcq.last_kernel(), "us": round(us, 2),
                             "GBps": round(by / us / 1e3, 1), "pct_of_hbm_peak": round(100 * by / us / 1e3 / HBM_PEAK_GBS, 2),
                             "TFLOPs": round(2.0 * m * n * batch / us / 1e6, 1)})
            if mixed:
                p_req_h = syn.make_p_req(batch, 2, 4, seed=(4, batch))
                p_req = torch.from_numpy(p_req_h).to(dev)

                def burst_mixed():
                    for i in range(launches):
                        pl, sc = sets[i % copies]
                        bcq.bcq_gemm_mixed(pl, sc, p_req, x, y)
                us = timed_graph(burst_mixed) * 1e3 / launches
                pmax = int(p_req_h.max())
                by = m * n * pmax // 8 + sum(m * (n // syn.GROUP) * q * 2 for q in sorted(set(p_req_h.tolist()))) + batch * (n + m) * 2
                rows.append({"m": m, "n": n, "batch": batch, "p": "mixed:" + ",".join(str(v) for v in p_req_h.tolist()[:16]) + ("..." if batch > 16 else ""),
                             "kernel": bcq.last_kernel(), "us": round(us, 2), "GBps": round(by / us / 1e3, 1),
                             "pct_of_hbm_peak": round(100 * by / us / 1e3 / HBM_PEAK_GBS, 2)})
        del sets

    if args.suite == "decode":
        for (m, n) in ((14336, 4096), (4096, 14336)):
            bench_shape(m, n, (1, 2, 4, 8, 16, 32), PRECISIONS)
    elif args.suite == "mixed":
        # the paper-sized case (16 requests, plane-wise kernel) and serving-sized batches (dequantising kernel)
        bench_shape(14336, 4096, (16, 64, 256), PRECISIONS, mixed=True)
    elif args.suite == "offset":
        # asymmetric scheme next to the symmetric one, batch 1 and a dequantising batch
        for (m, n) in ((4096, 4096), (14336, 4096), (4096, 14336)):
            bench_shape(m, n, (1, 64), PRECISIONS)
            bench_shape(m, n, (1, 64), PRECISIONS, offsets=True)
    elif args.suite == "generic":
        # the table look-up kernel and the per-bit kernel, which take every legal shape, beside the default choice: on
        # shapes of the main workload, and on a width the plane-wise FP4 kernel does not take (4224 columns: not a multiple of 256)
        for variant in ("auto", "lut", "sign_select"):
            bcq.select_kernel(variant)
            try:
                first = len(rows)
                bench_shape(14336, 4096, (1, 2, 8), (2, 4))
                bench_shape(4096, 4096, (1,), (2, 4))
                bench_shape(1024, 4096, (1,), (4,))
                bench_shape(14336, 4224, (1, 8), (4,))
                for r in rows[first:]:
                    r["forced"] = variant
            finally:
                bcq.select_kernel("auto")
    elif args.suite == "phi4":
        # second model of the paper's GEMV table; 17920 columns end in a half slice
        for (_, m, n) in syn.PHI4_14B_SHAPES:
            bench_shape(m, n, (1,), PRECISIONS)
    elif args.suite == "fused":
        # The linear layers of one Llama-3-8B decoder layer, batches 1, 16 and 64: seven bcq_gemv calls against four
        # calls in which q/k/v and gate/up (same activations) go through bcq_gemv_multi as one launch each.
        shapes = {"q": (4096, 4096), "k": (1024, 4096), "v": (1024, 4096), "o": (4096, 4096),
                  "gate": (14336, 4096), "up": (14336, 4096), "down": (4096, 14336)}
        copies = 8                                                   # 8 x 218 MB of planes: cold for the last-level cache
        sets = [{name: device_layer(m, n) for name, (m, n) in shapes.items()} for _ in range(copies)]
        for batch, p in [(b, q) for b in (1, 16, 64) for q in PRECISIONS]:
            x4k = torch.randn((batch, 4096), device=dev, generator=gen).half()
            x14k = torch.randn((batch, 14336), device=dev, generator=gen).half()
            ys = {name: torch.empty((batch, m), dtype=torch.float16, device=dev) for name, (m, n) in shapes.items()}
            def separate():
                for c in range(copies):
                    L = sets[c]
                    for name in ("q", "k", "v", "o", "gate", "up"):
                        bcq.bcq_gemv(L[name][0], L[name][1][p], p, x4k, ys[name])
                    bcq.bcq_gemv(L["down"][0], L["down"][1][p], p, x14k, ys["down"])

            def fused():
                for c in range(copies):
                    L = sets[c]
                    bcq.bcq_gemv_multi([L[k][0] for k in ("q", "k", "v")], [L[k][1][p] for k in ("q", "k", "v")], p, x4k,
                                       [ys[k] for k in ("q", "k", "v")])
                    bcq.bcq_gemv(L["o"][0], L["o"][1][p], p, x4k, ys["o"])
                    bcq.bcq_gemv_multi([L[k][0] for k in ("gate", "up")], [L[k][1][p] for k in ("gate", "up")], p, x4k,
                                       [ys[k] for k in ("gate", "up")])
                    bcq.bcq_gemv(L["down"][0], L["down"][1][p], p, x14k, ys["down"])
            by = sum(syn.algorithmic_bytes(m, n, p, batch) for (m, n) in shapes.values())
            us_sep = timed_graph(separate) * 1e3 / copies
            us_fus = timed_graph(fused) * 1e3 / copies
            rows.append({"workload": f"linear layers of one Llama-3-8B decoder layer, batch {batch}", "p": p, "batch": batch,
                         "seven_calls_us": round(us_sep, 2), "four_calls_us": round(us_fus, 2),
                         "seven_calls_GBps": round(by / us_sep / 1e3, 1), "four_calls_GBps": round(by / us_fus / 1e3, 1),
                         "pct_of_hbm_peak_four_calls": round(100 * by / us_fus / 1e3 / HBM_PEAK_GBS, 2)})
    elif args.suite == "step":
        # The linear layers of one whole decoding step of a Llama-3-8B-shaped model (32 decoder layers; batches 1, 16
        # and 64) as ONE HIP graph (128 launches at batch 1): per layer q/k/v together, o, gate/up together, down.  Every layer has its
        # own planes and scale sets (3.5 GB of planes), so nothing is warm.  Attention, norms and the vocabulary
        # projection are not part of the library and not in the figure: the tokens/s is an upper bound.
        shapes = {"q": (4096, 4096), "k": (1024, 4096), "v": (1024, 4096), "o": (4096, 4096),
                  "gate": (14336, 4096), "up": (14336, 4096), "down": (4096, 14336)}
        n_layers = 32
        model = [{name: device_layer(m, n) for name, (m, n) in shapes.items()} for _ in range(n_layers)]
        for batch in (1, 16, 64):
            x4k = torch.randn((batch, 4096), device=dev, generator=gen).half()
            x14k = torch.randn((batch, 14336), device=dev, generator=gen).half()
            ys = {name: torch.empty((batch, m), dtype=torch.float16, device=dev) for name, (m, n) in shapes.items()}
            for p in PRECISIONS:
                def step():
                    for L in model:
                        bcq.bcq_gemv_multi([L[k][0] for k in ("q", "k", "v")], [L[k][1][p] for k in ("q", "k", "v")], p, x4k,
                                           [ys[k] for k in ("q", "k", "v")])
                        bcq.bcq_gemv(L["o"][0], L["o"][1][p], p, x4k, ys["o"])
                        bcq.bcq_gemv_multi([L[k][0] for k in ("gate", "up")], [L[k][1][p] for k in ("gate", "up")], p, x4k,
                                           [ys[k] for k in ("gate", "up")])
                        bcq.bcq_gemv(L["down"][0], L["down"][1][p], p, x14k, ys["down"])
                by = n_layers * sum(syn.algorithmic_bytes(m, n, p, batch) for (m, n) in shapes.values())
                ms = timed_graph(step)
                # (the several-matrices call is one launch at every batch: 4 launches per layer)
                rows.append({"workload": f"linear layers of one decoding step, Llama-3-8B shapes, 32 layers, batch {batch}", "p": p,
                             "batch": batch, "launches": 4 * n_layers, "ms_per_step": round(ms, 4),
                             "ms_per_token": round(ms / batch, 4), "GBps": round(by / ms / 1e6, 1),
                             "pct_of_hbm_peak": round(100 * by / ms / 1e6 / HBM_PEAK_GBS, 2),
                             "tokens_per_s_upper_bound": round(batch * 1e3 / ms, 1)})
    elif args.suite == "issue":
        # What one SIMD issues when matrix and vector instructions alternate (include/bcq_bench.h): shader-clock ticks per
        # matrix instruction for one wave per SIMD (4 waves) and for two (8).  A matrix instruction keeps its SIMD from
        # issuing anything else for about 20 ticks whatever its size, a vector instruction for 4: the product kernels'
        # time after their data have arrived is the sum of these over their instructions, not the larger of the pipes.
        ticks = torch.zeros(32, dtype=torch.int64, device=dev)
        sink = torch.zeros(1024, dtype=torch.float32, device=dev)
        iters = 4000
        names = {0: "v_mfma_f32_16x16x32_f16", 1: "v_mfma_f32_32x32x16_f16", 2: "v_mfma_f32_16x16x128_f8f6f4 (E5M2 x FP4)"}
        for kind in (0, 1, 2):
            for valu in (0, 4, 8, 16):
                for waves in (4, 8):
                    bcq.bench_issue_probe(kind, valu, waves, iters, ticks, sink)      # warm-up (instruction cache)
                    bcq.bench_issue_probe(kind, valu, waves, iters, ticks, sink)
                    torch.cuda.synchronize()
                    t = ticks.cpu().numpy().reshape(16, 2)[:waves]
                    per_simd = waves // 4                                             # waves that share a SIMD
                    rows.append({"instruction": names[kind], "vector_fmas_per_matrix_instruction": valu, "waves_per_simd": per_simd,
                                 "ticks_per_matrix_instruction_per_simd": round(float(t[:, 0].max()) / (4 * iters) / per_simd, 1),
                                 "shader_clock_MHz": round(float(t[:, 0].max()) / float(t[:, 1].max()) * 100.0, 0)})
        return {"suite": args.suite, "unit": "shader-clock ticks", "data": "none", "rows": rows}
    elif args.suite == "quant":
        # The offline quantiser (Algorithm 1, p_L = 2, p_H = 4, T = 20, g = 128) on Llama-3-8B layer shapes.
        # Bound by double-precision vector arithmetic: per weight and cycle the base stage adds p signed terms
        # and compares against 2^p levels (sub + compare), an expansion stage to p bits spends p + 1 operations
        # (p - 1 level terms, the residual, the signed sum); the per-group solves add about one more per cycle.
        p_low, p_high, cycles = 2, 4, 20
        ops_per_weight = cycles * ((p_low + 2 * 2 ** p_low + 1) + sum(p + 2 for p in range(p_low + 1, p_high + 1))) + 3 * p_low
        peak_ops = 256 * 4 * 16 * 2.4e9                               # lanes x clock: one double operation per lane and cycle
        import time

        import numpy as np

        import oracle
        for (m, n) in ((4096, 4096), (14336, 4096), (4096, 14336)):
            w = torch.from_numpy(syn.make_weights(m, n, seed=(8, m))).to(dev)
            for with_offset in (False, True):
                out = bcq.bcq_quantize(w, p_low, p_high, cycles, with_offset=with_offset)
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                reps = 5
                e0.record()
                for _ in range(reps):
                    bcq.bcq_quantize(w, p_low, p_high, cycles, with_offset=with_offset, planes=out[0], scales_by_p=out[1],
                                     offsets_by_p=out[2])
                e1.record()
                torch.cuda.synchronize()
                ms = e0.elapsed_time(e1) / reps
                rows.append({"shape": f"{m}x{n}", "p_low": p_low, "p_high": p_high, "cycles": cycles, "offset": with_offset,
                             "ms": round(ms, 3), "Gweights_per_s": round(m * n / ms / 1e6, 2),
                             "roofline": {"bound": "alu", "unit": "Tops/s (fp64 lane operations)",
                                          "achieved": round(ops_per_weight * m * n / ms / 1e9, 2),
                                          "peak": round(peak_ops / 1e12, 2),
                                          "frac": round(ops_per_weight * m * n / (ms * 1e-3) / peak_ops, 4)}})
        sample = syn.make_weights(512, 4096, seed=(8, 0))
        t0 = time.perf_counter()
        oracle.quantize(sample, p_low, p_high, cycles)
        dt = time.perf_counter() - t0
        rows.append({"cpu_baseline": {"value": round(sample.size / dt / 1e9, 5), "unit": "Gweights/s", "cores": oracle.num_threads(),
                                      "kind": "oracle", "sample": "512x4096 weights, p 2..4, T = 20, symmetric"}})
        return {"suite": args.suite, "unit": "ms per matrix", "data": "synthetic", "ops_per_weight": ops_per_weight, "rows": rows}
    else:
        for (_, m, n) in syn.LLAMA3_70B_SHAPES:
            bench_shape(m, n, (1, 16, 64, 256), PRECISIONS)
    return {"suite": args.suite, "unit": "us per call", "data": "synthetic", "rows": rows}


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus must be 1 (no multi-GPU path exists)", file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2510_10467_amd as bcq
    import synthetic_inputs as syn

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    bcq.lib()                                        # fail loudly if the HIP library is missing

    if args.suite:
        print(json.dumps(run_suite(args, torch, bcq, syn, dev)))
        return

    layers = syn.LLAMA3_8B_LAYERS
    set_bytes = sum(m * n * syn.P_MAX // 8 + sum(m * (n // syn.GROUP) * p * 2 for p in PRECISIONS) for _, m, n in layers)
    copies = max(2, -(-MIN_ROTATION_BYTES // set_bytes))

    def upload(a):
        return torch.from_numpy(a.view(np.int32) if a.dtype == np.uint32 else a).to(dev)

    # ---- inputs: `copies` independent layer sets, resident in HBM ------------------------------
    host_copy0 = None
    dev_sets = []
    for c in range(copies):
        host = [syn.make_layer(m, n, seed=(2, c, li), precisions=PRECISIONS) for li, (_, m, n) in enumerate(layers)]
        if c == 0:
            host_copy0 = host
        dev_sets.append([(upload(L.planes), {p: upload(s) for p, s in L.scales.items()}) for L in host])
        del host
    xs_host = {n: syn.make_x(1, n, seed=(2, n)) for n in sorted({n for _, _, n in layers})}
    xs = {n: upload(x) for n, x in xs_host.items()}
    ys = [torch.empty((1, m), dtype=torch.float16, device=dev) for _, m, _ in layers]
    torch.cuda.synchronize()

    def run_step(c, precisions=PRECISIONS):
        for p in precisions:
            for li, (_, m, n) in enumerate(layers):
                planes, scales = dev_sets[c][li]
                bcq.bcq_gemv(planes, scales[p], p, xs[n], ys[li])

    bytes_per_p = {p: sum(syn.algorithmic_bytes(m, n, p, 1) for _, m, n in layers) for p in PRECISIONS}
    bytes_per_step = sum(bytes_per_p.values())

    # ---- one HIP graph per copy (a step = one replay) ----------------------------------------
    def capture(fn):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            fn()
        return g

    run_step(0)
    torch.cuda.synchronize()
    kernel_name = bcq.last_kernel()
    if args.no_graph:
        step_fns = [lambda c=c: run_step(c) for c in range(copies)]
    else:
        graphs = [capture(lambda c=c: run_step(c)) for c in range(copies)]
        step_fns = [g.replay for g in graphs]

    def timed(fns, count, warmup):
        for i in range(warmup):
            fns[i % len(fns)]()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(count):
            fns[i % len(fns)]()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / count            # ms per call

    ms_per_step = timed(step_fns, args.steps, args.warmup)
    value = bytes_per_step / (ms_per_step * 1e-3) / 1e9

    # ---- per-precision step times (7 calls each) ---------------------------------------------
    per_p = {}
    for p in PRECISIONS:
        if args.no_graph:
            fns = [lambda c=c, p=p: run_step(c, (p,)) for c in range(copies)]
        else:
            fns = [capture(lambda c=c, p=p: run_step(c, (p,))).replay for c in range(copies)]
        ms = timed(fns, max(args.steps, 40), max(args.warmup // 2, 8))
        per_p[str(p)] = {"us_per_layer_set": round(ms * 1e3, 3), "us_per_gemv_mean": round(ms * 1e3 / len(layers), 3),
                         "effective_GBps": round(bytes_per_p[p] / (ms * 1e-3) / 1e9, 1),
                         "pct_of_hbm_peak": round(100 * bytes_per_p[p] / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 2)}

    # ---- the same 21 products with q/k/v and gate/up handed to bcq_gemv_multi (12 launches per step):
    # a secondary figure; `value` above stays with one bcq_gemv call per product
    idx = {name: li for li, (name, _, _) in enumerate(layers)}
    groups = [("q_proj", "k_proj", "v_proj"), ("o_proj",), ("gate_proj", "up_proj"), ("down_proj",)]

    def run_step_multi(c):
        for p in PRECISIONS:
            for names in groups:
                lis = [idx[nm] for nm in names]
                n = layers[lis[0]][2]
                if len(lis) == 1:
                    planes, scales = dev_sets[c][lis[0]]
                    bcq.bcq_gemv(planes, scales[p], p, xs[n], ys[lis[0]])
                else:
                    bcq.bcq_gemv_multi([dev_sets[c][li][0] for li in lis], [dev_sets[c][li][1][p] for li in lis], p, xs[n],
                                       [ys[li] for li in lis])
    run_step_multi(0)
    torch.cuda.synchronize()
    multi_fns = [lambda c=c: run_step_multi(c) for c in range(copies)] if args.no_graph else \
                [capture(lambda c=c: run_step_multi(c)).replay for c in range(copies)]
    ms_multi = timed(multi_fns, args.steps, args.warmup)
    multi_call = {"what": "the same 21 products, q/k/v and gate/up through bcq_gemv_multi: 12 launches per step",
                  "value": round(bytes_per_step / (ms_multi * 1e-3) / 1e9, 1), "unit": "GB/s", "ms_per_step": round(ms_multi, 5),
                  "pct_of_hbm_peak": round(100 * bytes_per_step / (ms_multi * 1e-3) / 1e9 / HBM_PEAK_GBS, 2)}

    # ---- roofline of the dominant kernel: gate/up-shaped layer at p = 4 -----------------------
    def kernel_time_us(li, p, launches=64):
        """Mean duration of back-to-back launches of one (layer, p), rotating over the copies."""
        _, m, n = layers[li]
        same_shape = [k for k, (_, mm, nn) in enumerate(layers) if (mm, nn) == (m, n)]
        bufs = [(dev_sets[c][k][0], dev_sets[c][k][1][p]) for c in range(copies) for k in same_shape]

        def burst():
            for i in range(launches):
                pl, sc = bufs[i % len(bufs)]
                bcq.bcq_gemv(pl, sc, p, xs[n], ys[li])
        burst()
        torch.cuda.synchronize()
        fn = burst if args.no_graph else capture(burst).replay
        return timed([fn], 10, 3) * 1e3 / launches

    dom_li = [i for i, (name, _, _) in enumerate(layers) if name == "gate_proj"][0]
    dom_p = 4
    _, dm, dn = layers[dom_li]
    dom_us = kernel_time_us(dom_li, dom_p)
    dom_bytes = syn.algorithmic_bytes(dm, dn, dom_p, 1)
    achieved = dom_bytes / (dom_us * 1e-6) / 1e9
    traffic, traffic_note = profiled_traffic_bytes(dom_p, dm, dn)
    roofline = {"bound": "hbm", "kernel": f"plane_mfma_kernel<{dom_p}> m={dm} n={dn} batch=1",
                "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic, "traffic_source": traffic_note,
                "bytes_per_launch": dom_bytes, "us_per_launch": round(dom_us, 3)}

    # The same product in the other formulations the library holds (section 3.3 names table look-ups; the per-bit
    # add/subtract form is its plain reading): why the matrix-pipe kernel is the one that runs.
    formulations = {"workload": f"m={dm} n={dn} batch 1 p={dom_p}, us per call over cold copies",
                    "plane_mfma": round(dom_us, 3)}
    for variant in ("lut", "sign_select"):
        bcq.select_kernel(variant)
        try:
            formulations[variant] = round(kernel_time_us(dom_li, dom_p, launches=16), 3)
        finally:
            bcq.select_kernel("auto")

    # What a pure streaming read reaches on this GPU: as many bytes as the dominant kernel moves (cold, rotating
    # over distinct buffers, back-to-back launches in a graph), and 1 GiB in one launch.
    sink = torch.zeros(64, dtype=torch.int32, device=dev)
    small = [torch.empty(dom_bytes // 16 * 16, dtype=torch.uint8, device=dev).random_(0, 255) for _ in range(32)]

    def read_burst():
        for b in small:
            bcq.bench_stream_read(b, sink)
    read_burst()
    torch.cuda.synchronize()
    us_read = timed([capture(read_burst).replay], 10, 3) * 1e3 / len(small)
    del small
    big = torch.empty(1 << 30, dtype=torch.uint8, device=dev).random_(0, 255)
    bcq.bench_stream_read(big, sink)
    torch.cuda.synchronize()
    us_big = timed([lambda: bcq.bench_stream_read(big, sink)], 10, 3) * 1e3
    del big
    roofline["stream_read_same_bytes"] = {"us": round(us_read, 3), "GBps": round(dom_bytes / us_read / 1e3, 1),
                                          "kernel_vs_stream_read": round(us_read / dom_us, 4)}
    roofline["stream_read_1GiB"] = {"us": round(us_big, 1), "GBps": round((1 << 30) / us_big / 1e3, 1)}

    # ---- the same GPU on the half-precision product of the dominant shape (the paper's Table 2 sets its kernel
    # against one): the library's GEMV and a plain one-wavefront-per-row kernel, rotating over distinct matrices
    ws = [torch.randn((dm, dn), dtype=torch.float16, device=dev) for _ in range(12)]
    xv = xs[dn][0]
    yv = torch.empty((dm,), dtype=torch.float16, device=dev)

    def fp16_burst():
        for i in range(48):
            torch.mv(ws[i % len(ws)], xv)

    def fp16_own_burst():
        for i in range(48):
            bcq.bench_fp16_gemv(ws[i % len(ws)], xv, yv)
    fp16_burst()
    fp16_own_burst()
    torch.cuda.synchronize()
    us16 = timed([fp16_burst], 10, 3) * 1e3 / 48
    us16o = timed([fp16_own_burst if args.no_graph else capture(fp16_own_burst).replay], 10, 3) * 1e3 / 48
    del ws
    fp16_gemv = {"m": dm, "n": dn, "bytes": 2 * dm * dn,
                 "library_torch_mv": {"us": round(us16, 3), "GBps": round(2 * dm * dn / (us16 * 1e-6) / 1e9, 1)},
                 "plain_hip_kernel": {"us": round(us16o, 3), "GBps": round(2 * dm * dn / (us16o * 1e-6) / 1e9, 1)},
                 "bcq_p4_speedup_vs_plain_kernel": round(us16o / dom_us, 2)}

    # ---- other configurations, generated on the GPU with the same distributions (cold: >= 1 GiB of copies each)
    gen = torch.Generator(device=dev)
    gen.manual_seed(syn.BASE_SEED + 1)

    def device_layer(m, n, precisions):
        planes = torch.randint(-2 ** 31, 2 ** 31 - 1, (syn.P_MAX, m, n // 32), dtype=torch.int32, device=dev, generator=gen)
        scales = {}
        for p in precisions:
            rows = [(torch.randn((m, n // syn.GROUP), device=dev, generator=gen) * 0.02).abs()]
            for _ in range(1, p):
                rows.append(rows[-1] * (0.4 + 0.2 * torch.rand((m, n // syn.GROUP), device=dev, generator=gen)))
            scales[p] = torch.stack(rows).half().contiguous()
        return planes, scales

    def shape_times(m, n, precisions, launches=32):
        """us per bcq_gemv call at batch 1 for every p, back-to-back launches over cold copies."""
        ncopies = min(128, max(2, -(-MIN_ROTATION_BYTES // (m * n // 2))))
        sets = [device_layer(m, n, precisions) for _ in range(ncopies)]
        x = torch.randn((1, n), device=dev, generator=gen).half()
        y = torch.empty((1, m), dtype=torch.float16, device=dev)
        out = {}
        for p in precisions:
            def burst():
                for i in range(launches):
                    pl, sc = sets[(i * 7) % ncopies]
                    bcq.bcq_gemv(pl, sc[p], p, x, y)
            burst()
            torch.cuda.synchronize()
            # freshly allocated copies: the first passes over them run slower than the steady state, so the
            # warm-up is longer than elsewhere and the figure is the median of five timed runs of ten replays
            fn = burst if args.no_graph else capture(burst).replay
            runs = sorted(timed([fn], 10, 10 if k == 0 else 0) for k in range(5))
            us = runs[2] * 1e3 / launches
            by = syn.algorithmic_bytes(m, n, p, 1)
            out[str(p)] = {"us": round(us, 3), "GBps": round(by / us / 1e3, 1), "pct_of_hbm_peak": round(100 * by / us / 1e3 / HBM_PEAK_GBS, 2)}
        del sets
        return out

    single_gemv_4096 = {"workload": "single BCQ GEMV m=4096 n=4096 batch 1, p in {1,2,3,4}, group 128", "per_p": shape_times(4096, 4096, (1, 2, 3, 4))}
    llama70b = {"workload": "Llama-3-70B-shaped layer m=28672 n=8192 batch 1, group 128", "per_p": shape_times(28672, 8192, (2, 4), launches=16)}

    # ---- per-request precision against the uniform kernel: batch 16 on the gate/up shape, each request's precision
    # drawn uniformly from {2,3,4} (seeded), against uniform batches of 16 at the deepest precision; 40 repeats each,
    # alternating, the ratio taken over the medians
    same_shape = [k for k, (_, mm, nn) in enumerate(layers) if (mm, nn) == (dm, dn)]
    mix_sets = [dev_sets[c][k] for c in range(copies) for k in same_shape]
    x16 = torch.randn((16, dn), device=dev, generator=gen).half()
    y16 = torch.empty((16, dm), dtype=torch.float16, device=dev)
    p_req_h = syn.make_p_req(16, 2, 4, seed=(4, 16))
    p_req = torch.from_numpy(p_req_h).to(dev)

    def mixed_burst():
        for i in range(len(mix_sets)):
            pl, sc = mix_sets[i]
            bcq.bcq_gemm_mixed(pl, sc, p_req, x16, y16)

    def uniform_burst():
        for i in range(len(mix_sets)):
            pl, sc = mix_sets[i]
            bcq.bcq_gemv(pl, sc[int(p_req_h.max())], int(p_req_h.max()), x16, y16)
    mixed_burst()
    mixed_kernel = bcq.last_kernel()
    uniform_burst()
    uniform_kernel = bcq.last_kernel()
    torch.cuda.synchronize()
    fm = mixed_burst if args.no_graph else capture(mixed_burst).replay
    fu = uniform_burst if args.no_graph else capture(uniform_burst).replay
    tm, tu = [], []
    for _ in range(40):
        tm.append(timed([fm], 1, 1) * 1e3 / len(mix_sets))
        tu.append(timed([fu], 1, 1) * 1e3 / len(mix_sets))
    med = lambda v: sorted(v)[len(v) // 2]
    mixed_vs_uniform = {"workload": f"batch 16 on {dm}x{dn}, p per request drawn from {{2,3,4}}: " + ",".join(str(v) for v in p_req_h.tolist()),
                        "mixed_us": round(med(tm), 2), "uniform_p_max_us": round(med(tu), 2), "ratio": round(med(tm) / med(tu), 3),
                        "repeats": 40, "kernels": {"mixed": mixed_kernel, "uniform": uniform_kernel}, "target_ratio": 1.10}

    # ---- decode batches (uniform precision) on the gate/up and the down shape, over the copies already resident:
    # us per call, the kernel that ran, and the share of the HBM peak the algorithmic bytes come to
    decode_batches = {"workload": "decode batches 2..32, uniform p in {2,3,4}, group 128; us per call over cold copies", "rows": []}
    for (m_d, n_d) in ((dm, dn), (dn, dm)):
        shape_sets = [dev_sets[c][k] for c in range(copies) for k, (_, mm, nn) in enumerate(layers) if (mm, nn) == (m_d, n_d)]
        if not shape_sets:
            continue
        for batch in (2, 4, 8, 16, 32):
            xb = torch.randn((batch, n_d), device=dev, generator=gen).half()
            yb = torch.empty((batch, m_d), dtype=torch.float16, device=dev)
            for p in PRECISIONS:
                def burst():
                    for pl, sc in shape_sets:
                        bcq.bcq_gemv(pl, sc[p], p, xb, yb)
                burst()
                used = bcq.last_kernel()
                torch.cuda.synchronize()
                fn = burst if args.no_graph else capture(burst).replay
                us = sorted(timed([fn], 4, 2 if k == 0 else 0) for k in range(3))[1] * 1e3 / len(shape_sets)
                by = syn.algorithmic_bytes(m_d, n_d, p, batch)
                decode_batches["rows"].append({"m": m_d, "n": n_d, "batch": batch, "p": p, "kernel": used, "us": round(us, 2),
                                               "pct_of_hbm_peak": round(100 * by / us / 1e3 / HBM_PEAK_GBS, 1)})

    details = None
    if args.details:
        details = {"kernels": []}
        seen = set()
        for li, (name, m, n) in enumerate(layers):
            if (m, n) in seen:
                continue
            seen.add((m, n))
            for p in PRECISIONS:
                us = kernel_time_us(li, p)
                by = syn.algorithmic_bytes(m, n, p, 1)
                details["kernels"].append({"m": m, "n": n, "p": p, "us": round(us, 3),
                                           "GBps": round(by / (us * 1e-6) / 1e9, 1),
                                           "pct_of_hbm_peak": round(100 * by / (us * 1e-6) / 1e9 / HBM_PEAK_GBS, 2)})

    if args.calibrate_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- CPU baseline: the oracle as it stands, on one copy of the same layer set -------------
    cpu_baseline = None
    if not args.skip_cpu_baseline:
        import oracle
        reps = 8                                     # about 10 s of CPU work on the box's 16 cores
        t0 = time.perf_counter()
        for _ in range(reps):
            for p in PRECISIONS:
                for li, (_, m, n) in enumerate(layers):
                    oracle.gemv(host_copy0[li].planes, host_copy0[li].scales[p], xs_host[n])
        dt = (time.perf_counter() - t0) / reps
        cpu_baseline = {"value": round(bytes_per_step / dt / 1e9, 4), "unit": "GB/s", "cores": oracle.num_threads(),
                        "kind": "oracle", "seconds": round(dt * reps, 2),
                        "sample": f"{reps} steps of the 7 Llama-3-8B layers at p=2,3,4, batch 1 "
                                  f"({21 * reps} oracle products, float64), one weight copy"}

    out = {
        "metric": "bcq_gemv effective HBM GB/s, Llama-3-8B linear set, batch 1, p=2/3/4",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "Llama-3-8B-shaped linear set (q,k,v,o,gate,up,down), batch 1, group 128, p in {2,3,4}; "
                               "one step = 21 bcq_gemv calls", "kernel": kernel_name,
                   "arithmetic": "fp16 in/out; four E5M2 terms per activation (exact over all of binary16) x FP4 weight signs on the MFMA pipe, fp32 accumulate",
                   "weight_copies_rotated": copies, "rotation_bytes": copies * set_bytes,
                   "launch": "python loop" if args.no_graph else "hip graph replay per step"},
        "pct_of_hbm_peak": round(100 * value / HBM_PEAK_GBS, 2),
        "bytes_per_step": bytes_per_step,
        "per_precision": per_p,
        "multi_call": multi_call,
        "fp16_gemv": fp16_gemv,
        "single_gemv_4096": single_gemv_4096,
        "formulations": formulations,
        "llama70b_batch1": llama70b,
        "mixed_vs_uniform": mixed_vs_uniform,
        "decode_batches": decode_batches,
        "roofline": roofline,
        "cpu_baseline": cpu_baseline,
    }
    if details:
        out["details"] = details
    print(json.dumps(out))


if __name__ == "__main__":
    main()
