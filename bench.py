#!/usr/bin/env python3
"""Benchmark of the LUT-KAN layer forward on one MI355X.

One "step" is one pass of the whole hot path (locate kernel + edge kernel, i.e. lutkan_forward) over one batch of
seeded synthetic input that is already resident in HBM.  The workload is the largest single-GPU configuration:
one dense layer 1024 -> 1024, G = 10 segments on [-1,1], cubic splines with N(0,1) coefficients compiled to
L = 64 symmetric int8 tables, batch 32768 rows of x ~ N(0, 0.5) clipped to [-1.2, 1.2], closed + clip_x.

Prints ONE JSON line: edge-evaluations/s (batch*d*m per second), the roofline record of the dominant kernel
(the edge kernel) measured with HIP events on the launch stream, the B-spline baseline ratio, and the CPU
oracle timed on a bounded sample of the same rows.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# fp32 vector rate without the packed-fp32 forms (this library is built with them disabled):
# 256 CUs x 4 SIMDs x 16 lanes x 2 flop (FMA) x 2.4 GHz.  The published packed figure is 157.3 TFLOP/s.
PEAK_FP32_TFLOPS = 256 * 4 * 16 * 2 * 2.4e9 / 1e12
PEAK_FP32_PACKED_TFLOPS = 157.3
PEAK_HBM_GBS = 8000.0
# Algorithmic fp32 operations per edge evaluation (Eq. 10 twice: 2 mul + 2 add; Eq. 17: 2 mul + 1 add;
# Eq. 1: 1 add).  Integer->float conversions, address arithmetic and the 1-w subtraction are not counted.
FLOP_PER_EDGE = 8
# HBM traffic of one edge-kernel launch on the default workload, from rocprofv3 --pmc FETCH_SIZE (x2.0, the factor a
# plain 1 GiB copy gives) + WRITE_SIZE (x1.0); see profiles/lutkan_tiled_kernel_cfg4_B32768.md.
MEASURED_TRAFFIC_BYTES = {32768: 3.72e9}


def log(msg):
    print(msg, file=sys.stderr, flush=True)


def time_all_configs(lk, torch, dev, with_oracle):
    """Every workload of the scope table: one lutkan_model_forward and the chained B-spline layers (events, mean of 20
    after 3 warm-up runs), and the oracle chain on a bounded sample of rows with all host threads."""
    import numpy as np
    from lutkan_inputs import ASYM_UINT8, HALF_OPEN, SYM_INT8, ZERO_SPLINE, cfg1, cfg2, cfg3, cfg4, cfg5

    def timed(fn, n=20, warm=3):
        for _ in range(warm):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(n):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n

    def oracle_rate(wl, budget_s=4.0):
        import oracle
        arts = [oracle.compile_layer(s.d, s.m, s.G, s.p, s.ext_knots, s.coef, s.L, s.scheme) for s in wl.layers]
        per_row = sum(s.d * s.m for s in wl.layers)
        threads = oracle.default_threads()

        def chain(x):
            for a, s in zip(arts, wl.layers):
                x = oracle.lut_forward(a, s.boundary, s.oob, x, nthreads=threads).y
            return x

        rows = min(wl.x.shape[0], 64)
        t0 = time.perf_counter()
        chain(wl.x[:rows])
        rate = rows / (time.perf_counter() - t0)
        rows = int(min(wl.x.shape[0], max(rows, rate * budget_s)))
        t0 = time.perf_counter()
        chain(wl.x[:rows])
        return rows * per_row / (time.perf_counter() - t0), rows

    workloads = [("cfg1", cfg1()), ("cfg2", cfg2())]
    workloads += [(f"cfg3 L={L} {'sym' if sc == SYM_INT8 else 'asym'}", cfg3(L=L, scheme=sc)) for sc in (SYM_INT8, ASYM_UINT8)
                  for L in (16, 32, 64, 128)]
    workloads += [(f"cfg4 B={B}", cfg4(B=B)) for B in (256, 4096, 32768)]
    workloads += [("cfg5 closed+clip_x", cfg5()), ("cfg5 half_open+zero_spline", cfg5(boundary=HALF_OPEN, oob=ZERO_SPLINE))]
    rows_out = []
    log(f"[bench] {'workload':28s} {'B':>7s} {'LUT ms':>9s} {'G edge-evals/s':>15s} {'B-spline ms':>12s} {'ratio':>6s} {'oracle G/s':>11s}")
    for name, wl in workloads:
        arts = [lk.lutkan_compile(s.d, s.m, s.G, s.p, s.ext_knots, s.coef, s.L, s.scheme, s.boundary, s.oob) for s in wl.layers]
        layers = [a.to_device(dev) for a in arts]
        splines = [a.bspline_to_device(dev) for a in arts]
        x = torch.from_numpy(wl.x).to(dev)
        B = x.shape[0]
        ws = torch.empty(lk.lutkan_model_workspace_bytes(layers, B), dtype=torch.uint8, device=dev)
        y = torch.empty((B, layers[-1].m), dtype=torch.float32, device=dev)
        ms = timed(lambda: lk.lutkan_model_forward(layers, x, y, workspace=ws))
        acts = [x] + [torch.empty((B, s.m), dtype=torch.float32, device=dev) for s in wl.layers]
        wsb = torch.empty(max(lk.bspline_forward_workspace_bytes(b, B) for b in splines), dtype=torch.uint8, device=dev)

        def spline_chain():
            for li, b in enumerate(splines):
                lk.bspline_kan_forward(b, acts[li], acts[li + 1], workspace=wsb)

        msb = timed(spline_chain)
        edges = sum(B * s.d * s.m for s in wl.layers)
        rec = {"workload": name, "batch": B, "lut_ms": round(ms, 4), "edge_evals_per_s": round(edges / ms * 1e3, 1),
               "bspline_ms": round(msb, 4), "lut_vs_bspline_speedup": round(msb / ms, 3)}
        if with_oracle:
            rate, rows = oracle_rate(wl)
            rec.update(oracle_edge_evals_per_s=round(rate, 1), oracle_rows=rows)
        rows_out.append(rec)
        log(f"[bench] {name:28s} {B:7d} {ms:9.3f} {edges / ms / 1e6:15.1f} {msb:12.3f} {msb / ms:6.2f} "
            f"{rec.get('oracle_edge_evals_per_s', float('nan')) / 1e9:11.3f}")
        del arts, layers, splines, x, ws, y, acts, wsb
    return rows_out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--batch", type=int, default=32768)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-bspline", action="store_true")
    ap.add_argument("--no-probes", action="store_true", help="skip the peak-rate probes (FMA, instruction mix, LDS, L2, HBM)")
    ap.add_argument("--all-configs", action="store_true",
                    help="also time every workload of the scope table (LUT chain, B-spline chain, bounded oracle sample); "
                         "the results go to extra.configs and, as a table, to stderr")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device-to-device copy, as a known-size reference for HBM counters")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build is single-GPU by design (rows are independent: more GPUs would each run the "
                 "same kernel on B/N rows with replicated tables); run with --gpus 1")

    import numpy as np
    import torch

    import paper_2601_03332_amd as lk
    from lutkan_inputs import cfg4

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    t0 = time.time()
    w = cfg4(seed=0, B=args.batch)
    s = w.layers[0]
    B, d, m = w.x.shape[0], s.d, s.m
    log(f"[bench] inputs generated in {time.time() - t0:.1f}s: {w.name}")
    t0 = time.time()
    art = lk.lutkan_compile(s.d, s.m, s.G, s.p, s.ext_knots, s.coef, s.L, s.scheme, s.boundary, s.oob)
    log(f"[bench] lutkan_compile: {time.time() - t0:.1f}s, table {art.info.table_bytes / 2**20:.0f} MiB, jt={art.info.jt}")
    layer = art.to_device(dev)
    nbuf = 3                                            # rotate buffers so no step re-reads a cache-warm x / y
    xs = [torch.from_numpy(w.x).to(dev)]
    for r in range(1, nbuf):
        xs.append(xs[0].roll(r * 977, dims=0).contiguous())
    ys = [torch.empty((B, m), dtype=torch.float32, device=dev) for _ in range(nbuf)]
    ws = torch.empty(lk.lutkan_forward_workspace_bytes(layer, B), dtype=torch.uint8, device=dev)
    edges = B * d * m

    def step(n):
        lk.lutkan_forward(layer, xs[n % nbuf], ys[n % nbuf], workspace=ws)

    if args.copy_calibration:                           # 2^28 floats read + 2^28 floats written = 1 GiB each way
        ca = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        cb = torch.empty_like(ca)
        for _ in range(3):
            cb.copy_(ca)
        torch.cuda.synchronize()
        del ca, cb

    for n in range(args.warmup):
        step(n)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for n in range(args.steps):
        step(n)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    value = edges / (dt / args.steps)
    log(f"[bench] lutkan_forward: {ms_per_step:.3f} ms/step, {value:.4g} edge-evals/s")

    # Per-kernel durations with HIP events on the stream the kernels are launched on (torch's current stream).
    def time_phases(locate, edge_fn, steps):
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
        for n in range(steps):
            ev[n][0].record()
            locate(n)
            ev[n][1].record()
            edge_fn(n)
            ev[n][2].record()
        torch.cuda.synchronize()
        loc = sorted(e[0].elapsed_time(e[1]) for e in ev)
        edg = sorted(e[1].elapsed_time(e[2]) for e in ev)
        tot = sorted(e[0].elapsed_time(e[2]) for e in ev)
        mean = sum(tot) / len(tot)
        spread = {"median": tot[len(tot) // 2], "mean": mean, "std": (sum((t - mean) ** 2 for t in tot) / len(tot)) ** 0.5,
                  "min": tot[0], "max": tot[-1]}
        return sum(loc) / len(loc), sum(edg) / len(edg), edg[len(edg) // 2], spread

    loc_ms, edge_ms, edge_med, step_spread = time_phases(lambda n: lk.lutkan_forward_locate(layer, xs[n % nbuf], ws),
                                            lambda n: lk.lutkan_forward_edges(layer, B, ys[n % nbuf], ws), args.steps)
    log(f"[bench] locate kernel {loc_ms:.3f} ms, edge kernel {edge_ms:.3f} ms (median {edge_med:.3f})")
    achieved = FLOP_PER_EDGE * edges / (edge_ms * 1e-3) / 1e12
    roofline = {"bound": "alu", "kernel": "lutkan_tiled_kernel", "achieved": round(achieved, 3),
                "peak": round(PEAK_FP32_TFLOPS, 1), "unit": "TFLOP/s", "frac": round(achieved / PEAK_FP32_TFLOPS, 4),
                "traffic": MEASURED_TRAFFIC_BYTES.get(B), "kernel_ms": round(edge_ms, 4),
                "flop_per_edge_eval": FLOP_PER_EDGE, "peak_packed_fp32": PEAK_FP32_PACKED_TFLOPS,
                "compulsory_hbm_bytes": int(art.info.table_bytes + 8 * B * d + 4 * B * m),
                "hbm_time_floor_ms": round((art.info.table_bytes + 8 * B * d + 4 * B * m) / (PEAK_HBM_GBS * 1e9) * 1e3, 4)}

    extra = {"rows_per_s": round(B / (dt / args.steps), 1), "locate_kernel_ms": round(loc_ms, 4),
             "edge_kernel_edge_evals_per_s": round(edges / (edge_ms * 1e-3), 1),
             "step_ms_by_events": {k: round(v, 4) for k, v in step_spread.items()}}

    if not args.no_probes:
        # Rates this GPU sustains on one resource at a time (kernels of known work, timed with events), and what
        # the edge kernel asks of each resource per launch: the largest term is the bound, the others show the slack.
        probe_buf = torch.zeros((1 << 30) // 4 + 4, dtype=torch.float32, device=dev)      # 1 GiB + 16 B, finite floats

        def probe(kind, iters):
            best, work = None, 0.0
            for _ in range(3):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                work = lk.lutkan_probe_launch(kind, probe_buf, iters)
                e1.record()
                torch.cuda.synchronize()
                t = e0.elapsed_time(e1) * 1e-3
                best = t if best is None else min(best, t)
            return work / best

        fma_flops = probe(lk.PROBE_VALU_FMA, 2048)
        mix_rate = probe(lk.PROBE_VALU_MIX, 2048)                # lane-instructions/s of the kernel's own instruction mix
        lds_bps = probe(lk.PROBE_LDS_READ, 512)
        l2_bps = probe(lk.PROBE_L2_READ, 4)
        hbm_bps = probe(lk.PROBE_HBM_READ, 2)
        del probe_buf
        rec_bytes = 8 * (-(-B // 1024) * 1024) * d
        valu_ops = 4.5 * edges                                   # 18 vector instructions per 4 edges (lane-operations)
        lds_bytes = 8.0 * edges                                  # 32 B per lane and row step: record 8, codes 8, scales 16
        l2_bytes = -(-B // 1024) * art.info.table_bytes + art.info.n_tiles * rec_bytes   # slices and records staged into LDS
        hbm_bytes = MEASURED_TRAFFIC_BYTES.get(B) or (art.info.table_bytes + rec_bytes + 4 * B * m)
        # valu: every vector instruction at the FMA issue rate; valu_mix: at the measured rate of the kernel's mix
        # (permutes, packed-fp16 adds and mixed FMAs issue more slowly than plain FMAs on this chip)
        terms = {"valu": valu_ops / (fma_flops / 2.0), "valu_mix": valu_ops / mix_rate, "lds": (lds_bytes + l2_bytes) / lds_bps,
                 "l2": l2_bytes / l2_bps, "hbm": hbm_bytes / hbm_bps}
        binding = max(terms, key=terms.get)
        roofline.update({
            "measured_peaks": {"fp32_fma_TFLOPs": round(fma_flops / 1e12, 2),
                               "kernel_mix_Tlane_instr_s": round(mix_rate / 1e12, 3), "lds_read_TBs": round(lds_bps / 1e12, 2),
                               "l2_read_TBs": round(l2_bps / 1e12, 2), "hbm_read_TBs": round(hbm_bps / 1e12, 2)},
            "terms_ms": {k: round(v * 1e3, 4) for k, v in terms.items()},
            "binding_term": binding,
            "frac_of_measured_bound": round(terms[binding] / (edge_ms * 1e-3), 4)})
        log(f"[bench] measured peaks: FMA {fma_flops / 1e12:.1f} TFLOP/s, LDS {lds_bps / 1e12:.1f} TB/s, "
            f"L2 {l2_bps / 1e12:.1f} TB/s, HBM {hbm_bps / 1e12:.2f} TB/s; edge-kernel terms (ms): "
            + ", ".join(f"{k} {v * 1e3:.2f}" for k, v in terms.items()) + f" -> bound by {binding}")

    if not args.no_bspline:
        bl = art.bspline_to_device(dev)
        wsb = torch.empty(lk.bspline_forward_workspace_bytes(bl, B), dtype=torch.uint8, device=dev)
        for n in range(max(2, args.warmup // 2)):
            lk.bspline_kan_forward(bl, xs[n % nbuf], ys[n % nbuf], workspace=wsb)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for n in range(args.steps):
            lk.bspline_kan_forward(bl, xs[n % nbuf], ys[n % nbuf], workspace=wsb)
        torch.cuda.synchronize()
        bs_ms = (time.perf_counter() - t0) / args.steps * 1e3
        bloc_ms, bedge_ms, _, _ = time_phases(lambda n: lk.bspline_forward_locate(bl, xs[n % nbuf], wsb),
                                           lambda n: lk.bspline_forward_edges(bl, B, ys[n % nbuf], wsb), args.steps)
        extra.update({"bspline_ms_per_step": round(bs_ms, 4), "lut_vs_bspline_speedup": round(bs_ms / ms_per_step, 4),
                      "bspline_locate_kernel_ms": round(bloc_ms, 4), "bspline_edge_kernel_ms": round(bedge_ms, 4),
                      "paper_cpu_speedup_context": "LUT vs B-spline on a Ryzen 7 7840HS, 1 thread: ~12x NumPy, ~10x Numba (Tables 2-3)"})
        log(f"[bench] bspline_kan_forward: {bs_ms:.3f} ms/step -> LUT is {bs_ms / ms_per_step:.2f}x the B-spline layer")
        del wsb

    if not args.no_bspline:
        # The tabular chain 78 -> 16 -> 2 (L = 64 asymmetric uint8): throughput at batch 65536 through the per-layer
        # launches, and latency at batch 256 (the batch of the paper's deployment measurements, Sec. 8) through the
        # per-layer launches and through the fused one-launch chain.
        from lutkan_inputs import cfg2
        w2 = cfg2(seed=0)
        chain = [lk.lutkan_compile(c.d, c.m, c.G, c.p, c.ext_knots, c.coef, c.L, c.scheme, c.boundary, c.oob).to_device(dev)
                 for c in w2.layers]
        x2 = torch.from_numpy(w2.x).to(dev)

        def chain_ms(fn, n=50):
            for _ in range(5):
                fn()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(n):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / n

        B2 = x2.shape[0]
        y2 = torch.empty((B2, 2), dtype=torch.float32, device=dev)
        ws2 = torch.empty(lk.lutkan_model_workspace_bytes(chain, B2), dtype=torch.uint8, device=dev)
        full_ms = chain_ms(lambda: lk.lutkan_model_forward(chain, x2, y2, workspace=ws2))
        xs256, ys256 = x2[:256].contiguous(), y2[:256].contiguous()
        hid256 = torch.empty((256, chain[0].m), dtype=torch.float32, device=dev)

        def layer_by_layer():
            lk.lutkan_forward(chain[0], xs256, hid256, workspace=ws2)
            lk.lutkan_forward(chain[1], hid256, ys256, workspace=ws2)

        layers_ms = chain_ms(layer_by_layer)
        fused_ms = chain_ms(lambda: lk.lutkan_chain_forward(chain, xs256, ys256))
        chain_edges = sum(c.d * c.m for c in w2.layers)
        extra["tabular_chain_78_16_2"] = {"batch_65536_ms": round(full_ms, 4),
                                          "batch_65536_edge_evals_per_s": round(B2 * chain_edges / (full_ms * 1e-3), 1),
                                          "batch_256_per_layer_launches_ms": round(layers_ms, 4),
                                          "batch_256_fused_chain_ms": round(fused_ms, 4)}
        log(f"[bench] 78->16->2: batch {B2} {full_ms:.3f} ms; batch 256: {layers_ms:.4f} ms per-layer launches, "
            f"{fused_ms:.4f} ms fused chain")
        del chain, x2, y2, ws2

    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        t0 = time.time()
        ora = oracle.compile_layer(s.d, s.m, s.G, s.p, s.ext_knots, s.coef, s.L, s.scheme)
        log(f"[bench] oracle compile (not timed into the baseline): {time.time() - t0:.1f}s")
        threads = oracle.default_threads()
        probe = 64
        t0 = time.perf_counter()
        oracle.lut_forward(ora, s.boundary, s.oob, w.x[:probe], nthreads=threads)
        rate = probe / (time.perf_counter() - t0)
        rows = int(min(B, max(probe, rate * 12.0)))      # about 12 s of CPU work
        # a seeded random sample of the batch (sorted), so that every row tile of the launch is represented
        pick = np.sort(np.random.Generator(np.random.PCG64(2601)).choice(B, size=rows, replace=False))
        x_pick = np.ascontiguousarray(w.x[pick])
        t0 = time.perf_counter()
        ref = oracle.lut_forward(ora, s.boundary, s.oob, x_pick, nthreads=threads)
        cdt = time.perf_counter() - t0
        # the same rows on the GPU, as a last parity check of the timed configuration
        yg = ys[0]
        lk.lutkan_forward(layer, xs[0], yg, workspace=ws)
        torch.cuda.synchronize()
        err = np.abs(yg[torch.from_numpy(pick).to(dev)].cpu().numpy().astype(np.float64) - ref.y)
        ok = bool(np.all(err <= 1e-5 * ref.A + 1e-6))
        t0 = time.perf_counter()                              # the paper's protocol is single-threaded (Sec. 6.1)
        oracle.lut_forward(ora, s.boundary, s.oob, w.x[:probe // 2], nthreads=1)
        single = (probe // 2) * d * m / (time.perf_counter() - t0)
        cpu = {"value": round(rows * d * m / cdt, 1), "unit": "edge-evals/s", "cores": threads, "kind": "oracle",
               "sample": f"{rows} of the {B} rows of the same workload, drawn at random (seeded), {cdt:.1f}s", "gpu_matches_oracle_on_sample": ok,
               "single_thread_value": round(single, 1)}
        log(f"[bench] oracle: {rows} rows in {cdt:.1f}s on {threads} threads; GPU within tolerance on them: {ok}; "
            f"one thread: {single:.3g} edge-evals/s")
        del ora, ref

    if args.all_configs:
        del xs, ys, ws, layer, art
        extra["configs"] = time_all_configs(lk, torch, dev, with_oracle=not args.no_cpu_baseline)

    out = {"metric": "lutkan_layer_edge_evals_per_s", "value": round(value, 1), "unit": "edge-evals/s", "n_gpus": 1,
           "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": {"workload": f"cfg4: dense KAN layer {d}->{m}, G={s.G}, k=3, L={s.L} symmetric int8, batch {B}, "
                                  f"x~N(0,0.5) clipped to [-1.2,1.2], closed+clip_x, seed 0",
                      "d": d, "m": m, "K": s.G, "L": s.L, "batch": B, "scheme": "sym_int8"},
           "roofline": roofline, "cpu_baseline": cpu, "extra": extra}
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
