#!/usr/bin/env python3
"""Benchmark of the LUT-KAN layer forward on one MI355X.

One "step" is one pass of the whole hot path (lutkan_model_forward: per layer the locate kernel, the edge kernel and,
where the inputs were split, the summing pass) over one batch of seeded synthetic input that is already resident in
HBM.  The default workload is the largest single-GPU configuration: one dense layer 1024 -> 1024, G = 10 segments
on [-1,1], cubic splines with N(0,1) coefficients compiled to L = 64 symmetric int8 tables, batch 32768 rows of
x ~ N(0, 0.5) clipped to [-1.2, 1.2], closed + clip_x.  --workload names any other workload of the scope table.

Prints ONE JSON line: edge-evaluations/s (batch*d*m per second, summed over the layers), the roofline record of the
dominant kernel measured with HIP events on the launch stream, what one forward asks of each resource (HBM, L2, LDS,
vector ALU) priced at published / derived peaks and at rates measured in the same run, the B-spline baseline ratio,
and the CPU oracle timed on a bounded random sample of the same rows.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# ---- peaks.  "derived" = from the unit counts and the clock, not a published figure.
# fp32 vector rate WITHOUT the packed-fp32 forms (this library is built with them disabled):
# 256 CUs x 4 SIMDs x 16 lanes x 2 flop (FMA) x 2.4 GHz = 78.6 TFLOP/s (derived).  Published, with packed forms: 157.3.
PEAK_FP32_TFLOPS = 256 * 4 * 16 * 2 * 2.4e9 / 1e12
PEAK_FP32_PACKED_TFLOPS = 157.3
PEAK_LANE_INSTR = 256 * 4 * 16 * 2.4e9            # vector lane-instructions/s at one wave instruction per 4 cycles (derived)
PEAK_HBM_BPS = 8.0e12                              # published
PEAK_LDS_BPS = 256 * 256 * 2.4e9                   # 256 B per clock and compute unit (derived)
# Algorithmic fp32 operations per edge evaluation (Eq. 10 twice: 2 mul + 2 add; Eq. 17: 2 mul + 1 add;
# Eq. 1: 1 add).  Integer->float conversions, address arithmetic and the 1-w subtraction are not counted.
FLOP_PER_EDGE = 8
TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "hbm_traffic_per_launch.md")


def log(msg):
    print(msg, file=sys.stderr, flush=True)


# ------------------------------------------------------------------------------------------------ workloads
def workload_names():
    names = ["cfg1", "cfg2"]
    names += [f"cfg3_L{L}_{sc}" for sc in ("sym", "asym") for L in (16, 32, 64, 128)]
    names += ["cfg4_B256", "cfg4_B4096", "cfg4_B32768"]
    names += [f"cfg5_{b}_{o}" for b in ("closed", "half_open") for o in ("clip_x", "zero_spline")]
    return names


def make_workload(name, batch=None):
    """The seeded synthetic workload `name` of the scope table (lutkan_inputs); batch overrides its row count."""
    import lutkan_inputs as li
    kw = {} if batch is None else {"B": batch}
    if name == "cfg1":
        return li.cfg1(**kw)
    if name == "cfg2":
        return li.cfg2(**kw)
    mt = re.fullmatch(r"cfg3_L(\d+)_(sym|asym)", name)
    if mt:
        return li.cfg3(L=int(mt.group(1)), scheme=li.SYM_INT8 if mt.group(2) == "sym" else li.ASYM_UINT8, **kw)
    mt = re.fullmatch(r"cfg4_B(\d+)", name)
    if mt:
        return li.cfg4(B=batch or int(mt.group(1)))
    mt = re.fullmatch(r"cfg5_(closed|half_open)_(clip_x|zero_spline)", name)
    if mt:
        return li.cfg5(boundary=li.CLOSED if mt.group(1) == "closed" else li.HALF_OPEN,
                       oob=li.CLIP_X if mt.group(2) == "clip_x" else li.ZERO_SPLINE, **kw)
    sys.exit(f"bench.py: unknown workload {name!r}; known: {', '.join(workload_names())}")


# ------------------------------------------------------------------------------------------------ cost model
def kernel_costs(info, spec, B, plan):
    """What each kernel launch of one lutkan_forward call must move and compute, from the layer's shape and the launch
    plan the library reports (lutkan_last_plan): a list of dicts {kernel, hbm, l2, lds, valu[, valu2]} in bytes resp. vector
    lane-instructions (valu2: those in the two-operand fp32 encoding on registers, priced at their own rate).  hbm = compulsory bytes (every operand once); l2 = bytes staged from L2 into LDS, or read
    through L2 by the kernels that gather from global memory; lds = bytes the lanes read from LDS plus the staged
    bytes written into it; valu = lane-instructions of the inner loops (counted for the tiled kernel, estimated for
    the kernels that are bound by memory latency)."""
    d, m, K = spec.d, spec.m, info.K
    asym = (info.scheme == 1)
    base_product = "base_product" in plan                       # the base branch runs as a matrix product of its own
    base = (info.value_repr == 1) and not base_product         # ... else inside the edge kernel
    rec = 16 if base else 8
    prm = (8 if asym else 4) + (4 if base else 0)               # parameter bytes per edge
    Bp = -(-B // 1024) * 1024
    edges = B * d * m
    out = []
    last_split = 1
    for clause in [c.strip() for c in plan.split(";") if c.strip()]:
        nums = [int(v) for v in re.findall(r"=(\d+)", clause)]
        if clause == "locate":
            # about 30 + K vector instructions per (row, input): domain test, clip, K-1 compares, divide, floor, record
            silu_plane = 4 * B * d if (info.value_repr == 1 and "base_product" in plan) else 0
            out.append(dict(kernel="lutkan_locate_kernel", hbm=4 * B * d + rec * Bp * d + silu_plane, l2=0, lds=2 * rec * Bp * d,
                            valu=(30 + K) * B * d))
        elif clause.startswith("tiled"):
            np_, last_split = nums[:2]                                   # (the third number is the pipeline mode)
            # a wide form of the table: 16-bit codes (code rows twice as long), or fp32 values (four times, no parameter rows)
            wide = 4 if clause.startswith("tiled wide32") else 2 if clause.startswith("tiled wide") else 0
            rows_per_group = 16 * (64 // (info.jt // 4)) * np_
            code_bytes_all = info.n_tiles * d * (K * info.L + 2) * info.jt
            param_bytes_all = info.n_tiles * d * (K + 1) * info.jt * (8 if asym else 4)
            table_bytes = info.table_bytes + (3 * code_bytes_all - param_bytes_all if wide == 4 else code_bytes_all if wide else 0)
            staged = -(-B // rows_per_group) * table_bytes + info.n_tiles * rec * Bp * d
            # vector instructions per 4 edges: two addresses, [four byte permutes, two bias removals (int8)], two code
            # differences, four interpolations, four scalings [, four y_min] [, four base products]; on fp32 values one
            # address, four differences, four interpolations, four additions
            per4 = (13 if wide == 4 else (16 if asym else 12) if wide else (20 if asym else 18)) + (4 if base else 0)
            # record, two code rows, alpha (+ y_min) per lane
            lds_per4 = (12 if base else 8) + (32 if wide == 4 else (16 if wide else 8) + (32 if asym else 16))
            # on fp32 values all but the address instruction are two-operand fp32 instructions on registers, which
            # issue about twice as fast as the rest: counted apart (valu2) and priced at their own rate
            valu2 = edges / 4 * 12 if wide == 4 else 0
            out.append(dict(kernel="lutkan_tiled_kernel", hbm=table_bytes + rec * Bp * d + 4 * B * m * last_split,
                            l2=staged, lds=edges / 4 * lds_per4 + staged, valu=edges / 4 * per4 - valu2, valu2=valu2))
        elif clause.startswith("gather"):
            last_split = nums[0]
            touched = min(info.table_bytes, B * d * info.n_tiles * info.jt * (2 + prm))
            out.append(dict(kernel="lutkan_gather_kernel", hbm=touched + rec * Bp * d + 4 * B * m * last_split,
                            l2=edges * (2 + prm + rec), lds=0, valu=edges * 14))
        elif clause == "base_product":
            # SiLU(X) [B, d] times s_out*s_base [d, m] on the matrix cores, fp32 operands as three bf16 pieces each, six
            # piece products: not priced against the vector ALU (its conversions are, roughly 12 instructions per operand element)
            tiles = -(-B // 128) * -(-m // 128)
            out.append(dict(kernel="lutkan_base_gemm_kernel", hbm=4 * B * d + 4 * d * m + 4 * B * m, l2=tiles * 4 * 128 * 2 * d,
                            lds=tiles * (d / 32) * (2 * 61440), valu=tiles * 2 * 128 * d * 12, mfma_flop=12.0 * B * d * m))
        elif clause == "sum":
            out.append(dict(kernel="sum_partials_kernel", hbm=4 * B * m * (last_split + 1), l2=0, lds=0, valu=B * m * last_split / 4))
        elif clause.startswith("chain"):
            touched = min(info.table_bytes, B * d * info.jt * (2 + prm))
            out.append(dict(kernel="lutkan_chain_kernel", hbm=touched + 4 * B * (d + m), l2=edges * (2 + prm),
                            lds=16 * B * d * (1 + max(1, m)), valu=edges * 14 + (30 + K) * B * d))
    return out


def price(costs, rates):
    """Lower bound of one forward = sum over its kernels of the largest of that kernel's resource times; the binding
    resource is the one that contributes most to that sum."""
    rates = dict(rates)
    rate2 = rates.pop("valu2")
    total, by_resource, share = 0.0, {r: 0.0 for r in rates}, {r: 0.0 for r in rates}
    for c in costs:
        t = {r: c[r] / rates[r] for r in rates}
        t["valu"] += c.get("valu2", 0) / rate2                # the same issue port: the two classes add up
        worst = max(t, key=t.get)
        total += t[worst]
        share[worst] += t[worst]
        for r in rates:
            by_resource[r] += t[r]
    return total, by_resource, max(share, key=share.get)


def traffic_from_profiles(workload, kernel):
    """HBM bytes per launch of `kernel` on `workload` as rocprofv3 counted them (FETCH_SIZE and WRITE_SIZE, scaled by
    a plain copy of known size), read from the table of the committed profile summary; None when it has no such row."""
    try:
        for line in open(TRAFFIC_TABLE):
            cells = [c.strip().strip("`") for c in line.strip().strip("|").split("|")]
            if len(cells) >= 5 and cells[0] == workload and cells[1] == kernel:
                return float(cells[4]), os.path.relpath(TRAFFIC_TABLE, ROOT) + " (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE)"
    except (OSError, ValueError):
        pass
    return None, None


# ------------------------------------------------------------------------------------------------ measurement
class Rig:
    """Shared state of one bench process: torch, the binding, the device and the measured peak rates."""

    def __init__(self, probes=True):
        import numpy as np
        import torch

        import paper_2601_03332_amd as lk
        assert torch.cuda.is_available(), "bench.py needs a GPU"
        self.np, self.torch, self.lk, self.dev = np, torch, lk, "cuda:0"
        self.measured = self.measure_peaks() if probes else None

    def events(self):
        return self.torch.cuda.Event(enable_timing=True), self.torch.cuda.Event(enable_timing=True)

    def measure_peaks(self):
        """Rates this GPU sustains on one resource at a time (kernels of known work, best of three, HIP events)."""
        torch, lk = self.torch, self.lk
        buf = torch.zeros((1 << 30) // 4 + 4, dtype=torch.float32, device=self.dev)      # 1 GiB + 16 B, finite floats

        def probe(kind, iters):
            best, work = None, 0.0
            for _ in range(3):
                e0, e1 = self.events()
                e0.record()
                work = lk.lutkan_probe_launch(kind, buf, iters)
                e1.record()
                torch.cuda.synchronize()
                t = e0.elapsed_time(e1) * 1e-3
                best = t if best is None else min(best, t)
            return work / best

        fma = probe(lk.PROBE_VALU_FMA, 2048)
        rates = {"fp32_fma_flops": fma, "fp32_fmac_two_operand_flops": probe(lk.PROBE_VALU_FMAC, 2048),
                 "kernel_mix_lane_instr": probe(lk.PROBE_VALU_MIX, 2048),
                 "lds_read_Bps": probe(lk.PROBE_LDS_READ, 512), "l2_read_Bps": probe(lk.PROBE_L2_READ, 4),
                 "hbm_read_Bps": probe(lk.PROBE_HBM_READ, 2)}
        del buf
        log("[bench] measured peaks: FMA %.1f TFLOP/s (two-operand form on registers: %.1f), kernel mix %.1f T lane-instr/s, "
            "LDS %.1f TB/s, L2 %.1f TB/s, HBM %.2f TB/s"
            % (fma / 1e12, rates["fp32_fmac_two_operand_flops"] / 1e12, rates["kernel_mix_lane_instr"] / 1e12,
               rates["lds_read_Bps"] / 1e12, rates["l2_read_Bps"] / 1e12, rates["hbm_read_Bps"] / 1e12))
        return rates


def run_workload(rig, name, steps, warmup, batch=None, bspline=True, cpu_baseline=True, oracle_seconds=12.0, wide=None):
    """Times `name` and returns its record: throughput of the whole forward, per-kernel durations, roofline terms."""
    np, torch, lk, dev = rig.np, rig.torch, rig.lk, rig.dev
    t0 = time.time()
    wl = make_workload(name, batch)
    B = wl.x.shape[0]
    arts = [lk.lutkan_compile(s.d, s.m, s.G, s.p, s.ext_knots, s.coef, s.L, s.scheme, s.boundary, s.oob) for s in wl.layers]
    layers = [a.to_device(dev, wide=wide) for a in arts]
    log(f"[bench] {name}: {wl.name}; inputs and tables ready in {time.time() - t0:.1f}s "
        f"(tables {sum(a.info.table_bytes for a in arts) / 2**20:.1f} MiB)")
    edges = sum(B * s.d * s.m for s in wl.layers)
    nbuf = 3                                            # rotate buffers so no step re-reads a cache-warm x / y
    xs = [torch.from_numpy(wl.x).to(dev)]
    for r in range(1, nbuf):
        xs.append(xs[0].roll(r * 977, dims=0).contiguous())
    ys = [torch.empty((B, layers[-1].m), dtype=torch.float32, device=dev) for _ in range(nbuf)]
    ws = torch.empty(max(256, lk.lutkan_model_workspace_bytes(layers, B)), dtype=torch.uint8, device=dev)

    def step(n):
        lk.lutkan_model_forward(layers, xs[n % nbuf], ys[n % nbuf], workspace=ws)

    for n in range(warmup):
        step(n)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for n in range(steps):
        step(n)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / steps
    model_plan = lk.lutkan_last_plan()
    # the same steps by HIP events on the launch stream, one pair per step: spread of the step time
    ev = [rig.events() for _ in range(steps)]
    for n in range(steps):
        ev[n][0].record()
        step(n)
        ev[n][1].record()
    torch.cuda.synchronize()
    per_step = sorted(a.elapsed_time(b) for a, b in ev)
    mean = sum(per_step) / steps
    spread = {"median": per_step[steps // 2], "mean": mean, "std": (sum((t - mean) ** 2 for t in per_step) / steps) ** 0.5,
              "min": per_step[0], "max": per_step[-1]}
    log(f"[bench] {name}: lutkan_model_forward {dt * 1e3:.4f} ms/step, {edges / dt:.4g} edge-evals/s  [{model_plan.strip()}]")

    # ---- per layer: which kernels a forward launches, and their durations (HIP events around the two phases)
    acts = [xs[0]] + [torch.empty((B, l.m), dtype=torch.float32, device=dev) for l in layers]
    kernels, costs = [], []
    n_ev = max(5, min(steps, 50))
    for li, (layer, art, spec) in enumerate(zip(layers, arts, wl.layers)):
        lk.lutkan_forward(layer, acts[li], acts[li + 1], workspace=ws)
        plan = lk.lutkan_last_plan()
        costs += kernel_costs(art.info, spec, B, plan)
        if plan.startswith("chain"):                    # one launch: the whole call is the kernel
            evs = [rig.events() for _ in range(n_ev)]
            for a, b in evs:
                a.record()
                lk.lutkan_forward(layer, acts[li], acts[li + 1], workspace=ws)
                b.record()
            torch.cuda.synchronize()
            kernels.append({"layer": li, "kernel": "lutkan_chain_kernel", "ms": sum(a.elapsed_time(b) for a, b in evs) / n_ev,
                            "plan": plan.strip()})
            continue
        evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(n_ev)]
        for e in evs:
            e[0].record()
            lk.lutkan_forward_locate(layer, acts[li], ws)
            e[1].record()
            lk.lutkan_forward_edges(layer, B, acts[li + 1], ws)
            e[2].record()
        torch.cuda.synchronize()
        edge_plan = lk.lutkan_last_plan()
        assert edge_plan == plan.replace("locate; ", ""), (plan, edge_plan)
        edge_name = "lutkan_tiled_kernel" if "tiled" in plan else "lutkan_gather_kernel"
        kernels.append({"layer": li, "kernel": "lutkan_locate_kernel", "ms": sum(e[0].elapsed_time(e[1]) for e in evs) / n_ev,
                        "plan": "locate"})
        kernels.append({"layer": li, "kernel": edge_name + (" + sum_partials_kernel" if "sum" in plan else ""),
                        "ms": sum(e[1].elapsed_time(e[2]) for e in evs) / n_ev, "plan": edge_plan.strip()})
    dominant = max(kernels, key=lambda k: k["ms"])
    dspec, dart = wl.layers[dominant["layer"]], arts[dominant["layer"]]
    dom_costs = kernel_costs(dart.info, dspec, B, dominant["plan"])
    dom_edges = B * dspec.d * dspec.m

    # ---- roofline terms of the whole forward
    published = {"hbm": PEAK_HBM_BPS, "lds": PEAK_LDS_BPS, "valu": PEAK_LANE_INSTR, "valu2": 2 * PEAK_LANE_INSTR}
    t_pub, by_pub, bind_pub = price(costs, published)
    terms = {"at_published_or_derived_peaks_ms": {k: round(v * 1e3, 5) for k, v in by_pub.items()},
             "lower_bound_at_peaks_ms": round(t_pub * 1e3, 5), "binding_at_peaks": bind_pub,
             "frac_of_bound_at_peaks": round(t_pub / dt, 4),
             "work": {r: float(sum(c.get(r, 0) for c in costs)) for r in ("hbm", "l2", "lds", "valu", "valu2")},
             "peaks": {"hbm_Bps_published": PEAK_HBM_BPS, "lds_Bps_derived": PEAK_LDS_BPS, "valu_lane_instr_derived": PEAK_LANE_INSTR,
                       "valu2_lane_instr_derived": 2 * PEAK_LANE_INSTR}}
    if rig.measured:
        ms = rig.measured
        measured = {"hbm": ms["hbm_read_Bps"], "l2": ms["l2_read_Bps"], "lds": ms["lds_read_Bps"], "valu": ms["fp32_fma_flops"] / 2.0,
                    "valu2": ms["fp32_fmac_two_operand_flops"] / 2.0}
        t_ms, by_ms, bind_ms = price(costs, measured)
        t_mix, by_mix, _ = price(costs, dict(measured, valu=ms["kernel_mix_lane_instr"]))
        terms.update({"at_measured_rates_ms": {k: round(v * 1e3, 5) for k, v in by_ms.items()},
                      "valu_at_kernel_mix_rate_ms": round(by_mix["valu"] * 1e3, 5),
                      "lower_bound_at_measured_rates_ms": round(t_ms * 1e3, 5), "binding_at_measured_rates": bind_ms,
                      "frac_of_bound_at_measured_rates": round(t_ms / dt, 4),
                      "frac_of_bound_with_kernel_mix_rate": round(t_mix / dt, 4),
                      "measured_rates": {k: float(f"{v:.4g}") for k, v in ms.items()}})

    # ---- roofline record of the dominant kernel
    k_s = dominant["ms"] * 1e-3
    hbm_bytes = sum(c["hbm"] for c in dom_costs)
    t_dom = {"hbm": hbm_bytes / PEAK_HBM_BPS,
             "valu": sum(c["valu"] + c.get("valu2", 0) / 2 for c in dom_costs) / PEAK_LANE_INSTR,
             "lds": sum(c["lds"] for c in dom_costs) / PEAK_LDS_BPS}
    traffic, source = traffic_from_profiles(name, dominant["kernel"].split(" + ")[0])
    if max(t_dom, key=t_dom.get) == "hbm":
        achieved = hbm_bytes / k_s / 1e9
        roofline = {"bound": "hbm", "kernel": dominant["kernel"], "achieved": round(achieved, 1), "peak": PEAK_HBM_BPS / 1e9,
                    "unit": "GB/s", "frac": round(achieved / (PEAK_HBM_BPS / 1e9), 4)}
    else:
        achieved = FLOP_PER_EDGE * dom_edges / k_s / 1e12
        roofline = {"bound": "alu", "kernel": dominant["kernel"], "achieved": round(achieved, 3), "peak": round(PEAK_FP32_TFLOPS, 1),
                    "unit": "TFLOP/s", "frac": round(achieved / PEAK_FP32_TFLOPS, 4),
                    "peak_is": "derived: 256 CUs x 4 SIMDs x 16 lanes x 2 flop x 2.4 GHz, the 4-cycle issue rate that every instruction of "
                               "this kernel but its four fp32 FMAs per row step has (measured_rates: the FMA in its two-operand "
                               "encoding alone issues faster); the packed-fp32 forms are not used",
                    "peak_published_packed_fp32": PEAK_FP32_PACKED_TFLOPS,
                    "frac_vs_published_packed_fp32": round(achieved / PEAK_FP32_PACKED_TFLOPS, 4),
                    "flop_per_edge_eval": FLOP_PER_EDGE}
    if "wide32" in dominant["plan"]:
        roofline["note"] = ("this launch reads the table's fp32-value form: Eq. 10 was applied when that table was built, so 5 of the "
                            "8 algorithmic flops per edge evaluation execute in the kernel (13 vector instructions per 4 edges); "
                            "'achieved' counts all 8; at derived peaks the model gives this launch %.4f ms of vector instructions "
                            "and %.4f ms of LDS traffic: the LDS is its nearest bound" % (t_dom["valu"] * 1e3, t_dom["lds"] * 1e3))
    roofline.update({"traffic": traffic, "traffic_source": source, "kernel_ms": round(dominant["ms"], 5), "layer": dominant["layer"],
                     "launch_plan": dominant["plan"], "compulsory_hbm_bytes": int(hbm_bytes),
                     "hbm_time_floor_ms": round(hbm_bytes / PEAK_HBM_BPS * 1e3, 5), "terms": terms})

    rec = {"workload": name, "description": wl.name, "batch": B, "layers": [[s.d, s.m] for s in wl.layers],
           "ms_per_step": round(dt * 1e3, 5), "edge_evals_per_s": round(edges / dt, 1), "rows_per_s": round(B / dt, 1),
           "launch_plan": model_plan.strip(), "step_ms_by_events": {k: round(v, 5) for k, v in spread.items()},
           "kernels": [dict(k, ms=round(k["ms"], 5)) for k in kernels], "roofline": roofline}

    if bspline:
        splines = [a.bspline_to_device(dev) for a in arts]
        wsb = torch.empty(max(lk.bspline_forward_workspace_bytes(b, B) for b in splines), dtype=torch.uint8, device=dev)

        def spline_chain():
            for li, b in enumerate(splines):
                lk.bspline_kan_forward(b, acts[li], acts[li + 1], workspace=wsb)

        n_b = max(3, min(steps, 50))
        for _ in range(max(2, min(warmup, 10))):
            spline_chain()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n_b):
            spline_chain()
        torch.cuda.synchronize()
        bs = (time.perf_counter() - t0) / n_b
        rec.update({"bspline_ms_per_step": round(bs * 1e3, 5), "lut_vs_bspline_speedup": round(bs / dt, 4)})
        log(f"[bench] {name}: B-spline layers {bs * 1e3:.4f} ms/step -> LUT is {bs / dt:.2f}x the B-spline chain")
        del splines, wsb

    if cpu_baseline:
        import oracle
        oras = [oracle.compile_layer(s.d, s.m, s.G, s.p, s.ext_knots, s.coef, s.L, s.scheme) for s in wl.layers]
        threads = oracle.default_threads()
        per_row = sum(s.d * s.m for s in wl.layers)

        def chain(x, nthreads):
            outs = []
            for o, s in zip(oras, wl.layers):
                outs.append(oracle.lut_forward(o, s.boundary, s.oob, x, nthreads=nthreads))
                x = outs[-1].y
            return outs

        probe = min(B, 64)
        t0 = time.perf_counter()
        chain(wl.x[:probe], threads)
        rate = probe / (time.perf_counter() - t0)
        rows = int(min(B, max(probe, rate * oracle_seconds)))
        # a seeded random sample of the batch (sorted), so that every row tile of the launch is represented
        pick = np.sort(np.random.Generator(np.random.PCG64(2601)).choice(B, size=rows, replace=False))
        x_pick = np.ascontiguousarray(wl.x[pick])
        t0 = time.perf_counter()
        ref = chain(x_pick, threads)
        cdt = time.perf_counter() - t0
        # the same rows on the GPU at the timed batch, layer by layer on the oracle's own activations
        pick_t = torch.from_numpy(pick).to(dev)
        ok, cur = True, xs[0]
        for li, layer in enumerate(layers):
            if li > 0:
                cur = torch.zeros((B, layer.d), dtype=torch.float32, device=dev)
                cur[pick_t] = torch.from_numpy(ref[li - 1].y).to(dev)
            yg = lk.lutkan_forward(layer, cur, workspace=ws)
            torch.cuda.synchronize()
            err = np.abs(yg[pick_t].cpu().numpy().astype(np.float64) - ref[li].y)
            ok = ok and bool(np.all(err <= 1e-5 * ref[li].A + 1e-6))
        n1 = max(1, min(rows, probe // 2))              # the paper's protocol is single-threaded (Sec. 6.1)
        t0 = time.perf_counter()
        chain(wl.x[:n1], 1)
        single = n1 * per_row / (time.perf_counter() - t0)
        rec["cpu_baseline"] = {"value": round(rows * per_row / cdt, 1), "unit": "edge-evals/s", "cores": threads, "kind": "oracle",
                               "sample": f"{rows} of the {B} rows of the same workload, drawn at random (seeded), {cdt:.1f}s",
                               "gpu_matches_oracle_on_sample": ok, "single_thread_value": round(single, 1)}
        log(f"[bench] {name}: oracle {rows} rows in {cdt:.1f}s on {threads} threads ({rows * per_row / cdt:.3g} edge-evals/s); "
            f"GPU within tolerance on them: {ok}; one thread: {single:.3g} edge-evals/s")
        del oras, ref
    del layers, arts, xs, ys, ws, acts
    torch.cuda.empty_cache()
    return rec


def tabular_chain_latency(rig):
    """The tabular chain 78 -> 16 -> 2 at batch 256 (the batch of the paper's deployment measurements, Sec. 8): per-layer
    launches against the fused one-launch chain."""
    torch, lk, dev = rig.torch, rig.lk, rig.dev
    w2 = make_workload("cfg2", 256)
    chain = [lk.lutkan_compile(c.d, c.m, c.G, c.p, c.ext_knots, c.coef, c.L, c.scheme, c.boundary, c.oob).to_device(dev)
             for c in w2.layers]
    x = torch.from_numpy(w2.x).to(dev)
    y = torch.empty((256, 2), dtype=torch.float32, device=dev)
    hid = torch.empty((256, chain[0].m), dtype=torch.float32, device=dev)
    ws = torch.empty(max(256, lk.lutkan_model_workspace_bytes(chain, 256)), dtype=torch.uint8, device=dev)

    def ms(fn, n=200):
        for _ in range(20):
            fn()
        e0, e1 = rig.events()
        e0.record()
        for _ in range(n):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n

    def layer_by_layer():
        lk.lutkan_forward(chain[0], x, hid, workspace=ws)
        lk.lutkan_forward(chain[1], hid, y, workspace=ws)

    return {"batch_256_per_layer_launches_ms": round(ms(layer_by_layer), 5),
            "batch_256_fused_chain_ms": round(ms(lambda: lk.lutkan_chain_forward(chain, x, y)), 5)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200, help="timed steps (default: the 200 of Sec. 6.4's protocol)")
    ap.add_argument("--warmup", type=int, default=50, help="untimed warm-up steps (default: the 50 of Sec. 6.4's protocol)")
    ap.add_argument("--workload", default="cfg4_B32768", help="one of: " + ", ".join(workload_names()))
    ap.add_argument("--batch", type=int, default=None, help="override the workload's number of rows")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-bspline", action="store_true")
    ap.add_argument("--no-wide-tables", action="store_true", help="byte form of the LUT table only (no second copy with 16-bit codes or fp32 values)")
    ap.add_argument("--no-probes", action="store_true", help="skip the peak-rate probes (FMA, instruction mix, LDS, L2, HBM)")
    ap.add_argument("--all-configs", action="store_true",
                    help="also run every workload of the scope table; their records (throughput, kernels, roofline terms, "
                         "B-spline ratio, bounded oracle sample) go to extra.configs and, as a table, to stderr")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device-to-device copy, as a known-size reference for HBM counters")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build is single-GPU by design (rows are independent: more GPUs would each run the "
                 "same kernel on B/N rows with replicated tables); run with --gpus 1")
    if args.steps < 1 or args.warmup < 0:
        sys.exit("bench.py: --steps must be >= 1 and --warmup >= 0")
    if args.workload not in workload_names():
        sys.exit(f"bench.py: unknown workload {args.workload!r}; known: {', '.join(workload_names())}")

    rig = Rig(probes=not args.no_probes)
    torch = rig.torch
    if args.copy_calibration:                           # 2^28 floats read + 2^28 floats written = 1 GiB each way
        ca = torch.empty(1 << 28, dtype=torch.float32, device=rig.dev).normal_()
        cb = torch.empty_like(ca)
        for _ in range(3):
            cb.copy_(ca)
        torch.cuda.synchronize()
        del ca, cb

    wide = False if args.no_wide_tables else None      # None: the binding's default (layers of some size that have a wide form)
    rec = run_workload(rig, args.workload, args.steps, args.warmup, batch=args.batch, wide=wide, bspline=not args.no_bspline,
                       cpu_baseline=not args.no_cpu_baseline)
    extra = {k: rec[k] for k in ("rows_per_s", "launch_plan", "step_ms_by_events", "kernels", "bspline_ms_per_step",
                                 "lut_vs_bspline_speedup") if k in rec}
    if "lut_vs_bspline_speedup" in rec:
        extra["paper_cpu_speedup_context"] = "LUT vs B-spline on a Ryzen 7 7840HS, 1 thread: ~12x NumPy, ~10x Numba (Tables 2-3)"
        extra["tabular_chain_78_16_2"] = tabular_chain_latency(rig)

    if args.all_configs:
        configs = []
        log(f"[bench] {'workload':26s} {'B':>7s} {'LUT ms':>9s} {'G edge-evals/s':>15s} {'B-spline ms':>12s} {'ratio':>6s} "
            f"{'bound':>6s} {'frac@peaks':>10s} {'frac@measured':>13s} {'oracle G/s':>11s}")
        for name in workload_names():
            r = rec if (name == args.workload and args.batch is None) else run_workload(
                rig, name, args.steps, args.warmup, wide=wide, bspline=not args.no_bspline,       # the same protocol for every workload
                cpu_baseline=not args.no_cpu_baseline, oracle_seconds=3.0)
            configs.append(r)
            t = r["roofline"]["terms"]
            log(f"[bench] {name:26s} {r['batch']:7d} {r['ms_per_step']:9.4f} {r['edge_evals_per_s'] / 1e9:15.1f} "
                f"{r.get('bspline_ms_per_step', float('nan')):12.4f} {r.get('lut_vs_bspline_speedup', float('nan')):6.2f} "
                f"{t.get('binding_at_measured_rates', t['binding_at_peaks']):>6s} {t['frac_of_bound_at_peaks']:10.3f} "
                f"{t.get('frac_of_bound_at_measured_rates', float('nan')):13.3f} "
                f"{r.get('cpu_baseline', {}).get('value', float('nan')) / 1e9:11.3f}")
        extra["configs"] = configs

    config = {"workload": f"{args.workload}: {rec['description']}, batch {rec['batch']}, seed 0", "layers": rec["layers"], "batch": rec["batch"]}
    if len(rec["layers"]) == 1:
        s0 = make_workload(args.workload, 1).layers[0]
        config.update({"d": s0.d, "m": s0.m, "K": s0.G, "L": s0.L, "scheme": "sym_int8" if s0.scheme == 0 else "asym_uint8"})
    out = {"metric": "lutkan_layer_edge_evals_per_s", "value": rec["edge_evals_per_s"], "unit": "edge-evals/s", "n_gpus": 1,
           "steps": args.steps, "warmup": args.warmup, "ms_per_step": rec["ms_per_step"], "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic", "config": config,
           "roofline": rec["roofline"], "cpu_baseline": rec.get("cpu_baseline"), "extra": extra}
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
