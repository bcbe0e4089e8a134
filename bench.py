#!/usr/bin/env python3
"""Throughput of the banded local-operator chain on one MI355X.

One "step" is one pass of the whole hot path over one batch: plan-driven kernels for every
band and layer plus the per-band device-to-host copies, pipelined (band b's copy under band
b+1's kernels, and the last copy under the next step's first band). Inputs are resident in
HBM before the timed region. Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK = {"mfma_f32": 157.3, "mfma_bf16": 2500.0, "hbm": 8000.0}   # TFLOP/s, TFLOP/s, GB/s


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="resnet18")
    ap.add_argument("--also", default="resnet18:independent,tiny,vgg16,detector720p,mbv2,mlp",
                    help="comma list of further workload[:mode] entries reported under 'also' "
                         "(fewer steps; mode defaults to --mode)")
    ap.add_argument("--bands", type=int, default=None, help="override the workload's band count")
    ap.add_argument("--lanes", type=int, default=0, help="concurrent band streams (0 = library default)")
    ap.add_argument("--graph", type=int, default=1, help="1: replay the chain as a HIP graph")
    ap.add_argument("--dma-copy", type=int, default=0, help="1: band copies via hipMemcpyAsync")
    ap.add_argument("--replicas", type=int, default=1,
                    help="plans (each with its own lanes and scratch) the steady-state steps rotate over")
    ap.add_argument("--mode", default="reuse", choices=["independent", "reuse"],
                    help="independent: every band recomputes its halos; reuse: bands run in "
                         "order and reuse rows earlier bands produced")
    ap.add_argument("--pmc-calibrate", action="store_true",
                    help="also run a plain 256 MiB device-to-device copy (torch) a few times so "
                         "that a counter run can be scaled by a kernel of known traffic")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-reference-points", action="store_true",
                    help="skip the one-band run and the measured HBM / MFMA ceilings")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    ap.add_argument("--profile-iters", type=int, default=10)
    return ap.parse_args()


def device_tensors(torch, chain, tensors, plan, n_buf=2):
    import numpy as np
    if tensors.x.ndim == 2:   # a matrix of a row-wise chain: already row-major m x k
        x = torch.from_numpy(tensors.x)
    else:
        x = torch.from_numpy(np.ascontiguousarray(tensors.x.transpose(0, 2, 3, 1)))
    td = torch.bfloat16 if chain.dtype == "bf16" else torch.float32
    d_in = x.to(td).cuda()
    n, c, h, w = plan.out_shape()
    d_out = [torch.zeros((n, h, w, c), dtype=td, device="cuda") for _ in range(n_buf)]
    h_out = [torch.zeros((n, h, w, c), dtype=td, pin_memory=True) for _ in range(n_buf)]
    torch.cuda.synchronize()
    return d_in, d_out, h_out


def timed_steps(torch, plans, d_in, d_out, h_out, steps, warmup, copy=True):
    """Steady state: `steps` chains back to back; step i uses plan i % R and its own output
    buffers, so with R > 1 consecutive images overlap on the GPU."""
    R = len(plans)
    for i in range(warmup):
        plans[i % R].run_chain(d_in, d_out[i % len(d_out)], h_out[i % len(d_out)] if copy else None)
    for p in plans:
        p.synchronize()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        plans[i % R].run_chain(d_in, d_out[i % len(d_out)], h_out[i % len(d_out)] if copy else None)
    for p in plans:
        p.synchronize()
    torch.cuda.synchronize()
    return time.perf_counter() - t0


def timed_copies(torch, plan, d_out, h_out, steps, warmup):
    for i in range(warmup):
        plan.copy_chain(d_out[i % 2], h_out[i % 2])
    plan.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        plan.copy_chain(d_out[i % 2], h_out[i % 2])
    plan.synchronize()
    return time.perf_counter() - t0


def kernel_table(plan, d_in, d_out, iters, dtype):
    """Per kernel instance (named as rocprofv3 prints it): launches per chain, mean duration
    from a start and a stop HIP event attached to every dispatch on its stream (the kernel's
    own duration, as a profiler's kernel trace reports it), algorithmic work. The finish kernel
    of a split-K convolution is listed on its own; the layer's algorithmic FLOP and bytes
    are booked on the convolution kernel."""
    ms, fin = plan.profile_chain(d_in, d_out, iters)
    groups = {}

    def add(name, t, flop, byts):
        g = groups.setdefault(name, dict(name=name, launches=0, ms=0.0, flop=0.0, bytes=0.0))
        g["launches"] += 1
        g["ms"] += t
        g["flop"] += flop
        g["bytes"] += byts

    for b in range(plan.n_bands):
        for l in range(plan.n_layers):
            name, slices = plan.layer_kernel(b, l)
            if not name:
                continue
            flop, byts = plan.layer_work(b, l)
            add(name, float(ms[b, l]), flop, byts)
            if slices > 1:
                add("splitk_finish_kernel<%s>" % ("__bf16" if dtype == "bf16" else "float"),
                    float(fin[b, l]), 0.0, 0.0)
    out = []
    for g in sorted(groups.values(), key=lambda g: -g["ms"]):
        t = g["ms"] * 1e-3
        out.append(dict(name=g["name"], launches=g["launches"], total_ms=round(g["ms"], 4),
                        avg_us=round(g["ms"] * 1e3 / g["launches"], 3),
                        tflops=round(g["flop"] / t / 1e12, 3) if t > 0 and g["flop"] else None,
                        gbs=round(g["bytes"] / t / 1e9, 1) if t > 0 and g["bytes"] else None,
                        flop_per_launch=g["flop"] / g["launches"],
                        bytes_per_launch=g["bytes"] / g["launches"]))
    return out


def roofline_of(k, dtype):
    """Bound of a kernel variant: matrix cores for the dense convolution unless its
    arithmetic intensity is below the ridge point; HBM for the row-wise kernels."""
    mf_peak = PEAK["mfma_bf16"] if dtype == "bf16" else PEAK["mfma_f32"]
    ai = k["flop_per_launch"] / max(k["bytes_per_launch"], 1.0)
    ridge = mf_peak * 1e12 / (PEAK["hbm"] * 1e9)
    if k["name"].startswith("conv_igemm") and ai >= ridge:  # a dense contraction above the ridge
        a = k["tflops"]
        return dict(bound="mfma", achieved=a, peak=mf_peak, unit="TFLOP/s",
                    frac=round(a / mf_peak, 4), traffic=None, kernel=k["name"],
                    avg_us=k["avg_us"], launches_per_step=k["launches"])
    a = k["gbs"]
    return dict(bound="hbm", achieved=a, peak=PEAK["hbm"], unit="GB/s",
                frac=round(a / PEAK["hbm"], 4), traffic=None, kernel=k["name"],
                avg_us=k["avg_us"], launches_per_step=k["launches"])


def source_hash():
    """Hash of the kernel sources: counters taken for other kernels must not be reported."""
    import hashlib
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2507_05829_amd", "csrc")
    for f in sorted(os.listdir(csrc)):
        if f.endswith((".hip", ".hpp", ".cpp")):
            h.update(open(os.path.join(csrc, f), "rb").read())
    return h.hexdigest()[:16]


def measured_traffic(workload, kernel_name):
    """HBM bytes per launch of a kernel from the committed counter summary, or None when
    there is none for this workload or the kernel sources changed since it was taken."""
    path = os.path.join(ROOT, "profiles", f"traffic_{workload}.json")
    if not os.path.exists(path):
        return None
    doc = json.load(open(path))
    if doc.get("source_hash") != source_hash():
        return None
    k = doc["kernels"].get(kernel_name)
    if not k or k["fetch_bytes_per_launch"] is None or k["write_bytes_per_launch"] is None:
        return None
    return round(k["fetch_bytes_per_launch"] + k["write_bytes_per_launch"])


def run_workload(torch, lop, workloads, name, steps, warmup, bands, profile_iters, lanes=0, graph=1, dma=0, replicas=1, mode="independent"):
    rowwise = name == "mlp"   # chain of row-wise operators (matrix products), Eq. 1
    chain = workloads.mlp_chain() if rowwise else workloads.CONFIGS[name]()
    if bands:
        chain.n_bands = bands
    tensors = workloads.make_row_tensors(chain) if rowwise else workloads.make_tensors(chain)
    flags = (lop.LOP_FLAG_LANES(lanes) | (lop.LOP_FLAG_GRAPH if graph else 0)
             | (lop.LOP_FLAG_DMA_COPY if dma else 0)
             | (lop.LOP_FLAG_REUSE if mode == "reuse" else 0))
    make_plan = lop.Plan.rowwise if rowwise else lop.Plan
    plans = [make_plan(chain, tensors, flags=flags) for _ in range(max(1, replicas))]
    plan = plans[0]
    d_in, d_out, h_out = device_tensors(torch, chain, tensors, plan, n_buf=max(2, len(plans), 8 if mode == "reuse" else 2))
    n_img = 1 if rowwise else chain.in_shape[0]   # a matrix counts as one image
    useful, executed, scratch = plan.stats()

    t_c = timed_steps(torch, plans, d_in, d_out, h_out, steps, warmup, copy=True)
    t_a = timed_steps(torch, plans, d_in, d_out, h_out, steps, min(warmup, 5), copy=False)
    t_b = timed_copies(torch, plan, d_out, h_out, steps, min(warmup, 5))
    hidden_steady = 1.0 - max(0.0, t_c - t_a) / t_b

    # single request: one chain at a time, host clock around launch .. last byte
    lat, lat_nc, cp, first, last = [], [], [], [], []
    for i in range(min(steps, 30)):
        tm = plan.run_chain(d_in, d_out[0], h_out[0], timing=True)
        lat.append(tm.wall_ms)
        cp.append(tm.copy_ms)
        ready = [tm.band_ready_ms[b] for b in range(plan.n_bands) if tm.band_ready_ms[b] > 0]
        first.append(min(ready)); last.append(max(ready))
        tm = plan.run_chain(d_in, d_out[0], None, timing=True)
        lat_nc.append(tm.wall_ms)
    lat.sort(); lat_nc.sort(); cp.sort(); first.sort(); last.sort()
    med = lambda v: v[len(v) // 2]
    # (bands whose rows leave through the last kernel's own stores have no copy to time)
    hidden_single = (1.0 if med(cp) < 1e-3 else
                     1.0 - max(0.0, med(lat) - med(lat_nc)) / med(cp))

    kernels = kernel_table(plan, d_in, d_out[0], profile_iters, chain.dtype)
    res = dict(
        workload=name, mode=mode, dtype=chain.dtype, n_bands=plan.n_bands, n_layers=plan.n_layers,
        images_per_s=n_img * steps / t_c, ms_per_step=t_c / steps * 1e3,
        ms_per_step_no_d2h=t_a / steps * 1e3, ms_copies_only=t_b / steps * 1e3,
        d2h_hidden_steady=round(hidden_steady, 4), d2h_hidden_single=round(hidden_single, 4),
        d2h_hidden_single_bound=round((plan.n_bands - 1) / plan.n_bands, 4),
        latency_ms_single=round(med(lat), 4), latency_ms_single_no_d2h=round(med(lat_nc), 4),
        # device-timeline view of one request: when the first and the last band are on the host
        first_band_ready_ms=round(med(first), 4), last_band_ready_ms=round(med(last), 4),
        latency_ms_single_p10=round(lat[len(lat) // 10], 4),
        latency_ms_single_p90=round(lat[min(len(lat) - 1, len(lat) * 9 // 10)], 4),
        useful_gflop=round(useful / 1e9, 4), executed_over_useful=round(executed / useful, 4),
        useful_tflops=round(useful * steps / t_c / 1e12, 3),
        executed_tflops=round(executed * steps / t_c / 1e12, 3),
        scratch_mb=round(scratch / 2 ** 20, 2),
        kernels=[{k: v for k, v in kk.items() if not k.endswith("_per_launch")} for kk in kernels],
    )
    if rowwise:
        res["rows_per_s"] = round(chain.m * steps / t_c, 1)
        res["matrix"] = f"{chain.m} x {chain.k} -> " + " -> ".join(str(L.n) for L in chain.layers)
    roof = roofline_of(next(k for k in kernels if k["flop_per_launch"] > 0), chain.dtype)
    roof["traffic"] = measured_traffic(f"{name}_{mode}", roof["kernel"])
    roof["algorithmic_bytes_per_launch"] = round(
        next(k for k in kernels if k["name"] == roof["kernel"])["bytes_per_launch"])
    for p in plans:
        p.destroy()
    return chain, tensors, res, roof


def cpu_baseline(chain, tensors, budget_s):
    """The oracle as it stands, on the host cores, unbanded whole images."""
    from oracle import reference
    reference.build()
    times = []
    t_all = time.perf_counter()
    run = reference.run_row_chain if hasattr(chain, "m") else reference.run_chain
    while True:
        t0 = time.perf_counter()
        run(chain, tensors)
        times.append(time.perf_counter() - t0)
        if len(times) >= 3 or time.perf_counter() - t_all > budget_s:
            break
    times.sort()
    t = times[len(times) // 2]
    out = dict(value=round(chain.in_shape[0] / t, 4), unit="images/s",
               cores=reference.num_threads(), kind="oracle",
               sample=f"{len(times)} whole unbanded {chain.name} image(s) "
                      f"{'x'.join(map(str, chain.in_shape))}, median {t:.3f} s each")
    if not hasattr(chain, "m") and time.perf_counter() - t_all < budget_s:
        # the oracle band by band, every band on its own slabs with its halos recomputed: the
        # partition costs the CPU the same executed / useful operations it costs the GPU
        from oracle import planner
        useful, executed = planner.flop_counts(chain)
        t0 = time.perf_counter()
        reference.run_chain_banded(chain, tensors)
        tb = time.perf_counter() - t0
        out["banded_independent"] = dict(value=round(chain.in_shape[0] / tb, 4), unit="images/s",
                                         slowdown=round(tb / t, 3),
                                         executed_over_useful_flop=round(executed / useful, 3))
    return out


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py measures one GPU only: the path has no multi-GPU part "
              "(bands would shard with no exchange); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    import workloads
    from paper_2507_05829_amd import lop
    if not torch.cuda.is_available():
        print("bench.py needs a GPU (there is no CPU fallback)", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)

    if a.pmc_calibrate:
        src = torch.zeros(64 << 20, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    chain, tensors, res, roof = run_workload(torch, lop, workloads, a.workload, a.steps, a.warmup,
                                             a.bands, a.profile_iters, a.lanes, a.graph, a.dma_copy, a.replicas, a.mode)
    if not a.no_reference_points:
        # the same chain as one band (no partition): what splitting into bands costs or gains
        _, _, whole, _ = run_workload(torch, lop, workloads, a.workload, max(a.steps // 4, 10), 5, 1,
                                      1, a.lanes, a.graph, a.dma_copy, a.replicas, a.mode)
        res["unbanded_images_per_s"] = round(whole["images_per_s"], 2)
        res["unbanded_latency_ms_single"] = whole["latency_ms_single"]
        # what the chip sustains on the roofline's two resources, beside the published peaks
        c = lop.lop_measure_ceilings()
        measured = {"hbm": c.hbm_copy_gbs, "mfma": c.mfma_bf16_tflops if chain.dtype == "bf16" else c.mfma_f32_tflops}
        roof["measured_peak"] = round(measured[roof["bound"]], 1)
        roof["frac_of_measured"] = round(roof["achieved"] / measured[roof["bound"]], 4)
        res["measured_ceilings"] = {"hbm_copy_GBps": round(c.hbm_copy_gbs, 1),
                                    "mfma_bf16_TFLOPps": round(c.mfma_bf16_tflops, 1),
                                    "mfma_f32_TFLOPps": round(c.mfma_f32_tflops, 1)}
    also = []
    for entry in [e for e in a.also.split(",") if e]:
        name, _, mode = entry.partition(":")
        mode = mode or a.mode
        if name == a.workload and mode == a.mode:
            continue
        heavy = name in ("mbv2", "mlp")
        _, _, r, rf = run_workload(torch, lop, workloads, name, 10 if heavy else max(a.steps // 4, 10),
                                   2 if heavy else 5, None, 3 if heavy else a.profile_iters,
                                   a.lanes, a.graph, a.dma_copy, a.replicas, mode)
        r["roofline"] = rf
        also.append(r)

    line = {
        "metric": "images/sec for banded conv chain (steady state, per-band D2H pipelined)",
        "value": round(res["images_per_s"], 3), "unit": "images/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": round(res["ms_per_step"], 5), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if chain.dtype == "f32" else "bf16", "data": "synthetic",
        "config": {"workload": f"{a.workload} {'x'.join(map(str, chain.in_shape))} "
                               f"{chain.dtype}, {res['n_bands']} row bands, {res['n_layers']} layers",
                   "images_per_step": chain.in_shape[0],
                   "mode": ("reuse: bands in order, rows produced by earlier bands are reused"
                            if a.mode == "reuse" else
                            "independent: every band recomputes its halos"),
                   "executed_over_useful_flop": res["executed_over_useful"],
                   "hip_graph": bool(a.graph), "lanes": a.lanes or "default",
                   "replicas": a.replicas},
        "roofline": roof,
        # the other two figures the metric names, for the whole chain: executed matrix FLOP per
        # second against the MFMA peak of the arithmetic type, and the share of the per-band
        # copy time that did not lengthen the step
        "mfma_utilisation": round(res["executed_tflops"] / (2500.0 if chain.dtype == "bf16" else 157.3), 4),
        "d2h_hidden": res["d2h_hidden_steady"],
        "detail": res,
        "also": also,
    }
    if not a.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(chain, tensors, a.cpu_seconds)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
