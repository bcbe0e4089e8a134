#!/usr/bin/env python3
"""Throughput of the banded local-operator chain on one MI355X.

One "step" is CHAINS_PER_STEP passes of the whole hot path back to back, each over one batch
of synthetic input: plan-driven kernels for every band and layer plus the per-band
device-to-host copies, pipelined (band b's copy under the kernels of other bands, the last
copy under the next chain). Inputs are resident in HBM before the timed region. The timed
region is exactly --steps steps between two full synchronisations; it is repeated (at least
five times and until half a second has been timed) and the median region is reported.

The headline is the 224 x 224 ResNet-18-style chain in four INDEPENDENT row bands (every band
recomputes its halo rows); the same chain in reuse mode, the 720p encoder in both modes, the
other chains, the one-band reference and single-request latency of each, the per-launch
roofline table and the CPU oracle's speed are fields of the same JSON line.
"""
import argparse
import hashlib
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK = {"mfma_f32": 157.3, "mfma_bf16": 2500.0, "hbm": 8000.0}   # TFLOP/s, TFLOP/s, GB/s
MIN_TIMED_S = 0.5
MIN_REPEATS = 5
DENSE = ("conv_", "pointwise_", "mbconv_")   # kernel families that run on the matrix cores


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--chains-per-step", type=int, default=64,
                    help="chains (images, or batches for a batched chain) back to back in one step")
    ap.add_argument("--workload", default="resnet18")
    ap.add_argument("--mode", default="independent", choices=["independent", "reuse", "batched"],
                    help="independent: every band recomputes its halos (the method as stated); "
                         "reuse: bands run in order and reuse rows earlier bands produced")
    ap.add_argument("--also", default="detector720p,vgg16,mbv2,mbv2:nofuse,tiny",
                    help="further workloads, each measured in both modes with fewer steps")
    ap.add_argument("--bands", type=int, default=None, help="override the workload's band count")
    ap.add_argument("--lanes", type=int, default=0, help="concurrent band streams (0 = library default)")
    ap.add_argument("--graph", type=int, default=1, help="1: replay the chain as a HIP graph")
    ap.add_argument("--dma-copy", type=int, default=0, help="1: band copies via hipMemcpyAsync")
    ap.add_argument("--pmc-calibrate", action="store_true",
                    help="also run a plain 256 MiB device-to-device copy (torch) a few times so "
                         "that a counter run can be scaled by a kernel of known traffic")
    ap.add_argument("--only-kernel-table", action="store_true",
                    help="run only the one-lane pass that times every launch (the command the "
                         "rocprofv3 kernel-trace summaries under profiles/ are taken with)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    ap.add_argument("--profile-iters", type=int, default=10)
    return ap.parse_args()


def source_hash():
    """Hash of the kernel sources: counters taken for other kernels must not be reported."""
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2507_05829_amd", "csrc")
    for f in sorted(os.listdir(csrc)):
        if f.endswith((".hip", ".hpp", ".cpp")):
            h.update(open(os.path.join(csrc, f), "rb").read())
    return h.hexdigest()[:16]


def measured_traffic(tag, kernel_name):
    """HBM bytes per launch of a kernel from the committed counter summary, or None when
    there is none for this workload or the kernel sources changed since it was taken."""
    path = os.path.join(ROOT, "profiles", f"traffic_{tag}.json")
    if not os.path.exists(path):
        return None
    doc = json.load(open(path))
    if doc.get("source_hash") != source_hash():
        return None
    k = doc["kernels"].get(kernel_name)
    if not k or k["fetch_bytes_per_launch"] is None or k["write_bytes_per_launch"] is None:
        return None
    return round(k["fetch_bytes_per_launch"] + k["write_bytes_per_launch"])


class Case:
    """One workload in one mode: chain, tensors, plan and device buffers."""

    def __init__(self, torch, lop, workloads, name, mode, a, bands=None, nofuse=False, n_buf=8):
        import numpy as np
        self.torch, self.lop, self.name, self.mode, self.nofuse = torch, lop, name, mode, nofuse
        rowwise = name == "mlp"   # a chain of row-wise operators (matrix products, Eq. 1)
        self.chain = workloads.mlp_chain() if rowwise else workloads.CONFIGS[name]()
        if bands:
            self.chain.n_bands = bands
        self.tensors = workloads.make_row_tensors(self.chain) if rowwise else workloads.make_tensors(self.chain)
        flags = (lop.LOP_FLAG_LANES(a.lanes) | (lop.LOP_FLAG_GRAPH if a.graph else 0)
                 | (lop.LOP_FLAG_DMA_COPY if a.dma_copy else 0)
                 | (lop.LOP_FLAG_REUSE if mode == "reuse" else 0)
                 | (lop.LOP_FLAG_BATCH_BANDS if mode == "batched" else 0)
                 | (lop.LOP_FLAG_NO_FUSE if nofuse else 0))
        self.plan = (lop.Plan.rowwise if rowwise else lop.Plan)(self.chain, self.tensors, flags=flags)
        x = torch.from_numpy(self.tensors.x if rowwise else
                             np.ascontiguousarray(self.tensors.x.transpose(0, 2, 3, 1)))
        td = torch.bfloat16 if self.chain.dtype == "bf16" else torch.float32
        self.d_in = x.to(td).cuda()
        n, c, h, w = self.plan.out_shape()
        self.out_bytes = n * c * h * w * (2 if self.chain.dtype == "bf16" else 4)
        if self.out_bytes > (8 << 20):
            n_buf = 2
        self.d_out = [torch.zeros((n, h, w, c), dtype=td, device="cuda") for _ in range(n_buf)]
        self.h_out = [torch.zeros((n, h, w, c), dtype=td, pin_memory=True) for _ in range(n_buf)]
        self.images = 1 if rowwise else self.chain.in_shape[0]   # a matrix counts as one image
        torch.cuda.synchronize()

    def tag(self):
        return self.name + (":nofuse" if self.nofuse else "")

    def run(self, i, copy=True):
        k = i % len(self.d_out)
        self.plan.run_chain(self.d_in, self.d_out[k], self.h_out[k] if copy else None)

    def region(self, chains, copy=True):
        """Seconds for `chains` chains back to back between two full synchronisations."""
        self.plan.synchronize()
        self.torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(chains):
            self.run(i, copy)
        self.plan.synchronize()
        self.torch.cuda.synchronize()
        return time.perf_counter() - t0

    def close(self):
        self.plan.destroy()


def repeated_regions(case, chains, warm_chains, copy=True, min_s=MIN_TIMED_S, min_rep=MIN_REPEATS,
                     max_rep=40):
    for i in range(warm_chains):
        case.run(i, copy)
    times, total = [], 0.0
    while len(times) < min_rep or (total < min_s and len(times) < max_rep):
        t = case.region(chains, copy)
        times.append(t)
        total += t
    return times


def d2h_bandwidth(torch, nbytes=64 << 20):
    """GB/s of one large device-to-host copy into pinned memory (the link's rate, measured)."""
    src = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    dst = torch.empty(nbytes, dtype=torch.uint8, pin_memory=True)
    best = 0.0
    for _ in range(4):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        dst.copy_(src, non_blocking=True)
        torch.cuda.synchronize()
        best = max(best, nbytes / (time.perf_counter() - t0) / 1e9)
    return best


def weight_bytes(chain, l):
    """Bytes of layer l's weights as the work model counts them."""
    L = chain.layers[l]
    if getattr(L, "op", None) not in ("conv", "dwconv"):
        return 0.0
    esz = 2 if chain.dtype == "bf16" else 4
    groups = L.c_in if L.op == "dwconv" else 1
    return float(esz * L.c_out * (L.c_in // groups) * L.k[0] * L.k[1])


def launch_rows(case, iters):
    """Every (layer, band) launch of one chain, timed on one stream, one lane, with a start and
    a stop HIP event attached to the dispatch itself (the kernel's own duration, as a
    profiler's kernel trace reports it), with its algorithmic work and the roofline that
    bounds it: a dense convolution is priced against the matrix cores when its arithmetic
    intensity is at or above the ridge of its type, everything else against HBM."""
    plan, dtype = case.plan, case.chain.dtype
    ms, fin = plan.profile_chain(case.d_in, case.d_out[0], iters)
    mf_peak = PEAK["mfma_bf16"] if dtype == "bf16" else PEAK["mfma_f32"]
    ridge = mf_peak * 1e12 / (PEAK["hbm"] * 1e9)
    rows = []
    for l in range(plan.n_layers):
        op = getattr(case.chain.layers[l], "op", "rowwise")
        for b in range(plan.n_bands):
            name, slices = plan.layer_kernel(b, l)
            if not name:
                continue
            flop, byts = plan.layer_work(b, l)
            if case.mode == "batched":      # one launch for all bands: their work, the weights once
                parts = [plan.layer_work(bb, l) for bb in range(plan.n_bands)]
                active = sum(1 for f, _ in parts if f > 0)
                flop = sum(f for f, _ in parts)
                byts = sum(y for _, y in parts) - max(active - 1, 0) * weight_bytes(case.chain, l)
            us = float(ms[b, l]) * 1e3
            fus = float(fin[b, l]) * 1e3 if slices > 1 else 0.0
            ai = flop / max(byts, 1.0)
            bound = "mfma" if name.startswith(DENSE) and ai >= ridge else "hbm"
            t = (us + fus) * 1e-6
            ach = flop / t / 1e12 if bound == "mfma" else byts / t / 1e9
            rows.append(dict(layer=l, band=b, op=op, kernel=name, k_slices=slices, us=round(us, 2),
                             finish_us=round(fus, 2), gflop=round(flop / 1e9, 4), mbytes=round(byts / 1e6, 4),
                             ai=round(ai, 1), bound=bound, achieved=round(ach, 2),
                             unit="TFLOP/s" if bound == "mfma" else "GB/s",
                             frac=round(ach / (mf_peak if bound == "mfma" else PEAK["hbm"]), 4),
                             _flop=flop, _bytes=byts))
    return rows, ridge, mf_peak


def kernel_groups(rows, dtype):
    """The launches grouped by kernel instance (named as rocprofv3 prints it). The finish kernel
    of a convolution whose reduction is cut across workgroups is listed on its own; the layer's
    algorithmic work is booked on the convolution kernel."""
    groups = {}

    def add(name, us, flop, byts):
        g = groups.setdefault(name, dict(name=name, launches=0, us=0.0, flop=0.0, bytes=0.0))
        g["launches"] += 1
        g["us"] += us
        g["flop"] += flop
        g["bytes"] += byts

    for r in rows:
        add(r["kernel"], r["us"], r["_flop"], r["_bytes"])
        if r["k_slices"] > 1:
            add("splitk_finish_kernel<%s>" % ("__bf16" if dtype == "bf16" else "float"), r["finish_us"], 0.0, 0.0)
    out = []
    for g in sorted(groups.values(), key=lambda g: -g["us"]):
        t = g["us"] * 1e-6
        out.append(dict(name=g["name"], launches=g["launches"], total_us=round(g["us"], 2),
                        avg_us=round(g["us"] / g["launches"], 3),
                        tflops=round(g["flop"] / t / 1e12, 3) if t > 0 and g["flop"] else None,
                        gbs=round(g["bytes"] / t / 1e9, 1) if t > 0 and g["bytes"] else None,
                        _flop=g["flop"], _bytes=g["bytes"]))
    return out


def dominant_roofline(groups, ridge, mf_peak, tag):
    """Roofline object of the kernel instance with the largest total time that does
    algorithmic work, priced by the aggregate arithmetic intensity of its launches."""
    k = next(g for g in groups if g["_flop"] > 0 or g["_bytes"] > 0)
    ai = k["_flop"] / max(k["_bytes"], 1.0)
    if k["name"].startswith(DENSE) and ai >= ridge:
        roof = dict(bound="mfma", achieved=k["tflops"], peak=mf_peak, unit="TFLOP/s",
                    frac=round(k["tflops"] / mf_peak, 4))
    else:
        roof = dict(bound="hbm", achieved=k["gbs"], peak=PEAK["hbm"], unit="GB/s",
                    frac=round(k["gbs"] / PEAK["hbm"], 4))
    roof.update(traffic=measured_traffic(tag, k["name"]), kernel=k["name"], avg_us=k["avg_us"],
                launches_per_chain=k["launches"], ai_flop_per_byte=round(ai, 1), ridge=round(ridge, 1),
                algorithmic_bytes_per_launch=round(k["_bytes"] / k["launches"]),
                algorithmic_flop_per_launch=round(k["_flop"] / k["launches"]))
    return roof


def strip(rows):
    return [{k: v for k, v in r.items() if not k.startswith("_")} for r in rows]


def single_request(case, n=30):
    """One chain at a time, host clock around launch .. last byte on the host."""
    plan = case.plan
    lat, lat_nc, first, last = [], [], [], []
    for _ in range(n):
        tm = plan.run_chain(case.d_in, case.d_out[0], case.h_out[0], timing=True)
        lat.append(tm.wall_ms)
        ready = [tm.band_ready_ms[b] for b in range(plan.n_bands) if tm.band_ready_ms[b] > 0]
        first.append(min(ready))
        last.append(max(ready))
        tm = plan.run_chain(case.d_in, case.d_out[0], None, timing=True)
        lat_nc.append(tm.wall_ms)
    q = lambda v, f: sorted(v)[min(len(v) - 1, int(len(v) * f))]
    return dict(latency_ms=round(statistics.median(lat), 4), latency_ms_p10=round(q(lat, 0.1), 4),
                latency_ms_p90=round(q(lat, 0.9), 4), latency_ms_no_d2h=round(statistics.median(lat_nc), 4),
                first_band_on_host_ms=round(statistics.median(first), 4),
                last_band_on_host_ms=round(statistics.median(last), 4))


def measure(torch, lop, workloads, name, mode, a, steps, warmup, link_gbs, nofuse=False, tables=True,
            min_s=MIN_TIMED_S):
    case = Case(torch, lop, workloads, name, mode, a, a.bands if name == a.workload else None, nofuse)
    chain, plan = case.chain, case.plan
    # a batched chain is already many images per pass: keep a step near the same image count
    cps = max(1, a.chains_per_step // case.images)
    chains = steps * cps
    t_c = repeated_regions(case, chains, warmup * cps, copy=True, min_s=min_s)
    t_a = repeated_regions(case, chains, min(warmup, 2) * cps, copy=False, min_s=min_s / 2)
    med_c, med_a = statistics.median(t_c), statistics.median(t_a)
    useful, executed, scratch = plan.stats()
    # exposed copy time per chain: pipelined minus compute-only, with the spread of the repeats
    exposed_us = (med_c - med_a) / chains * 1e6
    noise_us = (statistics.pstdev(t_c) + statistics.pstdev(t_a)) / chains * 1e6
    copy_us_link = case.out_bytes / (link_gbs * 1e9) * 1e6
    # the same bytes as band copies alone, back to back on one stream
    for i in range(3):
        plan.copy_chain(case.d_out[i % len(case.d_out)], case.h_out[i % len(case.d_out)])
    plan.synchronize()
    t0 = time.perf_counter()
    n_copy = max(10, min(chains, 200))
    for i in range(n_copy):
        plan.copy_chain(case.d_out[i % len(case.d_out)], case.h_out[i % len(case.d_out)])
    plan.synchronize()
    copy_us_serial = (time.perf_counter() - t0) / n_copy * 1e6
    hidden = lambda denom: round(1.0 - max(0.0, exposed_us) / denom, 4) if denom > 0 else None
    res = dict(
        workload=case.tag(), mode=mode, dtype=chain.dtype, n_bands=plan.n_bands, n_layers=plan.n_layers,
        images_per_chain=case.images, chains_per_step=cps, steps=steps, repeats=len(t_c),
        images_per_s=round(case.images * chains / med_c, 2),
        images_per_s_min_max=[round(case.images * chains / max(t_c), 2), round(case.images * chains / min(t_c), 2)],
        ms_per_step=round(med_c / steps * 1e3, 5), ms_per_chain=round(med_c / chains * 1e3, 5),
        ms_per_chain_no_d2h=round(med_a / chains * 1e3, 5),
        d2h=dict(bytes_per_chain=case.out_bytes, exposed_us_per_chain=round(exposed_us, 3),
                 repeat_noise_us=round(noise_us, 3), within_noise=bool(abs(exposed_us) <= 2 * noise_us),
                 copy_us_at_link_rate=round(copy_us_link, 3), link_GBps=round(link_gbs, 1),
                 copy_us_serial_band_copies=round(copy_us_serial, 3),
                 hidden_vs_link_rate=hidden(copy_us_link), hidden_vs_serial_band_copies=hidden(copy_us_serial)),
        useful_gflop=round(useful / 1e9, 4), executed_over_useful=round(executed / useful, 4),
        useful_tflops=round(useful * chains / med_c / 1e12, 3),
        executed_tflops=round(executed * chains / med_c / 1e12, 3),
        scratch_mb=round(scratch / 2 ** 20, 2),
    )
    res["single_request"] = single_request(case)
    s = res["single_request"]
    extra_us = (s["latency_ms"] - s["latency_ms_no_d2h"]) * 1e3
    res["d2h"]["single_request_extra_us"] = round(extra_us, 2)
    res["d2h"]["hidden_single_vs_link_rate"] = round(1.0 - max(0.0, extra_us) / copy_us_link, 4)
    res["d2h"]["hidden_single_bound"] = round((plan.n_bands - 1) / plan.n_bands, 4)
    rows, ridge, mf_peak = launch_rows(case, a.profile_iters)
    groups = kernel_groups(rows, chain.dtype)
    res["kernels"] = strip(groups)
    res["roofline"] = dominant_roofline(groups, ridge, mf_peak, f"{case.tag().replace(':', '_')}_{mode}")
    # dense-convolution utilisation of the matrix cores over the chain: algorithmic FLOP of the
    # dense convolutions (executed, halo recompute included) over their kernel time
    dense = [r for r in rows if r["kernel"].startswith(DENSE)]
    t_dense = sum(r["us"] + r["finish_us"] for r in dense) * 1e-6
    if t_dense > 0:
        tf = sum(r["_flop"] for r in dense) / t_dense / 1e12
        res["dense_conv"] = dict(kernel_time_us=round(t_dense * 1e6, 1), executed_tflops=round(tf, 2),
                                 mfma_peak_tflops=mf_peak, frac_of_mfma_peak=round(tf / mf_peak, 4))
    hbm = [r for r in rows if not r["kernel"].startswith(DENSE)]
    t_hbm = sum(r["us"] for r in hbm) * 1e-6
    if t_hbm > 0:
        gbs = sum(r["_bytes"] for r in hbm) / t_hbm / 1e9
        res["depthwise_pool_eltwise"] = dict(kernel_time_us=round(t_hbm * 1e6, 1), gbs=round(gbs, 1),
                                             frac_of_hbm_peak=round(gbs / PEAK["hbm"], 4))
    if tables:
        res["launches"] = strip(rows)
    case.close()
    return case, res


def one_band_reference(torch, lop, workloads, name, mode, a, nofuse=False, tables=True):
    """The same chain as ONE band (no partition): throughput, single-request latency and the
    per-layer table at B = 1."""
    # (scheduled like reuse mode, so that consecutive chains rotate over the lanes: with one band
    # the modes compute the same, and independent mode would keep a single band on a single lane)
    case = Case(torch, lop, workloads, name, "reuse", a, 1, nofuse)
    cps = max(1, a.chains_per_step // case.images)
    chains = max(2, a.steps // 2) * cps
    t = repeated_regions(case, chains, 2 * cps, copy=True, min_s=0.2)
    med = statistics.median(t)
    out = dict(images_per_s=round(case.images * chains / med, 2), ms_per_chain=round(med / chains * 1e3, 5),
               single_request=single_request(case, 15))
    if tables:
        rows, _, _ = launch_rows(case, a.profile_iters)
        out["launches"] = strip(rows)
    case.close()
    return out


def cpu_baseline(chain, tensors, budget_s):
    """The oracle as it stands, on the host cores, unbanded whole images."""
    from oracle import reference
    reference.build()
    times = []
    t_all = time.perf_counter()
    while True:
        t0 = time.perf_counter()
        reference.run_chain(chain, tensors)
        times.append(time.perf_counter() - t0)
        if len(times) >= 3 or time.perf_counter() - t_all > budget_s:
            break
    t = statistics.median(times)
    out = dict(value=round(chain.in_shape[0] / t, 4), unit="images/s",
               cores=reference.num_threads(), kind="oracle",
               sample=f"{len(times)} whole unbanded {chain.name} image(s) "
                      f"{'x'.join(map(str, chain.in_shape))}, median {t:.3f} s each")
    if time.perf_counter() - t_all < budget_s:
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

    if a.only_kernel_table:
        name, _, nf = a.workload.partition(":")
        case = Case(torch, lop, workloads, name, a.mode, a, a.bands, nf == "nofuse")
        case.plan.profile_chain(case.d_in, case.d_out[0], 3)
        rows, _, _ = launch_rows(case, a.profile_iters)
        print(json.dumps(dict(workload=case.tag(), mode=a.mode, n_bands=case.plan.n_bands,
                              kernels=strip(kernel_groups(rows, case.chain.dtype)), launches=strip(rows))))
        case.close()
        return

    link = d2h_bandwidth(torch)
    others = [m for m in ("independent", "batched", "reuse") if m != a.mode]
    head_case, head = measure(torch, lop, workloads, a.workload, a.mode, a, a.steps, a.warmup, link)
    seconds = {}
    for m in others:
        try:
            _, seconds[m] = measure(torch, lop, workloads, a.workload, m, a, a.steps, a.warmup, link)
        except lop.LopError as e:     # (launches batched over the bands: not every kernel has that form)
            if e.code != lop.LOP_ERR_UNSUPPORTED:
                raise
    head["one_band"] = one_band_reference(torch, lop, workloads, a.workload, a.mode, a)
    c = lop.lop_measure_ceilings()
    ceil = {"hbm_copy_GBps": round(c.hbm_copy_gbs, 1), "mfma_bf16_TFLOPps": round(c.mfma_bf16_tflops, 1),
            "mfma_f32_TFLOPps": round(c.mfma_f32_tflops, 1), "launch_floor_us": round(c.launch_floor_us, 2),
            "graph_node_floor_us": round(c.graph_node_floor_us, 2)}

    def against_measured(roof, dtype):
        m = c.hbm_copy_gbs if roof["bound"] == "hbm" else (c.mfma_bf16_tflops if dtype == "bf16" else c.mfma_f32_tflops)
        roof["measured_peak"] = round(m, 1)
        roof["frac_of_measured"] = round(roof["achieved"] / m, 4)
        # what a launch of this size could reach at most: its work at the published peak behind
        # the measured cost of a launch that does nothing
        work = roof["algorithmic_bytes_per_launch"] / 1e3 if roof["bound"] == "hbm" else roof["algorithmic_flop_per_launch"] / 1e6
        t_peak_us = work / roof["peak"]            # kB / (GB/s) and MFLOP / (TFLOP/s) are both microseconds
        roof["launch_floor_us"] = round(c.launch_floor_us, 2)
        roof["frac_ceiling_at_this_launch_size"] = round(t_peak_us / (t_peak_us + c.launch_floor_us), 4)

    against_measured(head["roofline"], head["dtype"])
    for r in seconds.values():
        against_measured(r["roofline"], r["dtype"])

    also = {}
    light_steps = max(2, a.steps // 4)
    for entry in [e for e in a.also.split(",") if e]:
        name, _, nf = entry.partition(":")
        nofuse = nf == "nofuse"
        if name == a.workload and not nofuse:
            continue
        per_mode = {}
        for mode in [a.mode] + others:
            if nofuse and mode != a.mode:
                continue      # the layer-by-layer run is there for its kernels' own rates
            tables = name in ("vgg16", "detector720p") or nofuse
            try:
                _, r = measure(torch, lop, workloads, name, mode, a, light_steps, 1, link, nofuse,
                               tables=tables, min_s=0.25)
            except lop.LopError as e:
                if e.code != lop.LOP_ERR_UNSUPPORTED:
                    raise
                continue
            against_measured(r["roofline"], r["dtype"])
            if mode == a.mode and not nofuse:
                r["one_band"] = one_band_reference(torch, lop, workloads, name, mode, a, nofuse,
                                                   tables=name in ("vgg16", "detector720p"))
            per_mode[mode] = r
        also[entry] = per_mode

    chain = head_case.chain
    dense = head.get("dense_conv", {})
    line = {
        "metric": "images/sec for banded conv chain (independent row bands, steady state, per-band D2H pipelined)",
        "value": head["images_per_s"], "unit": "images/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if chain.dtype == "f32" else "bf16", "data": "synthetic",
        "config": {"workload": f"{a.workload} {'x'.join(map(str, chain.in_shape))} {chain.dtype}, "
                               f"{head['n_bands']} row bands, {head['n_layers']} layers",
                   "mode": {"independent": "independent: every band recomputes its halos, one launch per band and layer",
                            "batched": "independent bands (every band recomputes its halos), one launch per layer for "
                                       "all bands (operation batching, Sec. IV-D)",
                            "reuse": "reuse: bands in order, rows produced by earlier bands are reused"}[a.mode],
                   "chains_per_step": head["chains_per_step"], "images_per_chain": head["images_per_chain"],
                   "timed_region": f"{a.steps} steps, median of {head['repeats']} repeats",
                   "executed_over_useful_flop": head["executed_over_useful"],
                   "hip_graph": bool(a.graph), "lanes": a.lanes or "default"},
        "roofline": head["roofline"],
        # the other two figures the metric names: algorithmic FLOP of the dense convolutions over
        # their kernel time against the matrix-core peak of the type, and the share of the
        # output's link time (bytes / measured D2H rate) that did not lengthen the chain
        "mfma_utilisation": dense.get("frac_of_mfma_peak"),
        # (null when the exposed time is within the spread of the repeats: a 49 KiB output per
        # image is 1-2 us at the link's rate, which a difference of two timed runs cannot resolve)
        "d2h_hidden": None if head["d2h"]["within_noise"] else head["d2h"]["hidden_vs_link_rate"],
        "d2h_exposed_us_per_chain": head["d2h"]["exposed_us_per_chain"],
        # the same independent bands with every layer launched once for all bands (operation
        # batching, Sec. IV-D), and reuse mode: detail under "modes"
        "images_per_s_by_mode": {m: r["images_per_s"] for m, r in {a.mode: head, **seconds}.items()},
        "measured_ceilings": ceil,
        "modes": {a.mode: head, **seconds},
        "also": also,
    }
    if not a.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(chain, head_case.tensors, a.cpu_seconds)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
