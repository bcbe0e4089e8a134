"""Replays the library's host code paths against the stand-in HIP runtime under the sanitizers
(see build_stub.py). Run as `python replay.py <stub dir>` with the AddressSanitizer runtime
preloaded; exits non-zero on any sanitizer report, stub misuse report or leaked HIP object.

What runs: the create / run / destroy sequences of the GPU parity suite (the same seeded
random chains, all four (mode, type) sets, and the named workloads at reduced size), with
"device" buffers that are plain host arrays and kernels that do nothing, so only the host code
is exercised: planning, weight packing and upload, lanes, events, graph capture and replay,
the copy paths (mapped pinned, pageable, DMA flag), timing, the measurement aids, the
two-party runtime, the entry point that allocates nothing, and the teardown.
"""
import ctypes
import os
import sys
import types

stub_dir = sys.argv[1]
HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
sys.path[:0] = [stub_dir, ROOT, os.path.dirname(HERE)]
sys.modules["torch"] = types.ModuleType("torch")   # the binding imports it only for its runtime

import numpy as np  # noqa: E402

import workloads  # noqa: E402
from paper_2507_05829_amd import lop  # noqa: E402
from random_chains import random_conv_chain  # noqa: E402

assert lop.LIB_PATH.startswith(stub_dir), lop.LIB_PATH
stub = ctypes.CDLL(os.path.join(stub_dir, "paper_2507_05829_amd", "libhipstub.so"))
stub.hipstub_live.restype = ctypes.c_long
stub.hipstub_launches.restype = ctypes.c_long
stub.hipstub_pin.argtypes = [ctypes.c_void_p, ctypes.c_size_t]
stub.hipstub_unpin.argtypes = [ctypes.c_void_p]
KINDS = ["stream", "event", "graph", "graph exec", "allocation"]


def buffers(chain, plan, pinned=True):
    n, c, h, w = chain.in_shape
    esz = 2 if chain.dtype == "bf16" else 4
    d_in = np.zeros(n * c * h * w * esz, np.uint8)
    on, oc, oh, ow = plan.out_shape()
    d_out = np.zeros(on * oc * oh * ow * esz, np.uint8)
    h_out = np.zeros(on * oc * oh * ow * esz, np.uint8)
    if pinned:
        stub.hipstub_pin(h_out.ctypes.data, h_out.nbytes)
    return d_in, d_out, h_out


def release(h_out):
    stub.hipstub_unpin(h_out.ctypes.data)


def run_like_the_parity_suite(chain, t, flags):
    plan = lop.Plan(chain, t, None, flags)
    try:
        d_in, d_out, h_out = buffers(chain, plan)
        plan.run_chain(d_in, d_out, h_out)
        plan.synchronize()
        release(h_out)
    finally:
        plan.destroy()


def random_chain_sets():
    n = 0
    for dtype, reuse, base in (("f32", 0, 1234), ("f32", 0, 9001), ("f32", 1, 1234), ("bf16", 0, 1234),
                               ("bf16", 1, 1234)):
        if True:
            rng = np.random.Generator(np.random.PCG64(base + 17 * reuse + (dtype == "bf16")))
            done = 0
            while done < 24:
                chain = random_conv_chain(rng, dtype)
                if chain is None:
                    continue
                t = workloads.make_tensors(chain, zero_bias=False, seed=int(rng.integers(1, 1 << 30)))
                run_like_the_parity_suite(chain, t, lop.LOP_FLAG_REUSE if reuse else 0)
                done += 1
                n += 1
    return n


def named_workloads():
    n = 0
    scaled = [workloads.tiny_chain(), workloads.resnet18_chain(h=64, w=48), workloads.vgg16_chain(h=64, w=64),
              workloads.detector_chain(h=96, w=64), workloads.mbv2_chain(h=32, w=32, n=2, n_bands=4),
              workloads.mbv2_chain(h=192, w=192, n=8, n_bands=2),   # long band copies: the copy lane
              workloads.detector_chain()]   # full size: the kernels that only large launches take
    for chain in scaled:
        t = workloads.make_tensors(chain, zero_bias=False)
        for flags in (0, lop.LOP_FLAG_REUSE, lop.LOP_FLAG_GRAPH, lop.LOP_FLAG_GRAPH | lop.LOP_FLAG_REUSE,
                      lop.LOP_FLAG_DMA_COPY, lop.LOP_FLAG_NO_D2H, lop.LOP_FLAG_NO_FUSE, lop.LOP_FLAG_LANES(1),
                      lop.LOP_FLAG_LANES(1) | lop.LOP_FLAG_GRAPH, lop.LOP_FLAG_LANES(7) | lop.LOP_FLAG_REUSE,
                      lop.LOP_FLAG_BATCH_BANDS, lop.LOP_FLAG_BATCH_BANDS | lop.LOP_FLAG_GRAPH):
            try:
                plan = lop.Plan(chain, t, None, flags)
            except lop.LopError as e:      # chains with an operator whose kernel takes one band at a time
                assert e.code == lop.LOP_ERR_UNSUPPORTED and flags & lop.LOP_FLAG_BATCH_BANDS
                continue
            d_in, d_out, h_out = buffers(chain, plan)
            pageable = np.zeros_like(h_out)
            for rep in range(3):                      # graph: capture once, replay twice
                plan.run_chain(d_in, d_out, h_out)
                plan.synchronize()
            try:                                      # host memory that is not pinned is refused
                plan.run_chain(d_in, d_out, pageable)
                raise SystemExit("a pageable host buffer was accepted")
            except lop.LopError as e:
                assert e.code == lop.LOP_ERR_INVALID_ARG or flags & lop.LOP_FLAG_NO_D2H
            except SystemExit:
                if not flags & lop.LOP_FLAG_NO_D2H:
                    raise
            plan.run_chain(d_in, d_out, None)
            tm = plan.run_chain(d_in, d_out, h_out, timing=True)
            assert tm.n_bands == plan.n_bands
            order = range(plan.n_bands) if flags & lop.LOP_FLAG_REUSE else reversed(range(plan.n_bands))
            for b in order:
                plan.run_band(b, d_in, d_out, h_out)
            plan.synchronize()
            plan.profile_chain(d_in, d_out, 2)
            plan.copy_chain(d_out, h_out)
            plan.time_layer(0, plan.n_layers - 1, d_in, d_out, 2)
            for b in range(plan.n_bands):
                for l in range(plan.n_layers):
                    plan.layer_kernel(b, l)
                    plan.layer_work(b, l)
            plan.stats()
            if hasattr(lop, "lop_run_chain_static") and not flags & (lop.LOP_FLAG_REUSE | lop.LOP_FLAG_BATCH_BANDS):
                try:
                    lop.lop_run_chain_static(plan.handle, d_in, d_out, None)
                except lop.LopError as e:   # layer by layer the large chain needs more than the array holds
                    assert e.code == lop.LOP_ERR_TOO_LARGE and flags & lop.LOP_FLAG_NO_FUSE
                plan.synchronize()
            if not flags:
                heights = [plan.layer_shape(l)[2] for l in range(plan.n_layers)]
                sched = workloads.random_schedule(heights, seed=5)
                plan.run_two_party(d_in, d_out, [(a["M"], a["R"]) for a in sched], 1e12, 0.0)
            release(h_out)
            plan.destroy()
            n += 1
    # row-wise chain (Eq. 1)
    rc = workloads.mlp_chain(m=300, k=64, hidden=128)
    rt = workloads.make_row_tensors(rc)
    plan = lop.Plan.rowwise(rc, rt)
    esz = 2 if rc.dtype == "bf16" else 4
    d_in = np.zeros(rc.m * rc.k * esz, np.uint8)
    on, oc, oh, ow = plan.out_shape()
    d_out = np.zeros(on * oc * oh * ow * esz, np.uint8)
    plan.run_chain(d_in, d_out, None)
    plan.synchronize()
    plan.destroy()
    return n + 1


def scheduling_model_and_two_party():
    """The scheduling-model calls and the two-party runtime as the GPU tests drive them: a
    searched schedule for the full-size backbone with modelled device speeds, and seeded random
    chains under random schedules."""
    from oracle import loss, planner
    n = 0
    chain = workloads.resnet18_chain()
    t = workloads.make_tensors(chain, zero_bias=False)
    shapes = planner.infer_shapes(chain)
    layers = []
    for i, L in enumerate(chain.layers):
        nn, c, h, w = shapes[i]
        flop_row = planner.conv_flop(chain, shapes, i, 1) if L.op != "maxpool" else 40.0 * nn * c * w
        layers.append(loss.LossLayer(n_ops=h, input_from=L.input_from, residual_from=L.residual_from,
                                     k=L.k[0], s=L.s[0], p=L.p[0], d=L.d[0],
                                     cm_fixed=5e-5, cm_row=flop_row / 5e10, cr_fixed=1e-5, cr_row=flop_row / 2e12,
                                     row_bytes=float(nn * c * w * 4)))
    nn, c, h, w = chain.in_shape
    for bw in (4e6, 40e6):
        for model in (lop.LOP_LINK_QUEUED, lop.LOP_LINK_INDEPENDENT):
            sched, T, viol = lop.lop_loss_solve(layers, h, float(nn * c * w * 4), bw, 1e-3, generations=60,
                                                seed=3, link_model=model)
            lop.lop_loss_eval(layers, h, float(nn * c * w * 4), bw, 1e-3, sched, model)
        plan = lop.Plan(chain, t, 1)
        d_in, d_out, h_out = buffers(chain, plan)
        plan.run_two_party(d_in, d_out, sched, bw, 1e-3, layers)
        release(h_out)
        plan.destroy()
        n += 1
    def two_party_case(chain, t, sched, bw=1e12, lat=0.0, costs=None):
        plan = lop.Plan(chain, t, 1)
        d_in, d_out, h_out = buffers(chain, plan)
        plan.run_two_party(d_in, d_out, [(a["M"], a["R"]) for a in sched], bw, lat, costs)
        release(h_out)
        plan.destroy()

    heights_of = lambda ch: [sh[2] for sh in planner.infer_shapes(ch)]
    # the schedules of the other two-party GPU tests, case by case
    for mk, kw in ((workloads.tiny_chain, {}), (workloads.resnet18_chain, dict(h=64, w=48)),
                   (workloads.mbv2_chain, dict(h=48, w=40, n=2)), (workloads.detector_chain, dict(h=90, w=64)),
                   (workloads.vgg16_chain, dict(h=64, w=32))):
        chain = mk(**kw)
        t = workloads.make_tensors(chain, zero_bias=False)
        for seed in range(3):
            two_party_case(chain, t, workloads.random_schedule(heights_of(chain), seed=200 + seed, overlap=3))
            n += 1
    chain = workloads.resnet18_chain(h=40, w=24)
    chain.layers = chain.layers[:4]
    t = workloads.small_int_tensors(chain, seed=4)
    for seed in (1, 2):
        two_party_case(chain, t, workloads.random_schedule(heights_of(chain), seed=seed, overlap=2))
        n += 1
    from oracle import two_party as tp_oracle
    chain = workloads.resnet18_chain(h=64, w=48)
    t = workloads.make_tensors(chain, zero_bias=False)
    for party in ("M", "R"):
        two_party_case(chain, t, tp_oracle.all_on(chain, party))
        n += 1
    shapes = planner.infer_shapes(chain)
    costs = []
    for i, L in enumerate(chain.layers):
        nn, c, h, w = shapes[i]
        costs.append(loss.LossLayer(n_ops=h, input_from=L.input_from, residual_from=L.residual_from,
                                    k=L.k[0], s=L.s[0], p=L.p[0], d=L.d[0], cm_fixed=5e-4, cm_row=5e-5,
                                    cr_fixed=2e-4, cr_row=1e-5, row_bytes=float(nn * c * w * 4)))
    nn, c, h, w = chain.in_shape
    for seed in (1, 2, 3):
        sched = workloads.random_schedule(heights_of(chain), seed=300 + seed, overlap=2)
        lop.lop_loss_eval(costs, h, float(nn * c * w * 4), 20e6, 5e-4, [(a["M"], a["R"]) for a in sched],
                          lop.LOP_LINK_QUEUED)
        two_party_case(chain, t, sched, 20e6, 5e-4, costs)
        n += 1
    for dtype, base in (("f32", 4321), ("f32", 8765), ("bf16", 4321)):
        rng = np.random.Generator(np.random.PCG64(base + (dtype == "bf16")))
        done = 0
        while done < 10:
            chain = random_conv_chain(rng, dtype)
            if chain is None:
                continue
            t = workloads.make_tensors(chain, zero_bias=False, seed=int(rng.integers(1, 1 << 30)))
            heights = [sh[2] for sh in planner.infer_shapes(chain)]
            sched = workloads.random_schedule(heights, seed=int(rng.integers(1, 1 << 30)), overlap=2)
            plan = lop.Plan(chain, t, 1)
            d_in, d_out, h_out = buffers(chain, plan)
            plan.run_two_party(d_in, d_out, [(a["M"], a["R"]) for a in sched], 1e12, 0.0)
            release(h_out)
            plan.destroy()
            done += 1
            n += 1
    return n


def main():
    total = scheduling_model_and_two_party()
    print("two-party sequences replayed:", total, flush=True)
    total += random_chain_sets()
    print("random chains replayed:", total, flush=True)
    total += named_workloads()
    print("plans replayed:", total, "kernel launches:", stub.hipstub_launches(), flush=True)
    leaks = {k: stub.hipstub_live(i) for i, k in enumerate(KINDS) if stub.hipstub_live(i)}
    if leaks:
        print("LEAKED HIP objects after every plan was destroyed:", leaks, flush=True)
        sys.exit(1)
    print("REPLAY OK", flush=True)


if __name__ == "__main__":
    main()
