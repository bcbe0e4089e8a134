"""Bandwidth study of the two-party runtime (Sec. IV-C scheduling + Sec. IV-D runtime, the
setting of the paper's bandwidth-sensitivity experiment) on one GPU.

For each bandwidth the library searches a schedule (lop_loss_solve with the link model of the
runtime, LOP_LINK_QUEUED), predicts its completion time T (Eq. 2) and then executes it with
lop_run_two_party, where both parties are streams of the one GPU slowed down to modelled
device speeds and the link is a timed wait. Device-only and server-only schedules run beside it. Synthetic weights and input; the device speeds are
parameters, not measurements of any robot.

    python -m paper_2507_05829_amd.two_party_study --workload resnet18 --bandwidths 1,2,5,10,20,50

prints a markdown table (times in ms; bandwidth in MB/s as in the paper's 0-50 MB range).
"""
from __future__ import annotations

import argparse
import os
import sys
from types import SimpleNamespace

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))

import numpy as np  # noqa: E402
import torch  # noqa: E402

import workloads  # noqa: E402
from paper_2507_05829_amd import lop  # noqa: E402


def cost_layers(chain, plan, m_flops: float, r_flops: float, fixed_m: float, fixed_r: float):
    """One lop_loss_layer_t-shaped object per layer: time = fixed + rows * (flop per row / rate);
    layers without multiply-adds are priced by the bytes they move at 1/10 byte per flop."""
    esz = 2 if chain.dtype == "bf16" else 4
    out = []
    for i, L in enumerate(chain.layers):
        n, c, h, w = plan.layer_shape(i)
        flop, nbytes = plan.layer_work(0, i)
        work = max(flop, 10.0 * nbytes)
        out.append(SimpleNamespace(
            n_ops=h, input_from=L.input_from, residual_from=L.residual_from,
            k=L.k[0] if L.op != "eltwise" else 1, s=L.s[0] if L.op != "eltwise" else 1,
            p=L.p[0] if L.op != "eltwise" else 0, d=L.d[0] if L.op != "eltwise" else 1,
            cm_fixed=fixed_m, cm_row=work / h / m_flops, cr_fixed=fixed_r, cr_row=work / h / r_flops,
            row_bytes=float(n * c * w * esz)))
    return out


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="resnet18", choices=[k for k in workloads.CONFIGS if k != "mlp"])
    ap.add_argument("--bandwidths", default="1,2,5,10,20,50", help="MB/s, comma separated")
    ap.add_argument("--latency-ms", type=float, default=1.0)
    ap.add_argument("--client-tflops", type=float, default=0.1)
    ap.add_argument("--server-tflops", type=float, default=2.0)
    ap.add_argument("--generations", type=int, default=150)
    ap.add_argument("--seed", type=int, default=1)
    a = ap.parse_args()

    chain = workloads.CONFIGS[a.workload]()
    t = workloads.make_tensors(chain)
    plan = lop.Plan(chain, t, 1, 0)
    td = torch.bfloat16 if chain.dtype == "bf16" else torch.float32
    d_in = torch.from_numpy(np.ascontiguousarray(t.x.transpose(0, 2, 3, 1))).to(td).cuda()
    n, c, h, w = plan.out_shape()
    d_out = torch.zeros((n, h, w, c), dtype=td, device="cuda")
    torch.cuda.synchronize()
    layers = cost_layers(chain, plan, a.client_tflops * 1e12, a.server_tflops * 1e12, 50e-6, 10e-6)
    ni, ci, hi, wi = chain.in_shape
    in_row_bytes = float(ni * ci * wi * (2 if chain.dtype == "bf16" else 4))
    only_m = [((0, L.n_ops), (0, 0)) for L in layers]
    only_r = [((0, 0), (0, L.n_ops)) for L in layers]
    lat = a.latency_ms * 1e-3

    print(f"workload {a.workload}, client {a.client_tflops} TFLOP/s, server {a.server_tflops} TFLOP/s, "
          f"latency {a.latency_ms} ms; T = predicted (Eq. 2), run = measured by lop_run_two_party\n")
    print("| MB/s | client only T / run | server only T / run | searched T / run | rows on client | to server MB | to client MB | messages |")
    print("|---|---|---|---|---|---|---|---|")
    for bw_mb in [float(x) for x in a.bandwidths.split(",")]:
        bw = bw_mb * 1e6
        cells = []
        for sched in (only_m, only_r):
            T = lop.lop_loss_eval(layers, hi, in_row_bytes, bw, lat, sched, lop.LOP_LINK_QUEUED)[0]
            st = plan.run_two_party(d_in, d_out, sched, bw, lat, layers)
            cells.append(f"{T * 1e3:.1f} / {st.total_ms:.1f}")
        best, T, viol = lop.lop_loss_solve(layers, hi, in_row_bytes, bw, lat, 0, a.generations, a.seed,
                                           lop.LOP_LINK_QUEUED)
        st = plan.run_two_party(d_in, d_out, best, bw, lat, layers)
        on_m = sum(m[1] - m[0] for m, _ in best) / sum(L.n_ops for L in layers)
        cells.append(f"{T * 1e3:.1f} / {st.total_ms:.1f}")
        print(f"| {bw_mb:g} | " + " | ".join(cells) +
              f" | {on_m:.2f} | {st.bytes_to_r / 1e6:.2f} | {st.bytes_to_m / 1e6:.2f} | {st.transfers} |", flush=True)
    plan.destroy()


if __name__ == "__main__":
    main()
