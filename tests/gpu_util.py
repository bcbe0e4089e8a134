"""Helpers for the GPU parity tests: move seeded host tensors to the device in the
library's layout (NHWC, storage type), run the C-ABI path, bring the result back NCHW."""
import numpy as np
import torch

from paper_2507_05829_amd import lop

TOL = {"f32": 1e-4, "bf16": 2e-2}   # max |gpu - oracle| / max |oracle|


def to_device_nhwc(x_nchw: np.ndarray, dtype: str) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(x_nchw.transpose(0, 2, 3, 1)))
    if dtype == "bf16":
        t = t.to(torch.bfloat16)           # exact: values are bf16-representable
    t = t.cuda()
    torch.cuda.synchronize()
    return t


MARGIN = 2048          # elements of NaN in front of and behind every output buffer
_PARENTS = {}          # data_ptr of an output view -> the padded buffer it lives in


def empty_out(shape_nchw, dtype: str, pinned: bool = False) -> torch.Tensor:
    """NaN-filled NHWC output buffer that sits in the middle of a larger NaN-filled allocation,
    so that a store in front of or behind the buffer lands in memory check_margins looks at."""
    n, c, h, w = shape_nchw
    td = torch.bfloat16 if dtype == "bf16" else torch.float32
    numel = n * h * w * c
    if pinned:
        parent = torch.empty(numel + 2 * MARGIN, dtype=td, pin_memory=True)
    else:
        parent = torch.empty(numel + 2 * MARGIN, dtype=td, device="cuda")
    parent.fill_(float("nan"))
    torch.cuda.synchronize()
    t = parent[MARGIN:MARGIN + numel].view(n, h, w, c)
    _PARENTS[t.data_ptr()] = parent
    return t


def check_margins(*tensors) -> None:
    """The memory around output buffers made by empty_out is still NaN."""
    torch.cuda.synchronize()
    for t in tensors:
        if t is None:
            continue
        parent = _PARENTS.pop(t.data_ptr(), None)
        if parent is None:
            continue
        numel = t.numel()
        for part, name in ((parent[:MARGIN], "in front of"), (parent[MARGIN + numel:], "behind")):
            assert bool(torch.isnan(part.float()).all()), f"a kernel or copy stored {name} its output buffer"


def to_nchw(t: torch.Tensor) -> np.ndarray:
    return t.float().cpu().numpy().transpose(0, 3, 1, 2)


def run_gpu(chain, tensors, n_bands=None, use_host=True, flags=0):
    """Whole chain through lop_run_chain; returns (device result, host result) as NCHW."""
    plan = lop.Plan(chain, tensors, n_bands, flags)
    try:
        d_in = to_device_nhwc(tensors.x, chain.dtype)
        d_out = empty_out(plan.out_shape(), chain.dtype)
        h_out = empty_out(plan.out_shape(), chain.dtype, pinned=True) if use_host else None
        torch.cuda.synchronize()
        plan.run_chain(d_in, d_out, h_out)
        plan.synchronize()
        check_margins(d_out, h_out)
        return to_nchw(d_out), (to_nchw(h_out) if use_host else None)
    finally:
        plan.destroy()


def rel_err(got: np.ndarray, want: np.ndarray) -> float:
    scale = float(np.abs(want).max())
    return float(np.abs(got.astype(np.float64) - want.astype(np.float64)).max()) / max(scale, 1e-30)


def elementwise_err(got: np.ndarray, want: np.ndarray) -> float:
    """Second error figure: max over elements of |gpu - oracle| / max(|oracle|, 1e-3 max|oracle|)
    (a floor under the denominator because ReLU outputs hold exact zeros)."""
    w = np.abs(want.astype(np.float64))
    return float((np.abs(got.astype(np.float64) - want.astype(np.float64)) / np.maximum(w, 1e-3 * w.max())).max())
