"""lop_run_chain_static (scratch in the library's static device array, no allocation in the
call) against lop_run_chain on the same plan: bit for bit, two calls in a row on the shared
array, the second with a smaller input; then both against the oracle. Collected last: the
array is shared by everything in the process."""
import numpy as np
import pytest
import torch

import workloads
from gpu_util import TOL, empty_out, rel_err, to_device_nhwc, to_nchw
from paper_2507_05829_amd import lop

pytestmark = pytest.mark.gpu


def _both(chain, t, flags=0, stream=None):
    plan = lop.Plan(chain, t, None, flags)
    try:
        assert plan.stats()[2] <= lop.LOP_STATIC_SCRATCH_BYTES
        d_in = to_device_nhwc(t.x, chain.dtype)
        ref = empty_out(plan.out_shape(), chain.dtype)
        got = empty_out(plan.out_shape(), chain.dtype)
        plan.run_chain(d_in, ref, None)
        plan.synchronize()
        plan.run_chain_static(d_in, got, stream)
        if stream is not None:
            stream.synchronize()
        torch.cuda.synchronize()
        return to_nchw(ref), to_nchw(got)
    finally:
        plan.destroy()


@pytest.mark.parametrize("mode", [0, lop.LOP_FLAG_REUSE])
def test_static_scratch_two_calls_second_smaller(oracle, mode):
    big = workloads.resnet18_chain(h=96, w=80)            # fp32, split-K layers use the workspace
    small = workloads.resnet18_chain(h=64, w=48)
    stream = torch.cuda.Stream()
    for chain, s in ((big, stream), (small, None), (big, None)):
        t = workloads.make_tensors(chain, zero_bias=False)
        ref, got = _both(chain, t, mode, s)
        assert not np.isnan(got).any()
        np.testing.assert_array_equal(got, ref)
        assert rel_err(got, oracle.run_chain(chain, t)) <= TOL[chain.dtype]


def test_static_scratch_bf16_chains(oracle):
    for chain in (workloads.vgg16_chain(h=64, w=64), workloads.detector_chain(h=96, w=64),
                  workloads.mbv2_chain(h=32, w=32, n=2, n_bands=4), workloads.tiny_chain()):
        t = workloads.make_tensors(chain, zero_bias=False)
        ref, got = _both(chain, t)
        np.testing.assert_array_equal(got, ref)
        assert rel_err(got, oracle.run_chain(chain, t)) <= TOL[chain.dtype]


def test_static_scratch_rejects_a_plan_that_does_not_fit():
    chain = workloads.mbv2_chain(h=640, w=640, n=2, n_bands=2)     # layer by layer: > 64 MiB of slabs
    t = workloads.make_tensors(chain)
    plan = lop.Plan(chain, t, None, lop.LOP_FLAG_NO_FUSE | lop.LOP_FLAG_LANES(1))
    try:
        assert plan.stats()[2] > lop.LOP_STATIC_SCRATCH_BYTES
        d_in = to_device_nhwc(t.x, chain.dtype)
        d_out = empty_out(plan.out_shape(), chain.dtype)
        with pytest.raises(lop.LopError) as e:
            plan.run_chain_static(d_in, d_out)
        assert e.value.code == lop.LOP_ERR_TOO_LARGE
        torch.cuda.synchronize()
        assert torch.isnan(d_out.float()).all()          # nothing was enqueued
    finally:
        plan.destroy()
