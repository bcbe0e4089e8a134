"""The method's invariant on the CPU oracle: concatenating the bands' final rows
reproduces the unpartitioned chain bit for bit (Sec. IV-B: every local operation gets
the correct input and yields the correct output), and rows that two bands both compute
(local-operation replication, Sec. IV-C) are identical."""
import numpy as np
import pytest

import workloads
from oracle import planner


def _check(oracle, chain, t, n_bands=None):
    full = oracle.run_chain(chain, t)
    banded = oracle.run_chain_banded(chain, t, n_bands)
    assert not np.isnan(banded).any()
    np.testing.assert_array_equal(banded, full)
    return full


def test_tiny_banded_equals_unbanded(oracle):
    chain = workloads.tiny_chain()
    t = workloads.make_tensors(chain, zero_bias=False)
    full = _check(oracle, chain, t)
    assert full.shape == (1, 16, 32, 32) and full.max() > 0
    for b in (1, 2, 3, 5, 32, 40):
        _check(oracle, chain, t, b)


@pytest.mark.parametrize("name,kw", [
    ("resnet18", dict(h=64, w=48)),
    ("vgg16", dict(h=64, w=32)),
    ("detector720p", dict(h=90, w=64)),
    ("mbv2", dict(h=48, w=40, n=2)),
])
def test_scaled_configs_banded_equals_unbanded(oracle, name, kw):
    chain = workloads.CONFIGS[name](**kw)
    t = workloads.make_tensors(chain, zero_bias=False)
    _check(oracle, chain, t)
    _check(oracle, chain, t, 3)


def test_replicated_rows_are_identical(oracle):
    """Rows of an intermediate layer computed by two neighbouring bands agree bit for bit."""
    chain = workloads.tiny_chain()
    t = workloads.make_tensors(chain)
    plans = planner.plan(chain)
    sub = workloads.Chain("first", chain.in_shape, chain.dtype, 1, chain.layers[:1])
    full0 = oracle.run_chain(sub, t)
    for need in plans:
        lo, hi = need[0]
        slab = oracle.run_band(sub, t, {-1: need[-1], 0: need[0]})
        np.testing.assert_array_equal(slab.data, full0[:, :, lo:hi])


def test_band_never_reads_outside_its_slab(oracle):
    """Shrinking a band's input slab by one row makes the oracle refuse, so the planner's
    interval is not larger than needed at the chain input (d = 1)."""
    chain = workloads.tiny_chain()
    t = workloads.make_tensors(chain)
    need = dict(planner.plan(chain)[1])
    lo, hi = need[-1]
    for shrunk in ((lo + 1, hi), (lo, hi - 1)):
        bad = dict(need)
        bad[-1] = shrunk
        with pytest.raises(RuntimeError):
            oracle.run_band(chain, t, bad)
    assert oracle.run_band(chain, t, need).rows == 8


def test_bf16_chain_values_are_bf16(oracle):
    chain = workloads.vgg16_chain(h=32, w=32)
    t = workloads.make_tensors(chain)
    outs = oracle.run_chain(chain, t, keep_all=True)
    for o in outs:
        assert not np.any(o.view(np.uint32) & 0xFFFF)


@pytest.mark.parametrize("name,kw", [
    ("tiny", dict()),
    ("resnet18", dict(h=64, w=48)),
    ("vgg16", dict(h=64, w=32)),
    ("detector720p", dict(h=90, w=64)),
    ("mbv2", dict(h=48, w=40, n=2)),
])
def test_reuse_mode_equals_unbanded(oracle, name, kw):
    """Bands that reuse rows computed by earlier bands instead of recomputing them give the
    same chain output bit for bit, and no row is read before it exists (NaN poisoning)."""
    chain = workloads.CONFIGS[name](**kw)
    t = workloads.make_tensors(chain, zero_bias=False)
    full = oracle.run_chain(chain, t)
    for nb in (None, 3, 1):
        got = oracle.run_chain_reuse(chain, t, nb)
        assert not np.isnan(got).any()
        np.testing.assert_array_equal(got, full)
