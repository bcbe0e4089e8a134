"""Pins for the C oracle's operators: brute force, closed forms, library special cases.

Each pin is chosen so a plausible slip in the oracle (dropped tap, flipped kernel,
wrong stride/padding/dilation index, transposed weight, zero instead of -inf
padding, wrong rounding) fails at least one of them.
"""
import itertools

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from workloads import Layer, CONV, DWCONV, MAXPOOL, ELTWISE


def _conv(oracle, x, w, b=None, s=1, p=0, d=1, groups=1, act="none", dtype="f32", res=None,
          rows=None):
    n, c, h, wid = x.shape
    co = w.shape[0]
    pair = lambda v: (v, v) if isinstance(v, int) else tuple(v)
    L = Layer(DWCONV if groups == c and groups > 1 else CONV, c, co, (w.shape[2], w.shape[3]),
              pair(s), pair(p), pair(d), act)
    if groups not in (1, c):
        raise ValueError
    from oracle import planner
    ho = planner.out_size(h, L.k[0], L.s[0], L.p[0], L.d[0])
    wo = planner.out_size(wid, L.k[1], L.s[1], L.p[1], L.d[1])
    lo, hi = (0, ho) if rows is None else rows
    rs = None if res is None else oracle.Slab(res, 0, ho)
    return oracle.run_layer(L, oracle.Slab(x, 0, h), np.ascontiguousarray(w, np.float32),
                            b, rs, dtype, lo, hi - lo, ho, wo).data


def _brute_conv(x, w, b, s, p, d, groups):
    """Seven nested loops, python floats (double), written from the definition."""
    n_, c_, h_, w_ = x.shape
    co_, cig, kh, kw = w.shape
    ho = (h_ + 2 * p[0] - d[0] * (kh - 1) - 1) // s[0] + 1
    wo = (w_ + 2 * p[1] - d[1] * (kw - 1) - 1) // s[1] + 1
    cog = co_ // groups
    y = np.zeros((n_, co_, ho, wo))
    for n in range(n_):
        for co in range(co_):
            for oh in range(ho):
                for ow in range(wo):
                    acc = 0.0 if b is None else float(b[co])
                    for cl in range(cig):
                        for a in range(kh):
                            for bb in range(kw):
                                ih = oh * s[0] - p[0] + a * d[0]
                                iw = ow * s[1] - p[1] + bb * d[1]
                                if 0 <= ih < h_ and 0 <= iw < w_:
                                    ci = (co // cog) * cig + cl
                                    acc += float(x[n, ci, ih, iw]) * float(w[co, cl, a, bb])
                    y[n, co, oh, ow] = acc
    return y


@pytest.mark.parametrize("k,s,p,d,groups", [
    ((3, 3), (1, 1), (1, 1), (1, 1), 1),
    ((3, 2), (2, 1), (1, 0), (1, 2), 1),
    ((1, 1), (2, 2), (0, 0), (1, 1), 1),
    ((3, 3), (2, 2), (1, 1), (1, 1), 3),
    ((2, 3), (1, 2), (2, 1), (2, 1), 1),
])
def test_conv_brute_force(oracle, k, s, p, d, groups):
    rng = np.random.default_rng(1)
    x = rng.standard_normal((2, 3, 6, 5)).astype(np.float32)
    co = 3 if groups == 3 else 4
    w = rng.standard_normal((co, 3 // groups, *k)).astype(np.float32)
    b = rng.standard_normal(co).astype(np.float32)
    got = _conv(oracle, x, w, b, s, p, d, groups)
    want = _brute_conv(x, w, b, s, p, d, groups).astype(np.float32)
    np.testing.assert_array_equal(got, want)


def test_conv_all_ones_counts_taps(oracle):
    """3x3 p1 on all-ones: 9*C_in interior, 6*C_in edges, 4*C_in corners."""
    c_in = 5
    x = np.ones((1, c_in, 6, 7), np.float32)
    w = np.ones((2, c_in, 3, 3), np.float32)
    y = _conv(oracle, x, w, None, 1, 1)
    assert y.shape == (1, 2, 6, 7)
    assert np.all(y[:, :, 1:-1, 1:-1] == 9 * c_in)
    assert np.all(y[:, :, 0, 1:-1] == 6 * c_in) and np.all(y[:, :, 1:-1, -1] == 6 * c_in)
    for hh, ww in itertools.product((0, -1), (0, -1)):
        assert np.all(y[:, :, hh, ww] == 4 * c_in)


def test_conv_impulse_is_mirrored_kernel(oracle):
    """Unit impulse at (h0,w0), s=1: y[oh,ow] = w[h0-oh+p, w0-ow+p] (no kernel flip)."""
    rng = np.random.default_rng(2)
    w = rng.standard_normal((1, 1, 3, 3)).astype(np.float32)
    x = np.zeros((1, 1, 7, 7), np.float32)
    h0, w0, p = 3, 4, 1
    x[0, 0, h0, w0] = 1.0
    y = _conv(oracle, x, w, None, 1, p)
    for oh in range(7):
        for ow in range(7):
            a, b = h0 - oh + p, w0 - ow + p
            want = w[0, 0, a, b] if 0 <= a < 3 and 0 <= b < 3 else 0.0
            assert y[0, 0, oh, ow] == want


def test_conv_centre_tap_is_identity(oracle):
    rng = np.random.default_rng(3)
    x = rng.standard_normal((2, 4, 5, 6)).astype(np.float32)
    w = np.zeros((4, 4, 3, 3), np.float32)
    for c in range(4):
        w[c, c, 1, 1] = 1.0
    np.testing.assert_array_equal(_conv(oracle, x, w, None, 1, 1), x)


def test_conv1x1_is_row_wise_matrix_product(oracle):
    """Eq. (1): each NHWC pixel row times the full weight matrix; no other row is read."""
    rng = np.random.default_rng(4)
    x = rng.integers(-3, 4, (2, 6, 4, 5)).astype(np.float32)
    w = rng.integers(-3, 4, (7, 6, 1, 1)).astype(np.float32)
    y = _conv(oracle, x, w)
    a = x.transpose(0, 2, 3, 1).reshape(-1, 6).astype(np.float64)
    c = (a @ w[:, :, 0, 0].T.astype(np.float64)).reshape(2, 4, 5, 7).transpose(0, 3, 1, 2)
    np.testing.assert_array_equal(y, c.astype(np.float32))


def test_depthwise_equals_block_diagonal_dense(oracle):
    rng = np.random.default_rng(5)
    c = 6
    x = rng.standard_normal((1, c, 8, 7)).astype(np.float32)
    wd = rng.standard_normal((c, 1, 3, 3)).astype(np.float32)
    dense = np.zeros((c, c, 3, 3), np.float32)
    for i in range(c):
        dense[i, i] = wd[i, 0]
    got = _conv(oracle, x, wd, None, 2, 1, 1, groups=c)
    want = _conv(oracle, x, dense, None, 2, 1, 1)
    np.testing.assert_array_equal(got, want)


@pytest.mark.parametrize("k,s,p,d,groups", [
    (3, 1, 1, 1, 1), (3, 2, 1, 1, 1), (7, 2, 3, 1, 1), (1, 2, 0, 1, 1), (3, 1, 2, 2, 1),
    (3, 2, 1, 1, 8), ((3, 1), (1, 2), (1, 0), (1, 1), 1),
])
def test_conv_against_library(oracle, k, s, p, d, groups):
    """torch's float64 CPU conv2d as an independent third party."""
    rng = np.random.default_rng(6)
    kk = (k, k) if isinstance(k, int) else k
    x = rng.standard_normal((2, 8, 13, 11)).astype(np.float32)
    w = rng.standard_normal((16 if groups == 1 else 8, 8 // groups, *kk)).astype(np.float32)
    b = rng.standard_normal(w.shape[0]).astype(np.float32)
    got = _conv(oracle, x, w, b, s, p, d, groups)
    want = F.conv2d(torch.from_numpy(x).double(), torch.from_numpy(w).double(),
                    torch.from_numpy(b).double(), s, p, d, groups).numpy()
    np.testing.assert_allclose(got, want, rtol=0, atol=2e-6 * np.abs(want).max())


def test_small_integers_exact_any_order(oracle):
    """Small integers: the library (another summation order) must match bit for bit."""
    rng = np.random.default_rng(7)
    x = rng.integers(0, 4, (1, 16, 9, 9)).astype(np.float32)
    w = rng.integers(-2, 3, (8, 16, 3, 3)).astype(np.float32)
    got = _conv(oracle, x, w, None, 1, 1)
    want = F.conv2d(torch.from_numpy(x), torch.from_numpy(w), None, 1, 1).numpy()
    np.testing.assert_array_equal(got, want)


def test_conv_row_interval_equals_rows_of_full(oracle):
    rng = np.random.default_rng(8)
    x = rng.standard_normal((1, 3, 12, 6)).astype(np.float32)
    w = rng.standard_normal((4, 3, 3, 3)).astype(np.float32)
    full = _conv(oracle, x, w, None, 2, 1)
    part = _conv(oracle, x, w, None, 2, 1, rows=(2, 5))
    np.testing.assert_array_equal(part, full[:, :, 2:5])


def test_conv_refuses_rows_outside_slab(oracle):
    """A tap inside the image but outside the slab is an error, not silent zero padding."""
    x = np.ones((1, 1, 4, 4), np.float32)
    w = np.ones((1, 1, 3, 3), np.float32)
    L = Layer(CONV, 1, 1, (3, 3), (1, 1), (1, 1), (1, 1))
    slab = oracle.Slab(x[:, :, 1:3], 1, 4)         # holds rows 1,2 of 4
    with pytest.raises(RuntimeError):
        oracle.run_layer(L, slab, w, None, None, "f32", 1, 2, 4, 4)   # rows 1,2 need 0..3
    ok = oracle.run_layer(L, oracle.Slab(x, 0, 4), w, None, None, "f32", 1, 2, 4, 4)
    assert ok.data.shape == (1, 1, 2, 4)


# ------------------------------------------------------------------ pooling

def _pool(oracle, x, k, s, p):
    from oracle import planner
    n, c, h, w = x.shape
    L = Layer(MAXPOOL, c, c, (k, k), (s, s), (p, p))
    ho, wo = planner.out_size(h, k, s, p, 1), planner.out_size(w, k, s, p, 1)
    return oracle.run_layer(L, oracle.Slab(x, 0, h), None, None, None, "f32", 0, ho, ho, wo).data


@pytest.mark.parametrize("k,s,p", [(3, 2, 1), (2, 2, 0), (3, 1, 1)])
def test_pool_monotone_closed_form(oracle, k, s, p):
    """x[h,w] = h*W + w is increasing, so the max is the window's last in-range tap."""
    h, w = 9, 10
    x = (np.arange(h)[:, None] * w + np.arange(w)[None, :]).astype(np.float32)[None, None]
    y = _pool(oracle, x, k, s, p)
    for oh in range(y.shape[2]):
        for ow in range(y.shape[3]):
            ih = min(oh * s - p + k - 1, h - 1)
            iw = min(ow * s - p + k - 1, w - 1)
            assert y[0, 0, oh, ow] == ih * w + iw


def test_pool_padding_is_minus_infinity_not_zero(oracle):
    x = -np.ones((1, 2, 5, 5), np.float32) * 3
    y = _pool(oracle, x, 3, 2, 1)
    assert np.all(y == -3)


def test_pool_against_library(oracle):
    rng = np.random.default_rng(9)
    x = rng.standard_normal((2, 3, 11, 12)).astype(np.float32)
    for k, s, p in [(3, 2, 1), (2, 2, 0)]:
        want = F.max_pool2d(torch.from_numpy(x), k, s, p).numpy()
        np.testing.assert_array_equal(_pool(oracle, x, k, s, p), want)


# ------------------------------------------------------------------ element-wise

def test_epilogue_values(oracle):
    v = np.array([-1, 0, 3, 6, 7], np.float32).reshape(1, 1, 1, 5)
    zero = np.zeros_like(v)
    for act, want in (("none", [-1, 0, 3, 6, 7]), ("relu", [0, 0, 3, 6, 7]),
                      ("relu6", [0, 0, 3, 6, 6])):
        L = Layer(ELTWISE, 1, 1, act=act)
        y = oracle.run_layer(L, oracle.Slab(v, 0, 1), None, None, None, "f32", 0, 1, 1, 5).data
        assert y.ravel().tolist() == want
    # bias and residual are added before the activation
    L = Layer(ELTWISE, 1, 1, act="relu6")
    y = oracle.run_layer(L, oracle.Slab(v, 0, 1), None, np.array([1.0], np.float32),
                         oracle.Slab(zero + 2, 0, 1), "f32", 0, 1, 1, 5).data
    assert y.ravel().tolist() == [2, 3, 6, 6, 6]


def test_conv_epilogue_order_bias_residual_then_act(oracle):
    x = np.ones((1, 1, 3, 3), np.float32)
    w = -np.ones((1, 1, 1, 1), np.float32)
    b = np.array([0.25], np.float32)
    r = np.full((1, 1, 3, 3), 2.0, np.float32)
    y = _conv(oracle, x, w, b, act="relu", res=r)
    assert np.all(y == 1.25)                      # relu(-1 + 0.25 + 2)
    y = _conv(oracle, x, w, b, act="relu")
    assert np.all(y == 0.0)                       # relu(-0.75)


# ------------------------------------------------------------------ bf16 storage

def test_bf16_rounding_hand_values(oracle):
    r = oracle.round_bf16
    assert r(1 + 2 ** -8) == 1.0                        # tie -> even (down)
    assert r(1 + 3 * 2 ** -8) == 1 + 2 ** -6            # tie -> even (up)
    assert r(1 + 2 ** -8 + 2 ** -16) == 1 + 2 ** -7     # just above the tie
    assert r(-(1 + 3 * 2 ** -8)) == -(1 + 2 ** -6)
    assert r(255.5) == 256.0 and r(0.0) == 0.0
    assert r(2.0 ** 127 * 1.998) == float("inf")        # above the largest bf16 -> overflow
    assert r(2.0 ** -133) == 2.0 ** -133 and r(2.0 ** -135) == 0.0   # subnormal grid


def test_bf16_rounding_against_library(oracle):
    rng = np.random.default_rng(10)
    v = np.concatenate([rng.standard_normal(2000) * 10.0 ** rng.integers(-6, 6, 2000),
                        [1 + 2 ** -8, 1 + 3 * 2 ** -8, 0.1, -0.1, 65504.0]]).astype(np.float32)
    want = torch.from_numpy(v).to(torch.bfloat16).float().numpy()
    got = np.array([oracle.round_bf16(float(t)) for t in v], np.float32)
    np.testing.assert_array_equal(got, want)


def test_bf16_layer_output_is_rounded_once(oracle):
    """Sum 1 + 2^-9 + 2^-9 = 1 + 2^-8 exactly (a tie) -> 1.0; rounding each partial
    sum instead would also give 1.0, but 1 + 3*2^-9 + 3*2^-9 = 1 + 3*2^-8 -> 1 + 2^-6."""
    x = np.array([1.0, 2.0 ** -9, 2.0 ** -9], np.float32).reshape(1, 3, 1, 1)
    w = np.ones((1, 3, 1, 1), np.float32)
    assert _conv(oracle, x, w, dtype="bf16").item() == 1.0
    w[0, 1:] = 3.0
    assert _conv(oracle, x, w, dtype="bf16").item() == np.float32(1 + 2 ** -6)
    assert _conv(oracle, x, w, dtype="f32").item() == np.float32(1 + 3 * 2 ** -8)
