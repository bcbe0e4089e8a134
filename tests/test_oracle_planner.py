"""Pins for the planner oracle: library band split, worked halo example, receptive-field
closed forms, brute-force reachability, and the partition/contiguity invariants."""
import os

import numpy as np
import pytest

import workloads
from oracle import planner

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rows(path):
    with open(os.path.join(GOLDEN, path)) as f:
        return [l.split() for l in f if l.strip() and not l.startswith("#")]


@pytest.mark.parametrize("h,b", [(32, 4), (7, 4), (7, 8), (45, 16), (160, 8), (1, 1), (5, 7), (0, 3)])
def test_band_split_is_array_split(h, b):
    want = [(int(a[0]), int(a[-1]) + 1) if len(a) else None
            for a in np.array_split(np.arange(h), b)]
    got = planner.split_rows(h, b)
    assert len(got) == b
    for g, w in zip(got, want):
        if w is None:
            assert g[0] == g[1]
        else:
            assert g == w
    assert got[0][0] == 0 and got[-1][1] == h
    assert all(got[i][1] == got[i + 1][0] for i in range(b - 1))


def test_tiny_two_row_halo_golden():
    chain = workloads.tiny_chain()
    plans = planner.plan(chain)
    for row in _rows("tiny_band_rows.txt"):
        b, olo, ohi, l0lo, l0hi, ilo, ihi = map(int, row)
        assert plans[b][1] == (olo, ohi)
        assert plans[b][0] == (l0lo, l0hi)
        assert plans[b][-1] == (ilo, ihi)


def _main_path(chain):
    idx, i = [], len(chain.layers) - 1
    while i >= 0:
        idx.append(i)
        i = chain.layers[i].input_from
    return [chain.layers[j] for j in reversed(idx)]


def test_receptive_field_golden_and_brute_force():
    """RF recurrence == hand-worked values == span the brute-force marking reaches."""
    tall = {"tiny": dict(), "vgg16": dict(h=1024, w=8), "detector720p": dict(h=1024, w=8),
            "mbv2": dict(h=256, w=8, n=1), "resnet18": dict(h=2048, w=8)}
    for name, rf in _rows("receptive_fields.txt"):
        rf = int(rf)
        chain = workloads.CONFIGS[name](**tall[name])
        assert planner.receptive_field_rows(_main_path(chain)) == rf
        h_out = planner.infer_shapes(chain)[-1][2]
        mid = h_out // 2
        need = planner.plan_brute_force(chain, (mid, mid + 1))
        lo, hi = need[-1]
        assert lo > 0 and hi < chain.in_shape[2], "pick a taller input: the field is clamped"
        assert hi - lo == rf


@pytest.mark.parametrize("n,k,d", [(1, 3, 1), (2, 3, 1), (4, 3, 1), (3, 5, 1), (2, 3, 2)])
def test_stacked_convs_halo_closed_form(n, k, d):
    """n stacked kxk stride-1 'same' convs need a halo of n*d*(k-1)/2 rows per side."""
    c = workloads.Chain("stack", (1, 4, 64, 8), "f32", 4)
    for _ in range(n):
        c.add(workloads.CONV, 4, 4, k, 1, d * (k - 1) // 2, d)
    halo = n * d * (k - 1) // 2
    for b, need in enumerate(planner.plan(c)):
        lo, hi = 16 * b, 16 * (b + 1)
        assert need[-1] == (max(lo - halo, 0), min(hi + halo, 64))


def _random_chain(rng):
    h = int(rng.integers(9, 40))
    c = workloads.Chain("rand", (1, 4, h, 6), "f32", int(rng.integers(1, 7)))
    n_layers = int(rng.integers(1, 7))
    for i in range(n_layers):
        kind = rng.integers(0, 5)
        src = int(rng.integers(-1, i)) if i and rng.random() < 0.3 else i - 1
        if kind == 0:
            c.add(workloads.MAXPOOL, 4, 4, int(rng.integers(2, 4)), int(rng.integers(1, 3)),
                  int(rng.integers(0, 2)), input_from=src)
        elif kind == 1:
            c.add(workloads.ELTWISE, 4, 4, act="relu", input_from=src)
        else:
            k = int(rng.integers(1, 5))
            d = int(rng.integers(1, 3))
            c.add(workloads.DWCONV if kind == 2 else workloads.CONV, 4, 4, k,
                  int(rng.integers(1, 3)), int(rng.integers(0, k)), d, input_from=src)
    # add residual edges wherever an earlier tensor has the same shape
    try:
        shapes = planner.infer_shapes(c)
    except AssertionError:
        return None
    if any(s[2] < 1 or s[3] < 1 for s in shapes):
        return None
    for i, L in enumerate(c.layers):
        if L.op == workloads.MAXPOOL:
            continue
        cands = [j for j in range(-1, i) if (c.in_shape if j < 0 else shapes[j]) == shapes[i]
                 and j != i]
        if cands and rng.random() < 0.5:
            L.residual_from = int(rng.choice(cands))
    return c


def test_closed_form_equals_brute_force_random_chains():
    rng = np.random.default_rng(11)
    done = 0
    while done < 150:
        c = _random_chain(rng)
        if c is None:
            continue
        done += 1
        h_out = planner.infer_shapes(c)[-1][2]
        dilated = any(L.d[0] > 1 and L.k[0] > 1 for L in c.layers)
        for br in planner.split_rows(h_out, c.n_bands):
            cf, bf = planner.plan_closed_form(c, br), planner.plan_brute_force(c, br)
            if not dilated:
                assert cf == bf, (c, br)
                continue
            # With dilation the clamped hull of the tap range may hold up to d-1 border
            # rows that no tap lands on: the closed form is then a superset, never less.
            for t in cf:
                if bf[t] is None:
                    continue
                assert cf[t] is not None and cf[t][0] <= bf[t][0] and bf[t][1] <= cf[t][1]


@pytest.mark.parametrize("name", list(workloads.CONFIGS))
def test_configs_closed_form_equals_brute_force_and_invariants(name):
    chain = workloads.CONFIGS[name]()
    shapes = planner.infer_shapes(chain)
    nl = len(chain.layers)
    bands = planner.split_rows(shapes[-1][2], chain.n_bands)
    cover = np.zeros(shapes[-1][2], int)
    for br in bands:
        cf = planner.plan_closed_form(chain, br)
        assert cf == planner.plan_brute_force(chain, br)
        if br[1] > br[0]:
            assert cf[nl - 1] == br                      # the band's own final rows
            cover[br[0]:br[1]] += 1
            for t, iv in cf.items():                     # inside the image, non-empty
                h = chain.in_shape[2] if t < 0 else shapes[t][2]
                assert iv is None or (0 <= iv[0] < iv[1] <= h)
        else:
            assert all(v is None for v in cf.values())
    assert np.all(cover == 1)                            # x_M u x_R = OP(v), disjoint here


def test_config_shapes_and_replication_ratios():
    """Shapes the workload descriptions fix, and executed/useful work ratios worked from
    the interval tables (independent bands recompute their halos)."""
    want_out = {"tiny": (1, 16, 32, 32), "resnet18": (1, 512, 7, 7), "vgg16": (1, 512, 7, 7),
                "detector720p": (1, 256, 45, 80), "mbv2": (8, 32, 160, 160)}
    n_layers = {"tiny": 2, "resnet18": 21, "vgg16": 18, "detector720p": 10, "mbv2": 18}
    for name, f in workloads.CONFIGS.items():
        chain = f()
        assert planner.infer_shapes(chain)[-1] == want_out[name]
        assert len(chain.layers) == n_layers[name]
    # tiny: layer 0 computes 9+10+10+9 = 38 of 32 rows, layer 1 exactly 32: (38+32)/64
    u, e = planner.flop_counts(workloads.tiny_chain())
    assert u == 2 * 2 * 32 * 32 * 16 * 16 * 9
    assert e / u == pytest.approx(70 / 64)
    # receptive field >= image: every resnet18 band needs the whole 224-row input
    for need in planner.plan(workloads.resnet18_chain()):
        assert need[-1] == (0, 224)
    # vgg16 with 8 bands over 7 rows: the last band is empty
    assert planner.plan(workloads.vgg16_chain())[7][17] is None


@pytest.mark.parametrize("name", list(workloads.CONFIGS))
def test_reuse_plan_invariants(name):
    """Reuse mode: the rows the bands compute of a layer are disjoint, their union is the
    union of the bands' needs, and in total nothing is computed twice: executed work equals
    the work of the rows that are needed at all (for these chains: every row)."""
    chain = workloads.CONFIGS[name]()
    shapes = planner.infer_shapes(chain)
    fresh = planner.plan_reuse(chain)
    need = [planner.plan_brute_force(chain, br)
            for br in planner.split_rows(shapes[-1][2], chain.n_bands)]
    for t in range(len(chain.layers)):
        seen = set()
        for b in range(chain.n_bands):
            if fresh[b][t] is not None:
                rows = set(range(*fresh[b][t]))
                assert not (rows & seen)
                seen |= rows
        needed = set()
        for b in range(chain.n_bands):
            if need[b][t] is not None:
                needed |= set(range(*need[b][t]))
        assert seen == needed
    u, e = planner.flop_counts_reuse(chain)
    assert e <= u * (1 + 1e-12)
    if name in ("tiny", "vgg16", "detector720p", "mbv2"):
        assert e == pytest.approx(u)        # every row of every layer is needed by some band
