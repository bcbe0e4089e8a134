"""Seeded random chain descriptions for the parity tests and the host-code replay: layer
hyper-parameters only (no tensors, no arithmetic of the method beyond asking the planner
oracle for the running output shape so that every drawn window fits)."""
import workloads


def random_conv_chain(rng, dtype):
    """Two to four layers with random (valid) hyper-parameters, channel counts that are and are
    not multiples of the vector width, an optional residual and pool, random band count."""
    vec = 8 if dtype == "bf16" else 4
    n = int(rng.choice([1, 1, 2, 3]))
    h, w = int(rng.integers(9, 40)), int(rng.integers(5, 33))
    c = int(rng.choice([3, vec, 2 * vec, 24, 5 * vec, 64, 96]))
    chain = workloads.Chain("rand", (n, c, h, w), dtype, int(rng.integers(1, 7)))
    for _ in range(int(rng.integers(2, 5))):
        kind = rng.choice(["conv", "conv", "conv", "dw", "pool", "pw"])
        hh = workloads_h(chain)
        if kind == "conv":
            k = int(rng.choice([1, 2, 3, 3, 5])); d = int(rng.choice([1, 1, 2]))
            p = int(rng.integers(0, d * (k - 1) // 2 + 1)); s_ = int(rng.choice([1, 1, 2]))
            if hh + 2 * p - d * (k - 1) < 2 or min_w(chain) + 2 * p - d * (k - 1) < 2:
                continue
            c_out = int(rng.choice([vec, 2 * vec, 6, 40, 64, 72, 128]))
            same = (c_out == c and s_ == 1 and 2 * p == d * (k - 1))
            res = len(chain.layers) - 1 if (same and rng.random() < 0.5) else workloads.NO_RESIDUAL
            chain.add(workloads.CONV, c, c_out, k, s_, p, d, str(rng.choice(["none", "relu", "relu6"])),
                      residual_from=res)
            c = c_out
        elif kind == "pw":
            c_out = int(rng.choice([32, 64, 96, 192])) if dtype == "bf16" else int(rng.choice([vec, 48]))
            chain.add(workloads.CONV, c, c_out, 1, 1, 0, 1, str(rng.choice(["none", "relu6"])))
            c = c_out
        elif kind == "dw":
            s_ = int(rng.choice([1, 2]))
            if hh < 3 or min_w(chain) < 3:
                continue
            chain.add(workloads.DWCONV, c, c, 3, s_, 1, 1, str(rng.choice(["relu6", "none"])))
        else:
            if hh < 4 or min_w(chain) < 4:
                continue
            chain.add(workloads.MAXPOOL, c, c, 2, 2, 0, 1, "none", has_bias=False)
    return chain if chain.layers else None


def workloads_h(chain):
    from oracle import planner
    return planner.infer_shapes(chain)[-1][2] if chain.layers else chain.in_shape[2]


def min_w(chain):
    from oracle import planner
    return planner.infer_shapes(chain)[-1][3] if chain.layers else chain.in_shape[3]
