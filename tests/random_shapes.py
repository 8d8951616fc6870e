"""Seeded random shapes shared by the CPU schedule test and the GPU parity test: few rows with long prefixes
(key splits), short prefixes with many rows (row splits), ragged everything."""
import numpy as np


def random_shapes(n=12, seed=2024):
    rng = np.random.default_rng(seed)
    out = []
    for i in range(n):
        Hkv = int(rng.choice([1, 2, 4]))
        group = int(rng.choice([1, 2, 4, 7]))
        D = int(rng.choice([64, 128]))
        kind = i % 3
        if kind == 0:      # few rows, long prefix
            P = int(rng.integers(600, 4000))
            lens = [int(v) for v in rng.integers(1, 40, size=int(rng.integers(1, 4)))]
        elif kind == 1:    # short prefix, many rows
            P = int(rng.integers(1, 400))
            lens = [int(v) for v in rng.integers(400, 1500, size=int(rng.integers(2, 6)))]
        else:              # anything
            P = int(rng.integers(0, 1500))
            lens = [int(v) for v in rng.integers(1, 300, size=int(rng.integers(1, 6)))]
        out.append((Hkv * group, Hkv, D, P, tuple(lens)))
    return out
