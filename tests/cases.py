"""Seeded draws of shapes and options shared by the GPU parity sweeps and by the host-side
plan tests (which check that the draws reach the kernels the sweeps are meant to cover)."""
import numpy as np


def sweep_draws():
    """60 draws over (B, H, L, U, c, dtype, value distribution, ragged lengths, rule for u, fill)."""
    r = np.random.Generator(np.random.PCG64(20260))
    for k in range(60):
        dtype = "bf16" if r.random() < 0.5 else "f32"
        B, H = int(r.integers(1, 5)), int(r.integers(1, 6))
        L = int(r.choice([int(r.integers(1, 140)), int(r.integers(140, 700)), int(r.integers(700, 1300)),
                          int(r.integers(1300, 2600))]))
        U = int(r.choice([1, 3, 8, 12, 17, 32, 40, 41, 47]))
        c = float(r.choice([0.5, 1.0, 3.0, 5.0, 9.0]))
        ragged = bool(r.random() < 0.5) and L > 4
        values = str(r.choice(["normal", "mixture", "peaky"]))
        mode = int(r.integers(0, 4))
        r_sparse, fill = None, "mean"
        if mode == 1:
            r_sparse, fill = float(r.choice([0.1, 0.5, 0.9])), "value"
        elif mode == 2:
            r_sparse = float(r.choice([0.25, 0.5]))
        elif mode == 3:
            fill = "value"
        yield dict(k=k, B=B, H=H, L=L, U=U, c=c, dtype=dtype, values=values, ragged=ragged, mode=mode,
                   r_sparse=r_sparse, fill=fill)


def long_head_draws():
    """16 draws with 1025..17500 frames."""
    r = np.random.Generator(np.random.PCG64(20261))
    for k in range(16):
        dtype = "bf16" if r.random() < 0.6 else "f32"
        B, H = int(r.integers(1, 4)), int(r.integers(1, 5))
        L = int(r.choice([int(r.integers(1025, 2049)), int(r.integers(2049, 4200)), int(r.integers(4200, 9000)),
                          int(r.integers(9000, 17500))]))
        U = int(r.choice([4, 16, 33, 40, 44]))
        c = float(r.choice([1.0, 5.0, 12.0, 30.0]))
        ragged = bool(r.random() < 0.5)
        values = str(r.choice(["normal", "mixture", "peaky"]))
        mode = int(r.integers(0, 3))
        r_sparse, fill = None, "mean"
        if mode == 1:
            r_sparse, fill = float(r.choice([0.02, 0.1])), "value"
        elif mode == 2:
            fill = "value"
        yield dict(k=k, B=B, H=H, L=L, U=U, c=c, dtype=dtype, values=values, ragged=ragged, mode=mode,
                   r_sparse=r_sparse, fill=fill)


def many_head_draws():
    """16 draws with 8..384 heads, 64..1100 frames and a few dozen to a few hundred kept queries;
    mode 2 stands for caller-given index sets of row stride `stride`."""
    r = np.random.Generator(np.random.PCG64(20262))
    for k in range(16):
        dtype = "bf16" if r.random() < 0.5 else "f32"
        B, H = int(r.integers(4, 49)), int(r.choice([2, 4, 8]))
        L = int(r.integers(64, 1101))
        U = int(r.choice([4, 16, 32]))
        c = float(r.choice([5.0, 12.0, 20.0, 30.0, 40.0]))
        ragged = bool(r.random() < 0.6)
        values = str(r.choice(["normal", "mixture", "peaky"]))
        mode = int(r.integers(0, 3))
        stride = int(r.integers(1, min(L, 700) + 1))
        fill = "mean" if mode == 0 else "value" if mode == 1 else str(r.choice(["mean", "value"]))
        yield dict(k=k, B=B, H=H, L=L, U=U, c=c, dtype=dtype, values=values, ragged=ragged, mode=mode,
                   stride=stride, fill=fill)
