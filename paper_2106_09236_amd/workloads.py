"""Seeded synthetic inputs for the prob-sparse self-attention forward.

This module only draws numbers and converts storage formats.  It holds none of
the method's arithmetic (no scores, no measure, no selection, no softmax): both
the CPU oracle's tests and the HIP path's tests feed on the arrays made here,
so the two implementations see bit-identical inputs while sharing no code.

The paper evaluates on AISHELL-1 and LibriSpeech utterances run through a
Conformer encoder with 4 heads of 64 dims at 40 ms frames (Sec. 4.2); neither
the corpora nor a trained model are available, so the shapes of those
utterances (40..500 frames for corpus clips, up to 16384 frames for long-form
audio) are kept and the values are drawn from the distributions below.

Layout of every tensor: [B, H, L, d], C-contiguous, d fastest.
`sample_idx` is int32 [B, H, L, U]: the keys each query is scored against
(Sec. 3.2, the sampled key matrix), drawn uniformly with replacement from the
valid keys of its batch item.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np

BASE_SEED = 210609236
D_HEAD = 64


@dataclass(frozen=True)
class Config:
    """Shape and distribution of one workload."""
    name: str
    B: int
    H: int
    L: int
    U: int            # samples per query (last dim of sample_idx)
    c: float          # selection factor handed to the attention call
    dtype: str        # "f32" or "bf16": storage type of Q, K, V and out
    values: str       # "normal" | "peaky" | "mixture"
    ragged: bool = False
    len_lo: int = 0
    len_hi: int = 0
    seed_offset: int = 0


# The five benchmark workloads.  U is written out as a literal (it is an input
# shape, the number of columns of sample_idx), not computed here.
CONFIGS = {
    "tiny":        Config("tiny", 1, 4, 128, 25, 5.0, "f32", "normal", seed_offset=1),
    "conformer_s": Config("conformer_s", 16, 4, 512, 32, 5.0, "f32", "peaky", seed_offset=2),
    "ragged":      Config("ragged", 32, 4, 512, 32, 5.0, "bf16", "peaky", True, 40, 500, seed_offset=3),
    "conformer_l": Config("conformer_l", 8, 8, 2048, 39, 5.0, "bf16", "mixture", seed_offset=4),
    "longform":    Config("longform", 1, 8, 16384, 49, 5.0, "bf16", "mixture", seed_offset=5),
}


# ----------------------------------------------------------------------------
# bf16 storage helpers (format conversion only)
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even); returns uint16 bits.
    NaN stays NaN (quiet bit forced)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    r = ((u + bias) >> np.uint32(16)).astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        r = np.where(nan, ((u >> np.uint32(16)) | np.uint32(0x40)).astype(np.uint16), r)
    return r


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen uint16 bfloat16 bits to float32 (exact)."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass
class Workload:
    """One drawn batch.  Q/K/V are float32 for dtype "f32" and uint16 bfloat16
    bit patterns for dtype "bf16"; `as_f64` widens either to float64 exactly."""
    cfg: Config
    Q: np.ndarray
    K: np.ndarray
    V: np.ndarray
    lengths: Optional[np.ndarray]      # int32 [B] or None (all rows valid)
    sample_idx: np.ndarray             # int32 [B,H,L,U]
    seed: int

    def as_f64(self, name: str) -> np.ndarray:
        a = getattr(self, name)
        if self.cfg.dtype == "bf16":
            a = bf16_bits_to_f32(a)
        return a.astype(np.float64)

    @property
    def shape(self):
        c = self.cfg
        return (c.B, c.H, c.L, D_HEAD)

    def lengths_or_full(self) -> np.ndarray:
        if self.lengths is None:
            return np.full(self.cfg.B, self.cfg.L, dtype=np.int32)
        return self.lengths


# ----------------------------------------------------------------------------
# value distributions
# ----------------------------------------------------------------------------
def _draw_normal(rng, B, H, L):
    K = rng.standard_normal((B, H, L, D_HEAD), dtype=np.float32)
    V = rng.standard_normal((B, H, L, D_HEAD), dtype=np.float32)
    Q = rng.standard_normal((B, H, L, D_HEAD), dtype=np.float32)
    return Q, K, V


def _draw_peaky(rng, B, H, L, lengths):
    """K, V, Q i.i.d. N(0,1); then per (b,h) round(0.1*len_b) query rows, chosen
    without replacement among the valid rows, are overwritten by 4x a randomly
    chosen valid key row plus N(0, sigma=0.1) noise, so that a few queries have
    a sharply peaked score distribution."""
    Q, K, V = _draw_normal(rng, B, H, L)
    for b in range(B):
        n = int(lengths[b])
        n_peaky = int(round(0.1 * n))
        for h in range(H):
            rows = rng.choice(n, size=n_peaky, replace=False)
            keys = rng.integers(0, n, size=n_peaky)
            noise = rng.standard_normal((n_peaky, D_HEAD), dtype=np.float32) * np.float32(0.1)
            Q[b, h, rows, :] = np.float32(4.0) * K[b, h, keys, :] + noise
    return Q, K, V


def _draw_mixture(rng, B, H, L, n_comp=32, centre_scale=2.0, sigma=0.5):
    """32-component Gaussian mixture: one set of centres 2*N(0,I) per draw,
    shared by Q, K, V and by all (b,h); frame i of a head picks one component,
    shared by row i of Q, K and V (all three derive from the same frame in
    self-attention); row = centre + N(0, sigma=0.5) with independent noise."""
    centres = (rng.standard_normal((n_comp, D_HEAD), dtype=np.float32) * np.float32(centre_scale))
    z = rng.integers(0, n_comp, size=(B, H, L))
    out = []
    for _ in range(3):  # K, V, Q in that order
        noise = rng.standard_normal((B, H, L, D_HEAD), dtype=np.float32) * np.float32(sigma)
        out.append(centres[z] + noise)
    K, V, Q = out
    return Q, K, V


def _draw_sample_idx(rng, B, H, L, U, lengths):
    idx = np.zeros((B, H, L, U), dtype=np.int32)
    for b in range(B):
        n = int(lengths[b])
        idx[b, :, :n, :] = rng.integers(0, n, size=(H, n, U), dtype=np.int32)
    return idx


def make_workload(cfg: Config, seed: Optional[int] = None, pad_value: float = 0.0) -> Workload:
    """Draw one batch for `cfg`.  Draw order: lengths, K/V/Q, sample_idx.
    Rows at or beyond a batch item's length are set to `pad_value` (tests also
    use NaN there, which a correct implementation must never let through)."""
    if seed is None:
        seed = BASE_SEED + cfg.seed_offset
    rng = np.random.Generator(np.random.PCG64(seed))
    B, H, L, U = cfg.B, cfg.H, cfg.L, cfg.U
    if cfg.ragged:
        lengths = rng.integers(cfg.len_lo, cfg.len_hi + 1, size=B).astype(np.int32)
    else:
        lengths = np.full(B, L, dtype=np.int32)
    if cfg.values == "normal":
        Q, K, V = _draw_normal(rng, B, H, L)
    elif cfg.values == "peaky":
        Q, K, V = _draw_peaky(rng, B, H, L, lengths)
    elif cfg.values == "mixture":
        Q, K, V = _draw_mixture(rng, B, H, L)
    else:
        raise ValueError(cfg.values)
    idx = _draw_sample_idx(rng, B, H, L, U, lengths)
    if cfg.ragged:
        for b in range(B):
            n = int(lengths[b])
            for a in (Q, K, V):
                a[b, :, n:, :] = pad_value
    if cfg.dtype == "bf16":
        Q, K, V = (f32_to_bf16_bits(a) for a in (Q, K, V))
    elif cfg.dtype != "f32":
        raise ValueError(cfg.dtype)
    return Workload(cfg, np.ascontiguousarray(Q), np.ascontiguousarray(K), np.ascontiguousarray(V),
                    lengths if cfg.ragged else None, idx, seed)


def small_config(name: str, B: int, H: int, L: int, U: int, c: float, dtype: str = "f32",
                 values: str = "normal", ragged: bool = False, len_lo: int = 0, len_hi: int = 0,
                 seed_offset: int = 0) -> Config:
    """A custom-sized config for tests (same distributions as the named ones)."""
    return Config(name, B, H, L, U, c, dtype, values, ragged, len_lo, len_hi, seed_offset)


def make_mhsa_inputs(B: int, L: int, H: int, dtype: str = "f32", seed: int = 0, bias: bool = True):
    """Seeded inputs for the whole multi-head module: X [B, L, H*64] ~ N(0, 1), four
    matrices [H*64, H*64] ~ N(0, 1/d_model) stored [d_out, d_in], four bias vectors
    ~ N(0, 0.1) (or None).  Arrays are float32, or bfloat16 bit patterns (uint16)
    for dtype "bf16"; `as_f64` of each is what both the oracle and the device see."""
    r = np.random.Generator(np.random.PCG64(seed))
    dm = H * 64
    out = {"X": r.standard_normal((B, L, dm)).astype(np.float32)}
    for name in ("Wq", "Wk", "Wv", "Wo"):
        out[name] = (r.standard_normal((dm, dm)) / np.sqrt(dm)).astype(np.float32)
    for name in ("bq", "bk", "bv", "bo"):
        out[name] = (0.1 * r.standard_normal(dm)).astype(np.float32) if bias else None
    if dtype == "bf16":
        out = {k: (None if v is None else f32_to_bf16_bits(v)) for k, v in out.items()}
    return out


def make_upstream_gradient(cfg: Config, seed: int, pad_value: float = 0.0, lengths=None):
    """Seeded N(0, 1) gradient of a loss with respect to the attention output, [B, H, L, d] in the
    workload's storage type (float32, or bfloat16 bit patterns); rows at or beyond an item's length
    are set to `pad_value`."""
    r = np.random.Generator(np.random.PCG64(seed))
    G = r.standard_normal((cfg.B, cfg.H, cfg.L, D_HEAD), dtype=np.float32)
    if lengths is not None:
        for b in range(cfg.B):
            G[b, :, int(lengths[b]):, :] = pad_value
    return f32_to_bf16_bits(G) if cfg.dtype == "bf16" else G


def to_f64(a, dtype: str):
    """float64 view of an array made by the generators above (None passes through)."""
    if a is None:
        return None
    return bf16_bits_to_f32(a).astype(np.float64) if dtype == "bf16" else a.astype(np.float64)
