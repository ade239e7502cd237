"""Parity rules between the HIP path and the CPU oracle (used by the GPU tests,
the smoke check and the benchmark's self-check).

Selection (a2): the index sets must be equal, except that queries whose oracle
measure lies within SEL_TOL * max(1, |M_cut|) of the cut-off M_cut (the u-th
largest oracle measure) may be swapped one for one: the GPU computes the
measure in float32, the oracle in float64, and a hard threshold turns a
rounding difference into a different index.

Outputs (a3, a4): max over elements of |gpu - oracle| / max(|oracle|, tau),
tau = 1e-2 * RMS(oracle over valid rows), at most 1e-4 for float32 and 2e-2 for
bfloat16 storage.  Rows whose selected/unselected status legitimately differs
under the rule above are left out of the output comparison.
"""
from __future__ import annotations

import numpy as np

SEL_TOL = 1e-5
OUT_TOL = {"f32": 1e-4, "bf16": 2e-2}
M_TOL = {"f32": 2e-5, "bf16": 2e-5}     # |M_gpu - M_oracle| <= M_TOL * max(1, |M_oracle|)


def compare_selection(M_oracle_head, sel_oracle, sel_gpu):
    """Returns (ok, disputed_indices).  M_oracle_head: [n] float64 for one head."""
    so, sg = set(int(i) for i in sel_oracle), set(int(i) for i in sel_gpu)
    if len(sg) != len(sel_gpu) or len(so) != len(sg):
        return False, sorted(so ^ sg)
    if so == sg:
        return True, []
    cut = min(M_oracle_head[i] for i in so)
    tol = SEL_TOL * max(1.0, abs(cut))
    diff = so ^ sg
    ok = all(abs(M_oracle_head[i] - cut) <= tol for i in diff)
    return ok, sorted(diff)


def output_error(out_gpu, out_oracle, valid_mask=None):
    """max |g - o| / max(|o|, tau) with tau = 1e-2 RMS(o) over the compared rows."""
    g = np.asarray(out_gpu, dtype=np.float64)
    o = np.asarray(out_oracle, dtype=np.float64)
    if valid_mask is not None:
        g, o = g[valid_mask], o[valid_mask]
    if o.size == 0:
        return 0.0
    tau = 1e-2 * float(np.sqrt(np.mean(o * o)))
    if tau == 0.0:
        tau = 1e-30
    return float(np.max(np.abs(g - o) / np.maximum(np.abs(o), tau)))
