#!/usr/bin/env python3
"""Writes tests/golden/oracle_small_case.json from the CPU oracle alone.

    python tests/golden/make_golden.py

The file freezes what the oracle computes on one small seeded input, so that a
later change to the oracle's arithmetic shows up as a diff of this file (and
has to be justified against the paper).  Nothing here touches the GPU path.
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import probsparse_oracle as O                      # noqa: E402
from paper_2106_09236_amd import workloads as W                # noqa: E402  (seeded inputs only)


def small_case():
    cfg = W.small_config("golden", 2, 2, 24, 5, 2.0, "f32", "peaky", True, 9, 24)
    return cfg, W.make_workload(cfg, seed=20210609)


def main():
    cfg, w = small_case()
    out, M, sel, u = O.probsparse_attn_fwd(w.as_f64("Q"), w.as_f64("K"), w.as_f64("V"), w.lengths, w.sample_idx, cfg.c)
    out_r, _, sel_r, u_r = O.probsparse_attn_fwd(w.as_f64("Q"), w.as_f64("K"), w.as_f64("V"), w.lengths, w.sample_idx,
                                                 cfg.c, fill="value", r_sparse=0.5)
    doc = {
        "what": "CPU oracle on small_config('golden', B=2, H=2, L=24, U=5, c=2, f32, peaky, ragged 9..24), seed 20210609",
        "cites": "Sec. 3.2 Eq. 11 (M), text after Eq. 11 (I_sparse), Eq. 7/8/12 (rows), Sec. 3.1 (mean fill); "
                 "second block: L_sparse = r_sparse * L with r_sparse = 0.5 and Eq. 12's v_i",
        "lengths": w.lengths.tolist(),
        "u": u.tolist(),
        "sel": [[s.tolist() for s in row] for row in sel],
        "M": [[[None if np.isnan(x) else float(x) for x in M[b, h]] for h in range(cfg.H)] for b in range(cfg.B)],
        "out_row_sums": out.sum(axis=-1).tolist(),
        "out_first_selected_row": out[0, 0, sel[0][0][0]].tolist(),
        "ratio_u": u_r.tolist(),
        "ratio_sel": [[s.tolist() for s in row] for row in sel_r],
        "ratio_out_row_sums": out_r.sum(axis=-1).tolist(),
    }
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_small_case.json")
    with open(path, "w") as f:
        json.dump(doc, f, indent=1)
    print("wrote", path)


if __name__ == "__main__":
    main()
