"""The oracle against stored values: a closed-form case worked out by hand from the
paper's formulas, and a frozen copy of its own output on one small seeded input."""
import json
import math
import os

import numpy as np

from oracle import probsparse_oracle as O

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def test_closed_form_case():
    g = json.load(open(os.path.join(GOLDEN, "closed_form_case.json")))
    # the stored numbers are what the formulas give
    assert abs(g["sampled_measure_value"] - math.log(2)) < 1e-15
    assert abs(g["exact_measure_value"] - (math.log(7) - math.log(2))) < 1e-15
    assert abs(g["kl_measure_value"] - (math.log(7) - math.log(2) - math.log(3))) < 1e-15
    assert np.allclose(g["softmax"], [1 / 7, 2 / 7, 4 / 7], atol=1e-16)
    d, L = 64, 3
    K = np.zeros((L, d)); K[:, 0] = [0.0, 8 * math.log(2), 8 * math.log(4)]
    Q = np.zeros((L, d)); Q[:, 0] = 1.0
    V = np.arange(L, dtype=np.float64)[:, None] * np.ones((L, d))
    idx = np.tile(np.arange(L, dtype=np.int32), (L, 1))
    M = O.sampled_measure(Q, K, idx, L)
    assert np.allclose(M, g["sampled_measure_value"], atol=1e-14)
    assert np.allclose(O.exact_measure(Q, K, L), g["exact_measure_value"], atol=1e-14)
    assert np.allclose(O.kl_measure(Q, K, L), g["kl_measure_value"], atol=1e-14)
    rows = O.attention_rows(Q, K, V)
    assert np.allclose(rows, g["attention_row_every_element"], atol=1e-14)
    # the whole step list: u = 1 keeps query 0 (all measures tie), the others receive the mean of V
    out, _, I = O.probsparse_head(Q, K, V, idx, L, c=0.5)
    assert I.tolist() == [0]
    assert np.allclose(out[0], g["attention_row_every_element"], atol=1e-14)
    assert np.allclose(out[1:], g["mean_of_values_every_element"], atol=1e-14)


def test_frozen_small_case():
    import importlib.util
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(GOLDEN, "make_golden.py"))
    mg = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mg)
    cfg, w = mg.small_case()
    g = json.load(open(os.path.join(GOLDEN, "oracle_small_case.json")))
    out, M, sel, u = O.probsparse_attn_fwd(w.as_f64("Q"), w.as_f64("K"), w.as_f64("V"), w.lengths, w.sample_idx, cfg.c)
    assert w.lengths.tolist() == g["lengths"]
    assert u.tolist() == g["u"]
    assert [[s.tolist() for s in row] for row in sel] == g["sel"]
    Mg = np.array([[[np.nan if x is None else x for x in h] for h in b] for b in g["M"]])
    assert np.allclose(M, Mg, atol=1e-12, equal_nan=True)
    assert np.allclose(out.sum(axis=-1), np.array(g["out_row_sums"]), atol=1e-10)
    assert np.allclose(out[0, 0, sel[0][0][0]], np.array(g["out_first_selected_row"]), atol=1e-12)
    out_r, _, sel_r, u_r = O.probsparse_attn_fwd(w.as_f64("Q"), w.as_f64("K"), w.as_f64("V"), w.lengths, w.sample_idx,
                                                 cfg.c, fill="value", r_sparse=0.5)
    assert u_r.tolist() == g["ratio_u"]
    assert [[s.tolist() for s in row] for row in sel_r] == g["ratio_sel"]
    assert np.allclose(out_r.sum(axis=-1), np.array(g["ratio_out_row_sums"]), atol=1e-10)
