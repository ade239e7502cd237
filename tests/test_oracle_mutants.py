"""Plant plausible mistakes in a copy of the oracle (on the CPU) and require
that the pins catch each one: a dropped term, a wrong sign, a wrong index, a
transposed operand, a wrong denominator."""
import importlib.util
import os
import sys
import types

import pytest

from tests import oracle_pins

SRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle", "probsparse_oracle.py")

# (name, text in the oracle source, replacement)
MUTANTS = [
    ("measure_drops_mean", "M[i] = s.max() - s.sum() / j.size", "M[i] = s.max()"),
    ("measure_plus_mean", "M[i] = s.max() - s.sum() / j.size", "M[i] = s.max() + s.sum() / j.size"),
    ("measure_min_for_max", "M[i] = s.max() - s.sum() / j.size", "M[i] = s.min() - s.sum() / j.size"),
    ("measure_mean_over_n", "M[i] = s.max() - s.sum() / j.size", "M[i] = s.max() - s.sum() / n"),
    ("measure_no_scale", "s = (K[j] @ Q[i]) / math.sqrt(d)          # step 1", "s = (K[j] @ Q[i])  # step 1"),
    ("measure_scale_d", "s = (K[j] @ Q[i]) / math.sqrt(d)          # step 1", "s = (K[j] @ Q[i]) / d  # step 1"),
    ("measure_unique_samples", "j = j[(j >= 0) & (j < n)]", "j = np.unique(j[(j >= 0) & (j < n)])"),
    ("measure_keeps_masked", "j = j[(j >= 0) & (j < n)]", "j = j[(j >= 0)] % len(K)"),
    ("select_smallest", "key=lambda i: (-M[i], i)", "key=lambda i: (M[i], i)"),
    ("select_ties_high", "key=lambda i: (-M[i], i)", "key=lambda i: (-M[i], -i)"),
    ("u_floor", "x = math.ceil(c * math.log(n))", "x = math.floor(c * math.log(n))"),
    ("u_log2", "x = math.ceil(c * math.log(n))", "x = math.ceil(c * math.log2(n))"),
    ("u_no_clamp_low", "x = math.ceil(c * math.log(n))\n    return int(min(n, max(1, x)))",
     "x = math.ceil(c * math.log(n))\n    return int(min(n, x))"),
    ("attn_no_scale", "a = (Qrows @ K.T) / math.sqrt(d)              # [r, n]", "a = (Qrows @ K.T)"),
    ("attn_no_normalise", "p = p / p.sum(axis=1, keepdims=True)          # Eq. 7", "pass"),
    ("attn_normalise_cols", "p = p / p.sum(axis=1, keepdims=True)          # Eq. 7", "p = p / p.sum(axis=0, keepdims=True)"),
    ("attn_uses_k_for_v", "return p @ V                                  # Eq. 8", "return p @ K"),
    ("fill_sum_not_mean", "out[:n] = Vv.sum(axis=0) / n", "out[:n] = Vv.sum(axis=0)"),
    ("fill_mean_over_L", "out[:n] = Vv.sum(axis=0) / n", "out[:n] = V.sum(axis=0) / L"),
    ("fill_skipped", "out[I] = attention_rows(Qv[I], Kv, Vv)                     # step 4", "pass"),
    ("attend_wrong_rows", "out[I] = attention_rows(Qv[I], Kv, Vv)                     # step 4",
     "out[I] = attention_rows(Qv[np.sort(I)], Kv, Vv)"),
    ("attend_padded_keys", "out[I] = attention_rows(Qv[I], Kv, Vv)                     # step 4",
     "out[I] = attention_rows(Qv[I], np.nan_to_num(K), np.nan_to_num(V))"),
    ("ratio_floor", "x = math.ceil(r_sparse * n)", "x = math.floor(r_sparse * n)"),
    ("ratio_no_clamp", "x = math.ceil(r_sparse * n)\n    return int(min(n, max(1, x)))",
     "x = math.ceil(r_sparse * n)\n    return int(max(1, x))"),
    ("ratio_of_L", "n_select = n_selected_ratio(r_sparse, n)", "n_select = n_selected_ratio(r_sparse, L)"),
    ("given_fill_over_L", "out[b, h, :n] = Vv.sum(axis=0) / n", "out[b, h, :n] = Vv.sum(axis=0) / L"),
    ("given_value_is_mean", "out[b, h, :n] = Vv\n", "out[b, h, :n] = Vv.mean(axis=0)\n"),
    ("given_padded_keys", "out[b, h, I] = attention_rows(Q[b, h, I], K[b, h, :n], Vv)",
     "out[b, h, I] = attention_rows(Q[b, h, I], K[b, h], V[b, h])"),
    ("proj_no_transpose", "Y = X @ np.asarray(W, dtype=np.float64).T\n", "Y = X @ np.asarray(W, dtype=np.float64)\n"),
    ("proj_heads_interleaved", "return Y.reshape(B, L, H, dm // H).transpose(0, 2, 1, 3)",
     "return Y.reshape(B, L, dm // H, H).transpose(0, 3, 1, 2)"),
    ("merge_heads_wrong_axis", "Y = A.transpose(0, 2, 1, 3).reshape(B, L, H * d) @",
     "Y = A.transpose(0, 2, 3, 1).reshape(B, L, H * d) @"),
    ("out_bias_dropped", "        Y = Y + np.asarray(bo, dtype=np.float64)", "        pass"),
    ("bf16_truncates", "b = (b + 0x7FFF + ((b >> 16) & 1)) & 0xFFFF0000", "b = b & 0xFFFF0000"),
    ("exact_measure_no_mean", "return lse - s.sum(axis=1) / n", "return lse"),
    ("kl_plus_const", "return exact_measure(Q, K, n) - math.log(n)", "return exact_measure(Q, K, n) + math.log(n)"),
    ("bwd_no_softmax_term", "g = p * (c - (p * c).sum(axis=1, keepdims=True))", "g = p * c"),
    ("bwd_softmax_term_unweighted", "g = p * (c - (p * c).sum(axis=1, keepdims=True))",
     "g = p * (c - c.mean(axis=1, keepdims=True))"),
    ("bwd_dq_no_scale", "dQrows = (g @ K) / math.sqrt(d)", "dQrows = (g @ K)"),
    ("bwd_dk_no_scale", "dK = (g.T @ Qrows) / math.sqrt(d)", "dK = (g.T @ Qrows)"),
    ("bwd_dk_uses_k", "dK = (g.T @ Qrows) / math.sqrt(d)", "dK = (g.T @ (g @ K)) / math.sqrt(d)"),
    ("bwd_dv_unweighted", "dV = p.T @ Grows", "dV = np.ones_like(p).T @ Grows / p.shape[1]"),
    ("bwd_c_uses_k", "c = Grows @ V.T                               # [r, n]", "c = Grows @ K.T  # [r, n]"),
    ("bwd_mean_fill_over_L", "dV[b, h, :n] += G[b, h, :n][rest].sum(axis=0) / n  # every valid",
     "dV[b, h, :n] += G[b, h, :n][rest].sum(axis=0) / L  # every valid"),
    ("bwd_mean_fill_all_rows", "dV[b, h, :n] += G[b, h, :n][rest].sum(axis=0) / n  # every valid",
     "dV[b, h, :n] += G[b, h, :n].sum(axis=0) / n  # every valid"),
    ("bwd_value_fill_all_rows", "dV[b, h, :n][rest] += G[b, h, :n][rest]", "dV[b, h, :n] += G[b, h, :n]"),
    ("bwd_dk_overwrites", "dK[b, h, :n] += dk", "dK[b, h, :n] = -dk"),
    ("bwd_padded_keys", "dq, dk, dv = attention_rows_backward(Q[b, h, I], K[b, h, :n], V[b, h, :n], G[b, h, I])",
     "dq, dk, dv = attention_rows_backward(Q[b, h, I], K[b, h], V[b, h], G[b, h, I]); dk, dv = dk[:n], dv[:n]"),
]


def _load_mutant(name, old, new):
    src = open(SRC).read()
    assert src.count(old) == 1, f"mutant {name}: pattern must occur exactly once"
    mod = types.ModuleType("oracle_mutant_" + name)
    mod.__file__ = SRC
    sys.modules[mod.__name__] = mod      # dataclasses / typing need this
    exec(compile(src.replace(old, new), SRC, "exec"), mod.__dict__)
    return mod


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_pins_catch_mutant(name, old, new):
    mod = _load_mutant(name, old, new)
    caught = []
    for check in oracle_pins.ALL_CHECKS:
        try:
            check(mod)
        except AssertionError:
            caught.append(check.__name__)
        except Exception:
            caught.append(check.__name__)
    assert caught, f"no pin notices mutant {name}"
