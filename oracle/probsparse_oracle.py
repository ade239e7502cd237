"""CPU oracle for the prob-sparse self-attention forward (arXiv 2106.09236).

TEST INFRASTRUCTURE ONLY.  This file is a slow, plain float64 NumPy statement
of what the method computes, written from the paper.  Only the test-suite, the
smoke check and the benchmark's `cpu_baseline` leg may import it; the product
(the HIP library and its Python binding) never does, and this file imports
nothing from the product.  It shares no code, table or constant with the GPU
path.

The method is a heuristic (a sampled measure followed by a hard selection), so
the oracle is the algorithm taken step by step in the paper's order:

  1. scores of every query against its sampled keys      (Sec. 3.2, Eq. 11)
  2. sampled sparsity measure  M = max - mean             (Sec. 3.2, Eq. 11)
  3. the u queries with the largest measure -> I_sparse   (Sec. 3.2, text after Eq. 11)
  4. softmax attention for the queries in I_sparse        (Eq. 7, Eq. 8, Eq. 12 upper branch)
  5. fill for all other queries                           (Sec. 3.1 uniform-score argument)

Readings taken where the paper is silent or where the benchmark's problem
statement departs from it (each is listed again in the design notes):

  * u = ceil(c * ln n), clamped to [1, n], with n the valid length of the batch
    item: the rule of the Informer work the paper builds on (Sec. 1, Sec. 3.2),
    used by the benchmark instead of L_sparse = r_sparse * L.  An explicit-u
    variant (`n_select=`) covers the paper's own r_sparse * L.
  * fill = mean of the valid value rows.  Eq. 12's lower branch prints v_i;
    Sec. 3.1 argues that a query with uniform scores yields the plain average
    of all values, which is what the benchmark specifies.  `fill="value"`
    gives Eq. 12 as printed.
  * the sampled keys are given per query (a shared sampled key matrix is the
    special case of identical rows); duplicates count with multiplicity in the
    mean; the mean divides by the number of samples actually used (Eq. 11's
    1 / L-tilde).
  * padding: key j and query i of batch item b are valid iff j, i < lengths[b];
    invalid keys are left out of steps 1, 2, 4 and 5, invalid queries are never
    selected and their output rows are zero.  A sample index outside [0, n) is
    dropped; a query with no usable sample gets measure 0.
  * ties in step 3 go to the lower query index.
  * Eq. 7 is typeset with the 1/sqrt(d) outside the exponent; Eq. 6 and Eq. 9
    fix the intended exp(q.k / sqrt(d)).

The projections around the path (`project_heads`, `merge_heads`, `mhsa_forward`:
Sec. 3.1, Sec. 2.2) are plain matrix products, pinned against the library's
multi-head attention in the all-queries-kept limit.

The two variants the paper itself describes are here as well: the number of
kept queries as r_sparse * n (`n_selected_ratio`, `r_sparse=`) with Eq. 12's
v_i fill (`fill="value"`), and steps 4-5 for given index sets
(`attention_with_indices`, Sec. 4.4), and the gradients of steps 4 and 5 for a
fixed index set (`attention_with_indices_backward`; retraining from a trained
dense model, Sec. 4.2).

Pins (tests/test_oracle_pins.py): u = L_Q reproduces textbook dense attention
(library SDPA and a hand loop); M >= 0 and M = 0 for constant scores; the
sandwich M_sampled <= M_exact <= M_sampled + ln L when every key is sampled
once; Eq. 9 against a library KL divergence; brute-force selection on tiny
inputs; mean(V) rows; one-hot limit; masking and permutation invariances; the
gradients against the library's automatic differentiation in float64 and
against central differences of the forward.
"""
from __future__ import annotations

import math
from typing import List, Optional, Tuple

import numpy as np


# ----------------------------------------------------------------------------
# Step 3 helper: how many queries are kept
# ----------------------------------------------------------------------------
def n_selected(c: float, n: int) -> int:
    """u = ceil(c ln n) clamped to [1, n]  (Sec. 3.2 with the Informer rule;
    ln 1 = 0 would select nothing, hence the lower clamp).  n = 0 selects 0."""
    if n <= 0:
        return 0
    x = math.ceil(c * math.log(n))
    return int(min(n, max(1, x)))


def n_selected_ratio(r_sparse: float, n: int) -> int:
    """u = L_sparse = r_sparse * n  (Sec. 3.2, "L_sparse = r_sparse x L"; the
    experiments use r_sparse = 0.5, Sec. 4.2), rounded up when it is not an
    integer and clamped to [1, n].  n = 0 selects 0."""
    if n <= 0:
        return 0
    x = math.ceil(r_sparse * n)
    return int(min(n, max(1, x)))


# ----------------------------------------------------------------------------
# Steps 1 + 2: sampled scores and sampled sparsity measure (Eq. 11)
# ----------------------------------------------------------------------------
def sampled_measure(Q: np.ndarray, K: np.ndarray, sample_idx: np.ndarray, n: int) -> np.ndarray:
    """M-bar for the n valid queries of one head.

    Q, K: [L, d] float64; sample_idx: [L, U] int; returns [n] float64.
    For query i:  s_t = q_i . k_{j_t} / sqrt(d) over its usable samples j_t,
    M_i = max_t s_t - (1 / #usable) sum_t s_t                      (Eq. 11)
    """
    d = Q.shape[1]
    M = np.zeros(n, dtype=np.float64)
    for i in range(n):
        j = sample_idx[i]
        j = j[(j >= 0) & (j < n)]                 # drop masked / out-of-range samples
        if j.size == 0:
            M[i] = 0.0
            continue
        s = (K[j] @ Q[i]) / math.sqrt(d)          # step 1: scores on the samples
        M[i] = s.max() - s.sum() / j.size         # step 2: max - mean
    return M


# ----------------------------------------------------------------------------
# Step 3: top-u selection
# ----------------------------------------------------------------------------
def select_top_u(M: np.ndarray, u: int) -> np.ndarray:
    """Indices of the u largest entries of M, ties to the lower index, returned
    in order of decreasing M (then increasing index)."""
    order = sorted(range(len(M)), key=lambda i: (-M[i], i))
    return np.asarray(order[:u], dtype=np.int64)


# ----------------------------------------------------------------------------
# Step 4: softmax attention of given query rows over the valid keys (Eq. 7-8)
# ----------------------------------------------------------------------------
def attention_rows(Qrows: np.ndarray, K: np.ndarray, V: np.ndarray) -> np.ndarray:
    """SA(q_i) = sum_j p(k_j | q_i) v_j with p = softmax_j(q_i . k_j / sqrt(d))."""
    d = K.shape[1]
    a = (Qrows @ K.T) / math.sqrt(d)              # [r, n]
    a = a - a.max(axis=1, keepdims=True)          # max-subtraction, value unchanged
    p = np.exp(a)
    p = p / p.sum(axis=1, keepdims=True)          # Eq. 7
    return p @ V                                  # Eq. 8


# ----------------------------------------------------------------------------
# One head, all five steps
# ----------------------------------------------------------------------------
def probsparse_head(Q: np.ndarray, K: np.ndarray, V: np.ndarray, sample_idx: np.ndarray,
                    n: int, c: float, n_select: Optional[int] = None,
                    fill: str = "mean") -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Returns (out [L, d], M [n], I_sparse [u]) for one (batch, head)."""
    L, d = Q.shape
    out = np.zeros((L, d), dtype=np.float64)      # rows >= n stay zero
    if n <= 0:
        return out, np.zeros(0), np.zeros(0, dtype=np.int64)
    Qv, Kv, Vv = Q[:n], K[:n], V[:n]
    M = sampled_measure(Qv, Kv, sample_idx[:n], n)                 # steps 1, 2
    u = n_selected(c, n) if n_select is None else int(min(n, max(0, n_select)))
    I = select_top_u(M, u)                                         # step 3
    if fill == "mean":                                             # step 5
        out[:n] = Vv.sum(axis=0) / n
    elif fill == "value":                                          # Eq. 12 as printed
        out[:n] = Vv
    else:
        raise ValueError(fill)
    if u > 0:
        out[I] = attention_rows(Qv[I], Kv, Vv)                     # step 4
    return out, M, I


def probsparse_attn_fwd(Q: np.ndarray, K: np.ndarray, V: np.ndarray,
                        lengths: Optional[np.ndarray], sample_idx: np.ndarray, c: float,
                        n_select: Optional[int] = None, fill: str = "mean",
                        r_sparse: Optional[float] = None):
    """Whole batch.  Q, K, V: [B, H, L, d]; lengths: [B] or None; sample_idx
    [B, H, L, U].  Returns (out [B,H,L,d] f64, M [B,H,L] f64 with NaN on
    padded queries, sel: list over (b,h) of index arrays, u [B]).
    `r_sparse` switches the number of kept queries of item b from
    n_selected(c, len_b) to the paper's own n_selected_ratio(r_sparse, len_b)."""
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    B, H, L, d = Q.shape
    out = np.zeros((B, H, L, d), dtype=np.float64)
    Mall = np.full((B, H, L), np.nan, dtype=np.float64)
    sel: List[List[np.ndarray]] = []
    u_of_b = np.zeros(B, dtype=np.int64)
    for b in range(B):
        n = L if lengths is None else int(lengths[b])
        row = []
        if r_sparse is not None:
            n_select = n_selected_ratio(r_sparse, n)
        for h in range(H):
            o, M, I = probsparse_head(Q[b, h], K[b, h], V[b, h], sample_idx[b, h], n, c, n_select, fill)
            out[b, h] = o
            Mall[b, h, :n] = M
            row.append(I)
            u_of_b[b] = len(I)
        sel.append(row)
    return out, Mall, sel, u_of_b


def attention_with_indices(Q: np.ndarray, K: np.ndarray, V: np.ndarray,
                           lengths: Optional[np.ndarray], sel, fill: str = "mean") -> np.ndarray:
    """Steps 4 and 5 alone, for index sets that are given (Sec. 4.4: the index
    set of one layer is reused by the layers that follow it, so they skip
    steps 1 to 3).  sel[b][h] holds the kept queries of (b, h); every entry
    must be a valid query of the item.  Returns out [B, H, L, d] float64."""
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    B, H, L, d = Q.shape
    out = np.zeros((B, H, L, d), dtype=np.float64)
    for b in range(B):
        n = L if lengths is None else int(lengths[b])
        if n <= 0:
            continue
        for h in range(H):
            Vv = V[b, h, :n]
            if fill == "mean":
                out[b, h, :n] = Vv.sum(axis=0) / n
            elif fill == "value":
                out[b, h, :n] = Vv
            else:
                raise ValueError(fill)
            I = np.asarray(sel[b][h], dtype=np.int64)
            if I.size:
                assert I.min() >= 0 and I.max() < n
                out[b, h, I] = attention_rows(Q[b, h, I], K[b, h, :n], Vv)
    return out


# ----------------------------------------------------------------------------
# Gradients of steps 4 and 5 for a fixed index set (retraining a prob-sparse
# model from a trained dense one, Sec. 4.2, needs them).  I_sparse is a hard
# choice, so no gradient flows through steps 1 to 3: with the set held fixed the
# output is, per head,
#   out_i = sum_j p_ij v_j,  p_i = softmax_j(q_i . k_j / sqrt(d))   for i in I_sparse   (Eq. 7, 8, 12)
#   out_i = (1/n) sum_j v_j  (or v_i with fill="value")            for the other valid i
#   out_i = 0                                                       for i >= n
# and the chain rule gives, for an upstream gradient G = dLoss/dout:
#   i in I_sparse:   c_ij  = G_i . v_j                    (gradient w.r.t. p_ij)
#                    g_ij  = p_ij (c_ij - sum_j' p_ij' c_ij')   (through the softmax, w.r.t. the scaled score)
#                    dQ_i  = (1/sqrt(d)) sum_j g_ij k_j
#                    dK_j += (1/sqrt(d)) g_ij q_i
#                    dV_j += p_ij G_i
#   other valid i:   mean fill:  dV_j += G_i / n for every valid j;   value fill:  dV_i += G_i
# ----------------------------------------------------------------------------
def attention_rows_backward(Qrows: np.ndarray, K: np.ndarray, V: np.ndarray, Grows: np.ndarray):
    """Gradients of attention_rows(Qrows, K, V) for the upstream gradient Grows
    [r, d]: returns (dQrows [r, d], dK [n, d], dV [n, d])."""
    d = K.shape[1]
    a = (Qrows @ K.T) / math.sqrt(d)
    a = a - a.max(axis=1, keepdims=True)
    p = np.exp(a)
    p = p / p.sum(axis=1, keepdims=True)          # the weights of Eq. 7 again
    c = Grows @ V.T                               # [r, n]: d out_i / d p_ij contracted with G_i
    g = p * (c - (p * c).sum(axis=1, keepdims=True))
    dQrows = (g @ K) / math.sqrt(d)
    dK = (g.T @ Qrows) / math.sqrt(d)
    dV = p.T @ Grows
    return dQrows, dK, dV


def attention_with_indices_backward(Q: np.ndarray, K: np.ndarray, V: np.ndarray,
                                    lengths: Optional[np.ndarray], sel, G: np.ndarray, fill: str = "mean"):
    """Gradients of attention_with_indices(Q, K, V, lengths, sel, fill) for the
    upstream gradient G [B, H, L, d].  Returns (dQ, dK, dV), each [B, H, L, d]
    float64; rows at or beyond an item's length are zero, and so are the rows of
    dQ of the queries outside I_sparse."""
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    G = np.asarray(G, dtype=np.float64)
    B, H, L, d = Q.shape
    dQ, dK, dV = np.zeros_like(Q), np.zeros_like(Q), np.zeros_like(Q)
    for b in range(B):
        n = L if lengths is None else int(lengths[b])
        if n <= 0:
            continue
        for h in range(H):
            I = np.asarray(sel[b][h], dtype=np.int64)
            rest = np.ones(n, dtype=bool)
            rest[I] = False                                        # valid queries outside I_sparse
            if fill == "mean":
                dV[b, h, :n] += G[b, h, :n][rest].sum(axis=0) / n  # every valid v_j holds 1/n of each filled row
            elif fill == "value":
                dV[b, h, :n][rest] += G[b, h, :n][rest]
            else:
                raise ValueError(fill)
            if I.size:
                dq, dk, dv = attention_rows_backward(Q[b, h, I], K[b, h, :n], V[b, h, :n], G[b, h, I])
                dQ[b, h, I] = dq
                dK[b, h, :n] += dk
                dV[b, h, :n] += dv
    return dQ, dK, dV


# ----------------------------------------------------------------------------
# The multi-head module around the path (Sec. 3.1: Q = X W_q, K = X W_k,
# V = X W_v; Sec. 2.2, Eq. 5: the MHSA module of the Conformer block; Sec. 4.2:
# 4 heads of 64 dimensions)
# ----------------------------------------------------------------------------
def round_to(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round float64 values to the storage type of a tensor and return them as
    float64: "f32" = IEEE binary32, "bf16" = bfloat16 (round to nearest even on
    the upper 16 bits of binary32), "f64" = unchanged."""
    if dtype == "f64":
        return np.asarray(x, dtype=np.float64)
    f = np.asarray(x, dtype=np.float32)
    if dtype == "f32":
        return f.astype(np.float64)
    if dtype != "bf16":
        raise ValueError(dtype)
    b = f.view(np.uint32).astype(np.uint64)
    b = (b + 0x7FFF + ((b >> 16) & 1)) & 0xFFFF0000
    out = b.astype(np.uint32).view(np.float32).astype(np.float64)
    return np.where(np.isnan(f), np.nan, out)


def project_heads(X: np.ndarray, W: np.ndarray, bias: Optional[np.ndarray], H: int) -> np.ndarray:
    """X [B, L, d_model] times one projection matrix, cut into heads:
    out[b, h, l, e] = sum_k X[b, l, k] W[h*d + e, k] (+ bias[h*d + e]).  W is
    stored [d_out, d_in], i.e. row n holds column n of the paper's W_q / W_k / W_v."""
    X = np.asarray(X, dtype=np.float64)
    B, L, dm = X.shape
    Y = X @ np.asarray(W, dtype=np.float64).T
    if bias is not None:
        Y = Y + np.asarray(bias, dtype=np.float64)
    return Y.reshape(B, L, H, dm // H).transpose(0, 2, 1, 3)


def merge_heads(A: np.ndarray, Wo: np.ndarray, bo: Optional[np.ndarray]) -> np.ndarray:
    """Concatenate the heads of A [B, H, L, d] along the feature axis and apply
    the output matrix: Y[b, l, j] = sum_{h,e} A[b, h, l, e] Wo[j, h*d + e] (+ bo[j])."""
    A = np.asarray(A, dtype=np.float64)
    B, H, L, d = A.shape
    Y = A.transpose(0, 2, 1, 3).reshape(B, L, H * d) @ np.asarray(Wo, dtype=np.float64).T
    if bo is not None:
        Y = Y + np.asarray(bo, dtype=np.float64)
    return Y


def mhsa_forward(X, Wq, Wk, Wv, Wo, bq, bk, bv, bo, H: int, lengths, sample_idx, c: float,
                 dtype: str = "f64", fill: str = "mean", r_sparse: Optional[float] = None):
    """The whole module: projections, prob-sparse attention per head, output
    matrix.  Q, K, V and the attention output are rounded to the tensors' storage
    type `dtype` where the device path stores them.  Returns (Y, Q, K, V, A)."""
    Q = round_to(project_heads(X, Wq, bq, H), dtype)
    K = round_to(project_heads(X, Wk, bk, H), dtype)
    V = round_to(project_heads(X, Wv, bv, H), dtype)
    A, _, _, _ = probsparse_attn_fwd(Q, K, V, lengths, sample_idx, c, fill=fill, r_sparse=r_sparse)
    A = round_to(A, dtype)
    Y = merge_heads(A, Wo, bo)
    return Y, Q, K, V, A


# ----------------------------------------------------------------------------
# Independent definitions used only to pin the steps above
# ----------------------------------------------------------------------------
def dense_attention(Q: np.ndarray, K: np.ndarray, V: np.ndarray,
                    lengths: Optional[np.ndarray] = None) -> np.ndarray:
    """A(Q,K,V) = softmax(Q K^T / sqrt(d)) V per head (Eq. 6), over valid rows;
    padded query rows are zero."""
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    B, H, L, d = Q.shape
    out = np.zeros_like(Q)
    for b in range(B):
        n = L if lengths is None else int(lengths[b])
        for h in range(H):
            if n > 0:
                out[b, h, :n] = attention_rows(Q[b, h, :n], K[b, h, :n], V[b, h, :n])
    return out


def exact_measure(Q: np.ndarray, K: np.ndarray, n: int) -> np.ndarray:
    """M_sparse(q_i, K) = ln sum_j exp(s_ij) - (1/L) sum_j s_ij over the n valid
    keys (Eq. 10), s_ij = q_i . k_j / sqrt(d)."""
    d = Q.shape[1]
    s = (Q[:n] @ K[:n].T) / math.sqrt(d)
    mx = s.max(axis=1)
    lse = mx + np.log(np.exp(s - mx[:, None]).sum(axis=1))
    return lse - s.sum(axis=1) / n


def kl_measure(Q: np.ndarray, K: np.ndarray, n: int) -> np.ndarray:
    """Right-hand side of Eq. 9: Eq. 10 minus the constant ln L."""
    return exact_measure(Q, K, n) - math.log(n)
