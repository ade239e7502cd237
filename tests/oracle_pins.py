"""Pins for the CPU oracle, written as functions of the oracle module so that
the same checks can be run against deliberately broken copies of it
(tests/test_oracle_mutants.py).  Every check compares the oracle with
something that is not the oracle: a library routine, a closed form, a brute
force, or an invariant the paper's definitions imply.
"""
from __future__ import annotations

import itertools
import math

import numpy as np


def _rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def _rand_head(seed, L, d=64, U=8, scale=1.0):
    r = _rng(seed)
    Q = r.standard_normal((L, d)) * scale
    K = r.standard_normal((L, d)) * scale
    V = r.standard_normal((L, d))
    idx = r.integers(0, L, size=(L, U)).astype(np.int32)
    return Q, K, V, idx


# --- u = ceil(c ln n): closed-form values ------------------------------------
def check_n_selected_closed_form(O):
    # ceil(5 ln 128) = 25 is printed in the benchmark's first workload; the
    # others follow from ln 512 = 6.238.., ln 2048 = 7.624.., ln 16384 = 9.704..,
    # ln 40 = 3.688.., ln 500 = 6.214..
    assert O.n_selected(5.0, 128) == 25
    assert O.n_selected(5.0, 512) == 32
    assert O.n_selected(5.0, 2048) == 39
    assert O.n_selected(5.0, 16384) == 49
    assert O.n_selected(5.0, 40) == 19
    assert O.n_selected(5.0, 500) == 32
    assert O.n_selected(1.0, 512) == 7
    assert O.n_selected(5.0, 1) == 1          # ln 1 = 0 -> clamped to 1
    assert O.n_selected(5.0, 2) == 2          # ceil(3.47) = 4 -> clamped to n
    assert O.n_selected(1e9, 77) == 77
    assert O.n_selected(5.0, 0) == 0


# --- steps 1-5 together: u = L_Q is textbook dense attention (Eq. 6) ---------
def _dense_loops(Q, K, V):
    """Hand-written triple loop, no vectorised step shared with the oracle."""
    L, d = Q.shape
    out = np.zeros((L, d))
    for i in range(L):
        s = [sum(Q[i, e] * K[j, e] for e in range(d)) / math.sqrt(d) for j in range(L)]
        m = max(s)
        w = [math.exp(x - m) for x in s]
        z = sum(w)
        for e in range(d):
            out[i, e] = sum(w[j] * V[j, e] for j in range(L)) / z
    return out


def check_full_selection_is_dense(O):
    import torch
    Q, K, V, idx = _rand_head(11, 24, d=8, U=5)
    out, M, I = O.probsparse_head(Q, K, V, idx, 24, c=1e9)
    assert sorted(I.tolist()) == list(range(24))
    ref = _dense_loops(Q, K, V)
    assert np.allclose(out, ref, rtol=0, atol=1e-13)
    # library SDPA, float64, default scale 1/sqrt(d)
    Q, K, V, idx = _rand_head(12, 96, d=64, U=9)
    out, _, _ = O.probsparse_head(Q, K, V, idx, 96, c=1e9)
    t = lambda a: torch.from_numpy(a)[None, None]
    ref = torch.nn.functional.scaled_dot_product_attention(t(Q), t(K), t(V))[0, 0].numpy()
    assert np.allclose(out, ref, rtol=0, atol=1e-12)
    # the batch-level dense routine agrees with the same library call
    ref2 = O.dense_attention(Q[None, None], K[None, None], V[None, None])[0, 0]
    assert np.allclose(ref2, ref, rtol=0, atol=1e-12)


# --- step 2: properties of max - mean (Eq. 11) --------------------------------
def check_measure_properties(O):
    L, U = 40, 12
    Q, K, V, idx = _rand_head(21, L, U=U)
    M = O.sampled_measure(Q, K, idx, L)
    assert M.shape == (L,)
    assert (M >= 0).all() and (M > 0).any()
    # direct value for one query, by scalar arithmetic
    i = 7
    s = [float(np.dot(Q[i], K[j])) / 8.0 for j in idx[i]]
    assert abs(M[i] - (max(s) - sum(s) / len(s))) < 1e-12
    # permuting the sample columns changes nothing
    perm = _rng(5).permutation(U)
    assert np.allclose(O.sampled_measure(Q, K, idx[:, perm], L), M, atol=1e-12)
    # constant scores -> M = 0: zero query, identical keys, one key sampled U times
    assert np.all(O.sampled_measure(np.zeros_like(Q), K, idx, L) == 0)
    Ksame = np.tile(K[3], (L, 1))
    assert np.allclose(O.sampled_measure(Q, Ksame, idx, L), 0, atol=1e-12)
    one = np.tile(idx[:, :1], (1, U))
    assert np.allclose(O.sampled_measure(Q, K, one, L), 0, atol=1e-12)
    # duplicates weigh the mean, not the max: samples (a, a, b) with s_a > s_b
    q = np.zeros((3, 64)); q[0, 0] = 8.0
    k = np.zeros((3, 64)); k[0, 0] = 3.0; k[1, 0] = 1.0; k[2, 0] = -2.0
    m = O.sampled_measure(q, k, np.array([[0, 0, 1]] * 3, dtype=np.int32), 3)
    assert abs(m[0] - (3.0 - (3.0 + 3.0 + 1.0) / 3.0)) < 1e-12
    # scaling is 1/sqrt(d): d = 16 -> /4
    q = np.zeros((2, 16)); q[0, 1] = 2.0
    k = np.zeros((2, 16)); k[0, 1] = 6.0; k[1, 1] = -6.0
    m = O.sampled_measure(q, k, np.array([[0, 1], [0, 1]], dtype=np.int32), 2)
    assert abs(m[0] - (3.0 - 0.0)) < 1e-12


def check_measure_sandwich_and_kl(O):
    # every key sampled exactly once: max <= LSE <= max + ln L   (Eq. 10 vs Eq. 11)
    from scipy.stats import entropy
    from scipy.special import softmax
    L = 48
    Q, K, V, _ = _rand_head(31, L)
    idx = np.tile(np.arange(L, dtype=np.int32), (L, 1))
    Mbar = O.sampled_measure(Q, K, idx, L)
    Mex = O.exact_measure(Q, K, L)
    assert (Mbar <= Mex + 1e-12).all()
    assert (Mex <= Mbar + math.log(L) + 1e-12).all()
    # Eq. 9's right-hand side is the divergence of the uniform distribution from
    # the attention distribution; scipy computes sum u ln(u/p) independently.
    kl = O.kl_measure(Q, K, L)
    s = (Q @ K.T) / 8.0
    p = softmax(s, axis=1)
    ref = np.array([entropy(np.full(L, 1.0 / L), p[i]) for i in range(L)])
    assert np.allclose(kl, ref, atol=1e-10)
    assert (kl >= -1e-12).all()
    assert np.allclose(Mex - math.log(L), kl, atol=1e-12)


# --- step 3: selection ---------------------------------------------------------
def _is_valid_top_u(M, I, u):
    I = list(I)
    if len(I) != u or len(set(I)) != u:
        return False
    S = set(I)
    for i in S:
        for j in range(len(M)):
            if j in S:
                continue
            if not (M[i] > M[j] or (M[i] == M[j] and i < j)):
                return False
    return True


def check_selection_brute_force(O):
    r = _rng(41)
    for trial in range(40):
        n = int(r.integers(1, 13))
        u = int(r.integers(0, n + 1))
        # few distinct values -> many ties
        M = r.integers(0, 4, size=n).astype(np.float64) if trial % 2 else r.standard_normal(n)
        I = O.select_top_u(M, u)
        assert _is_valid_top_u(M, I, u)
        # enumerate all subsets: exactly one is valid under the tie rule
        valid = [c for c in itertools.combinations(range(n), u) if _is_valid_top_u(M, c, u)]
        assert len(valid) == 1 and set(valid[0]) == set(I.tolist())
        # order: decreasing M, then increasing index
        keys = [(-M[i], i) for i in I]
        assert keys == sorted(keys)
    # all ties -> the first u indices
    assert O.select_top_u(np.zeros(9), 4).tolist() == [0, 1, 2, 3]
    # against numpy's stable sort on the negated values
    M = r.standard_normal(200)
    assert O.select_top_u(M, 17).tolist() == np.argsort(-M, kind="stable")[:17].tolist()


def check_zero_query_selects_first_u(O):
    L = 30
    Q, K, V, idx = _rand_head(51, L)
    out, M, I = O.probsparse_head(np.zeros_like(Q), K, V, idx, L, c=2.0)
    u = O.n_selected(2.0, L)
    assert I.tolist() == list(range(u))
    # Q = 0 -> uniform softmax -> every row, selected or not, is mean(V):
    # here steps 4 and 5 must agree with each other and with numpy's mean.
    assert np.allclose(out, np.mean(V, axis=0)[None, :], atol=1e-13)


# --- steps 4, 5 ------------------------------------------------------------------
def check_fill_and_attention_rows(O):
    L = 64
    Q, K, V, idx = _rand_head(61, L, U=10, scale=1.5)
    out, M, I = O.probsparse_head(Q, K, V, idx, L, c=3.0)
    u = O.n_selected(3.0, L)
    assert len(I) == u == 13
    rest = np.setdiff1d(np.arange(L), I)
    mu = np.mean(V, axis=0)
    assert np.allclose(out[rest], mu[None, :], atol=1e-14)
    assert (out[rest] == out[rest[0]]).all()          # bit-identical rows
    # selected rows are softmax attention: library check on those rows
    from scipy.special import softmax
    p = softmax((Q[I] @ K.T) / 8.0, axis=1)
    assert np.allclose(out[I], p @ V, atol=1e-12)
    assert not np.allclose(out[I], mu[None, :], atol=1e-3)
    # I is what the measure says
    assert set(I.tolist()) == set(np.argsort(-M, kind="stable")[:u].tolist())
    # softmax rows sum to one: V = 1 -> out = 1
    out1, _, _ = O.probsparse_head(Q, K, np.ones_like(V), idx, L, c=3.0)
    assert np.allclose(out1, 1.0, atol=1e-13)
    # paper-literal fill (Eq. 12 lower branch) and explicit u
    out2, _, I2 = O.probsparse_head(Q, K, V, idx, L, c=3.0, n_select=L // 2, fill="value")
    assert len(I2) == L // 2
    rest2 = np.setdiff1d(np.arange(L), I2)
    assert (out2[rest2] == V[rest2]).all()


def check_one_hot_limit(O):
    # orthogonal keys, q_i = beta * k_j: softmax -> one-hot on j, out_i -> v_j
    L, d = 16, 64
    K = np.zeros((L, d)); K[np.arange(L), np.arange(L)] = 1.0
    r = _rng(71)
    V = r.standard_normal((L, d))
    tgt = r.permutation(L)
    Q = 4000.0 * K[tgt]
    idx = np.tile(np.arange(L, dtype=np.int32), (L, 1))
    out, M, I = O.probsparse_head(Q, K, V, idx, L, c=1e9)
    assert np.allclose(out, V[tgt], atol=1e-12)
    # and its measure is max - mean = (beta/8) (1 - 1/L)
    assert np.allclose(M, 500.0 * (1 - 1.0 / L), atol=1e-9)


# --- masking and equivariance -----------------------------------------------------
def check_masking(O):
    B, H, L, d, U = 3, 2, 20, 64, 6
    r = _rng(81)
    lengths = np.array([20, 7, 13], dtype=np.int32)
    Q = r.standard_normal((B, H, L, d)); K = r.standard_normal((B, H, L, d)); V = r.standard_normal((B, H, L, d))
    idx = np.zeros((B, H, L, U), dtype=np.int32)
    for b in range(B):
        idx[b, :, :lengths[b]] = r.integers(0, lengths[b], size=(H, lengths[b], U))
    out, M, sel, u = O.probsparse_attn_fwd(Q, K, V, lengths, idx, 2.0)
    assert u.tolist() == [O.n_selected(2.0, int(n)) for n in lengths]
    # garbage in the padding changes nothing
    Qn, Kn, Vn, idxn = Q.copy(), K.copy(), V.copy(), idx.copy()
    for b in range(B):
        n = lengths[b]
        Qn[b, :, n:] = np.nan; Kn[b, :, n:] = np.nan; Vn[b, :, n:] = np.nan
        idxn[b, :, n:] = 12345
    out2, M2, sel2, _ = O.probsparse_attn_fwd(Qn, Kn, Vn, lengths, idxn, 2.0)
    assert np.array_equal(out, out2) and not np.isnan(out2).any()
    for b in range(B):
        n = lengths[b]
        assert (out[b, :, n:] == 0).all()
        assert np.isnan(M[b, :, n:]).all() and not np.isnan(M[b, :, :n]).any()
        # equals the unpadded run of that item alone
        o1, M1, s1, _ = O.probsparse_attn_fwd(Q[b:b + 1, :, :n], K[b:b + 1, :, :n], V[b:b + 1, :, :n],
                                              None, idx[b:b + 1, :, :n], 2.0)
        assert np.array_equal(o1[0], out[b, :, :n])
        for h in range(H):
            assert s1[0][h].tolist() == sel[b][h].tolist()
            assert (sel[b][h] < n).all()
    # a sample index outside [0, n) is dropped from max and mean
    q = np.zeros((4, 64)); q[:, 0] = 8.0
    k = np.zeros((4, 64)); k[:, 0] = [1.0, 2.0, 50.0, 60.0]
    m = O.sampled_measure(q[:2], k[:2], np.array([[0, 1, 3, -1], [0, 0, 2, 2]], dtype=np.int32), 2)
    assert abs(m[0] - (2.0 - 1.5)) < 1e-12 and abs(m[1]) < 1e-12


def check_key_permutation_equivariance(O):
    L = 36
    Q, K, V, idx = _rand_head(91, L, U=7)
    out, M, I = O.probsparse_head(Q, K, V, idx, L, c=2.5)
    perm = _rng(92).permutation(L)          # new position p holds old key perm[p]
    inv = np.argsort(perm)
    out2, M2, I2 = O.probsparse_head(Q, K[perm], V[perm], inv[idx].astype(np.int32), L, c=2.5)
    assert np.allclose(M2, M, atol=1e-12)
    assert set(I2.tolist()) == set(I.tolist())
    assert np.allclose(out2, out, atol=1e-12)


# --- the paper's own u rule and the given-index variant ------------------------------
def check_ratio_rule_closed_form(O):
    assert O.n_selected_ratio(0.5, 512) == 256
    assert O.n_selected_ratio(0.5, 7) == 4           # 3.5 rounds up
    assert O.n_selected_ratio(0.35, 100) == 35
    assert O.n_selected_ratio(0.35, 101) == 36
    assert O.n_selected_ratio(0.5, 1) == 1
    assert O.n_selected_ratio(0.1, 3) == 1
    assert O.n_selected_ratio(1.0, 33) == 33
    assert O.n_selected_ratio(2.0, 33) == 33         # clamped to n
    assert O.n_selected_ratio(0.5, 0) == 0
    # whole batch: u_b follows each item's own length, rows outside I_sparse are V (Eq. 12)
    B, H, L, d, U = 2, 2, 30, 64, 5
    r = _rng(101)
    lengths = np.array([30, 11], dtype=np.int32)
    Q = r.standard_normal((B, H, L, d)); K = r.standard_normal((B, H, L, d)); V = r.standard_normal((B, H, L, d))
    idx = np.zeros((B, H, L, U), dtype=np.int32)
    for b in range(B):
        idx[b, :, :lengths[b]] = r.integers(0, lengths[b], size=(H, lengths[b], U))
    out, M, sel, u = O.probsparse_attn_fwd(Q, K, V, lengths, idx, 5.0, fill="value", r_sparse=0.5)
    assert u.tolist() == [15, 6]
    from scipy.special import softmax
    for b in range(B):
        n = int(lengths[b])
        for h in range(H):
            I = sel[b][h]
            assert len(I) == u[b]
            assert set(I.tolist()) == set(np.argsort(-M[b, h, :n], kind="stable")[:u[b]].tolist())
            rest = np.setdiff1d(np.arange(n), I)
            assert (out[b, h, rest] == V[b, h, rest]).all()
            p = softmax((Q[b, h, I] @ K[b, h, :n].T) / 8.0, axis=1)
            assert np.allclose(out[b, h, I], p @ V[b, h, :n], atol=1e-12)
        assert (out[b, :, n:] == 0).all()


def check_given_indices(O):
    import torch
    B, H, L, d = 2, 2, 24, 64
    r = _rng(111)
    lengths = np.array([24, 9], dtype=np.int32)
    Q = r.standard_normal((B, H, L, d)); K = r.standard_normal((B, H, L, d)); V = r.standard_normal((B, H, L, d))
    # every valid query kept -> dense attention over the valid keys (library SDPA), padded rows zero
    full = [[np.arange(int(lengths[b])) for _ in range(H)] for b in range(B)]
    out = O.attention_with_indices(Q, K, V, lengths, full)
    for b in range(B):
        n = int(lengths[b])
        ref = torch.nn.functional.scaled_dot_product_attention(
            torch.from_numpy(Q[b, :, :n]), torch.from_numpy(K[b, :, :n]), torch.from_numpy(V[b, :, :n])).numpy()
        assert np.allclose(out[b, :, :n], ref, atol=1e-12)
        assert (out[b, :, n:] == 0).all()
    # nothing kept -> the fill alone
    none = [[np.zeros(0, dtype=np.int64) for _ in range(H)] for _ in range(B)]
    o_mean = O.attention_with_indices(Q, K, V, lengths, none, fill="mean")
    o_val = O.attention_with_indices(Q, K, V, lengths, none, fill="value")
    for b in range(B):
        n = int(lengths[b])
        assert np.allclose(o_mean[b, :, :n], V[b, :, :n].mean(axis=1, keepdims=True), atol=1e-14)
        assert (o_val[b, :, :n] == V[b, :, :n]).all() and (o_val[b, :, n:] == 0).all()
    # a hand-picked set: kept rows are attention rows (hand loop), the others the fill
    pick = [[np.array([1, 5, 7]), np.array([0])], [np.array([8, 2]), np.array([3, 4, 6])]]
    o = O.attention_with_indices(Q, K, V, lengths, pick)
    for b in range(B):
        n = int(lengths[b])
        for h in range(H):
            for i in range(n):
                if i in pick[b][h].tolist():
                    w = np.array([math.exp(float(Q[b, h, i] @ K[b, h, j]) / 8.0) for j in range(n)])
                    ref = sum(w[j] * V[b, h, j] for j in range(n)) / w.sum()
                else:
                    ref = V[b, h, :n].mean(axis=0)
                assert np.allclose(o[b, h, i], ref, atol=1e-12)
    # the index set of the full method, handed back in, reproduces the full method
    idx = r.integers(0, 9, size=(B, H, L, 6)).astype(np.int32)
    o_full, _, sel, _ = O.probsparse_attn_fwd(Q, K, V, lengths, idx, 2.0)
    assert np.array_equal(O.attention_with_indices(Q, K, V, lengths, sel), o_full)


# --- the projections around the path ---------------------------------------------------
def check_mhsa_against_library(O):
    import torch
    B, L, H, d = 2, 12, 2, 64
    dm = H * d
    r = _rng(121)
    X = r.standard_normal((B, L, dm)) * 0.5
    Wq, Wk, Wv, Wo = (r.standard_normal((dm, dm)) / math.sqrt(dm) for _ in range(4))
    bq, bk, bv, bo = (r.standard_normal(dm) * 0.1 for _ in range(4))
    idx = r.integers(0, L, size=(B, H, L, 4)).astype(np.int32)
    # every query kept (c huge): the module is the textbook multi-head attention
    Y, Q, K, V, A = O.mhsa_forward(X, Wq, Wk, Wv, Wo, bq, bk, bv, bo, H, None, idx, 1e9)
    t = lambda a: torch.from_numpy(np.asarray(a))
    ref, _ = torch.nn.functional.multi_head_attention_forward(
        t(X).transpose(0, 1), t(X).transpose(0, 1), t(X).transpose(0, 1), dm, H,
        torch.cat([t(Wq), t(Wk), t(Wv)]), torch.cat([t(bq), t(bk), t(bv)]), None, None, False, 0.0,
        t(Wo), t(bo), need_weights=False)
    assert np.allclose(Y, ref.transpose(0, 1).numpy(), atol=1e-11)
    # layout of the projected heads: element (b, h, l, e) is feature h*d + e of frame l
    assert np.allclose(Q[1, 1, 3, 5], X[1, 3] @ Wq[d + 5] + bq[d + 5], atol=1e-12)
    assert np.allclose(V[0, 0, 7, 63], X[0, 7] @ Wv[63] + bv[63], atol=1e-12)
    # identity matrices, no bias: the module is the attention on X cut into heads
    I = np.eye(dm)
    lengths = np.array([L, 7], dtype=np.int32)
    idx2 = np.minimum(idx, 6)
    Y2, Q2, _, _, A2 = O.mhsa_forward(X, I, I, I, I, None, None, None, None, H, lengths, idx2, 2.0)
    Xh = X.reshape(B, L, H, d).transpose(0, 2, 1, 3)
    assert np.array_equal(Q2, Xh)
    ref2, _, _, _ = O.probsparse_attn_fwd(Xh, Xh, Xh, lengths, idx2, 2.0)
    assert np.allclose(Y2, ref2.transpose(0, 2, 1, 3).reshape(B, L, dm), atol=1e-13)
    # storage rounding: bfloat16 keeps 8 significant bits, ties to even
    assert O.round_to(np.array([1.0 + 2.0 ** -8]), "bf16")[0] == 1.0
    assert O.round_to(np.array([1.0 + 3 * 2.0 ** -8]), "bf16")[0] == 1.0 + 2.0 ** -6
    assert O.round_to(np.array([1.0 + 2.0 ** -7]), "bf16")[0] == 1.0 + 2.0 ** -7
    assert O.round_to(np.array([0.1]), "f32")[0] == float(np.float32(0.1))


# --- gradients of steps 4 and 5 for a fixed index set -------------------------------
def _torch_forward_fixed_sets(Q, K, V, lengths, sel, fill):
    """The forward for given index sets written with the library's differentiable ops (float64)."""
    import torch
    B, H, L, d = Q.shape
    rows = []
    for b in range(B):
        n = L if lengths is None else int(lengths[b])
        for h in range(H):
            q, k, v = Q[b, h, :n], K[b, h, :n], V[b, h, :n]
            base = v.mean(dim=0, keepdim=True).expand(n, d) if fill == "mean" else v
            I = torch.as_tensor(np.asarray(sel[b][h], dtype=np.int64))
            if I.numel():
                att = torch.softmax(q[I] @ k.T / math.sqrt(d), dim=1) @ v
                keep = torch.ones(n, 1, dtype=torch.float64)
                keep[I] = 0.0
                scat = torch.zeros(n, d, dtype=torch.float64).index_add(0, I, att)
                o = base * keep + scat
            else:
                o = base
            rows.append(torch.cat([o, torch.zeros(L - n, d, dtype=torch.float64)], dim=0))
    return torch.stack(rows).reshape(B, H, L, d)


def check_backward_against_autograd(O):
    import torch
    r = _rng(4100)
    B, H, L, d = 3, 2, 23, 64
    lengths = np.array([23, 9, 1], dtype=np.int32)
    Q, K, V, G = (r.standard_normal((B, H, L, d)) for _ in range(4))
    sel = [[np.sort(r.choice(int(lengths[b]), size=min(int(lengths[b]), 5), replace=False)) for _ in range(H)]
           for b in range(B)]
    sel[1][1] = np.zeros(0, dtype=np.int64)                        # a head that keeps no query
    sel[0][0] = r.permutation(23)[:11]                             # any order
    for fill in ("mean", "value"):
        tq, tk, tv = (torch.tensor(a, dtype=torch.float64, requires_grad=True) for a in (Q, K, V))
        out_t = _torch_forward_fixed_sets(tq, tk, tv, lengths, sel, fill)
        # the torch forward itself must be the oracle's forward
        out_o = O.attention_with_indices(Q, K, V, lengths, sel, fill=fill)
        assert np.abs(out_t.detach().numpy() - out_o).max() < 1e-12
        (out_t * torch.tensor(G)).sum().backward()
        dQ, dK, dV = O.attention_with_indices_backward(Q, K, V, lengths, sel, G, fill=fill)
        for got, ref in ((dQ, tq.grad), (dK, tk.grad), (dV, tv.grad)):
            assert np.abs(got - ref.numpy()).max() < 1e-11, fill
        for b in range(B):
            n = int(lengths[b])
            assert (dQ[b, :, n:] == 0).all() and (dK[b, :, n:] == 0).all() and (dV[b, :, n:] == 0).all()
            for h in range(H):
                outside = np.setdiff1d(np.arange(n), sel[b][h])
                assert (dQ[b, h, outside] == 0).all()              # no gradient reaches an unselected query


def check_backward_finite_differences(O):
    # central differences of the oracle's own forward, contracted with the upstream gradient
    r = _rng(4200)
    B, H, L, d = 1, 2, 12, 64
    Q, K, V, G = (r.standard_normal((B, H, L, d)) for _ in range(4))
    lengths = np.array([10], dtype=np.int32)
    sel = [[np.array([7, 2, 4]), np.array([0, 9])]]
    eps = 1e-6
    for fill in ("mean", "value"):
        grads = O.attention_with_indices_backward(Q, K, V, lengths, sel, G, fill=fill)
        for which, arr in enumerate((Q, K, V)):
            for _ in range(12):
                pos = (0, int(r.integers(H)), int(r.integers(10)), int(r.integers(d)))
                keep = arr[pos]
                arr[pos] = keep + eps
                fp = (O.attention_with_indices(Q, K, V, lengths, sel, fill=fill) * G).sum()
                arr[pos] = keep - eps
                fm = (O.attention_with_indices(Q, K, V, lengths, sel, fill=fill) * G).sum()
                arr[pos] = keep
                fd = (fp - fm) / (2 * eps)
                assert abs(fd - grads[which][pos]) < 1e-6 * max(1.0, abs(fd)), (fill, which, pos)


def check_backward_closed_forms(O):
    r = _rng(4300)
    d = 64
    # one key: the softmax weight is 1 whatever q and k are, so dQ = dK = 0 and dV_0 collects every row of G
    Q, K, V, G = (r.standard_normal((1, 1, 1, d)) for _ in range(4))
    dQ, dK, dV = O.attention_with_indices_backward(Q, K, V, None, [[np.array([0])]], G)
    assert np.abs(dQ).max() < 1e-15 and np.abs(dK).max() < 1e-15 and np.abs(dV[0, 0, 0] - G[0, 0, 0]).max() < 1e-15
    # nothing kept, mean fill: out_i = mean(V) for all i, so every dV_j = (sum_i G_i) / n; value fill: dV = G
    L = 9
    Q, K, V, G = (r.standard_normal((1, 1, L, d)) for _ in range(4))
    none = [[np.zeros(0, dtype=np.int64)]]
    lengths = np.array([7], dtype=np.int32)
    dQ, dK, dV = O.attention_with_indices_backward(Q, K, V, lengths, none, G, fill="mean")
    assert np.abs(dV[0, 0, :7] - G[0, 0, :7].sum(axis=0) / 7).max() < 1e-14 and (dV[0, 0, 7:] == 0).all()
    assert (dQ == 0).all() and (dK == 0).all()
    dQ, dK, dV = O.attention_with_indices_backward(Q, K, V, lengths, none, G, fill="value")
    assert np.array_equal(dV[0, 0, :7], G[0, 0, :7]) and (dV[0, 0, 7:] == 0).all()
    # q = 0: uniform weights 1/n; with G_i orthogonal to nothing in particular the score gradient is
    # g_ij = (1/n) (G_i . v_j - mean_j' G_i . v_j'), so dK_j = (1/sqrt(d)) g_ij q_i = 0 and
    # dQ_i = (1/sqrt(d)) (1/n) sum_j (G_i . (v_j - vbar)) k_j
    n = 5
    Q = np.zeros((1, 1, n, d)); K, V, G = (r.standard_normal((1, 1, n, d)) for _ in range(3))
    dQ, dK, dV = O.attention_with_indices_backward(Q, K, V, None, [[np.array([3])]], G, fill="value")
    vbar = V[0, 0].mean(axis=0)
    want = sum((G[0, 0, 3] @ (V[0, 0, j] - vbar)) * K[0, 0, j] for j in range(n)) / n / math.sqrt(d)
    assert np.abs(dQ[0, 0, 3] - want).max() < 1e-13 and np.abs(dK).max() < 1e-15
    # rows of the softmax gradient sum to zero: adding a constant to every score of a query changes nothing,
    # i.e. dQ_i . t = 0 whenever every key has the same component along t (all k_j . t equal)
    K2 = K.copy(); t = r.standard_normal(d); t /= np.linalg.norm(t)
    K2[0, 0] = K2[0, 0] - np.outer(K2[0, 0] @ t, t) + 0.7 * t        # every key now has component 0.7 along t
    Qr = r.standard_normal((1, 1, n, d))
    dQ, _, _ = O.attention_with_indices_backward(Qr, K2, V, None, [[np.array([1, 2])]], G)
    assert np.abs(dQ[0, 0, [1, 2]] @ t).max() < 1e-13


ALL_CHECKS = [
    check_n_selected_closed_form,
    check_full_selection_is_dense,
    check_measure_properties,
    check_measure_sandwich_and_kl,
    check_selection_brute_force,
    check_zero_query_selects_first_u,
    check_fill_and_attention_rows,
    check_one_hot_limit,
    check_masking,
    check_key_permutation_equivariance,
    check_ratio_rule_closed_form,
    check_given_indices,
    check_mhsa_against_library,
    check_backward_against_autograd,
    check_backward_finite_differences,
    check_backward_closed_forms,
]
