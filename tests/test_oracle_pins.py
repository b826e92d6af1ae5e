"""Pins for the CPU oracle: closed forms, invariants, library routines and brute force.

The paper prints no worked numeric example, so the oracle is pinned to what the
equations and the mathematics fix.  Each test names the passage it checks."""
import itertools
import math
import os

import numpy as np
import pytest

from oracle import ficoco_oracle as O
from tests import brute_force as BF

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rng(seed):
    return np.random.default_rng(seed)


def softmax_rows(z):
    e = np.exp(z - z.max(axis=-1, keepdims=True))
    return e / e.sum(axis=-1, keepdims=True)


# ------------------------------------------------------------------ number formats
def test_widen_bf16_bits():
    # 0x3F80 = 1.0, 0xC000 = -2.0, 0x3DCC = 0.099609375 (bfloat16 patterns are the top half of float32)
    got = O.widen(np.array([0x3F80, 0xC000, 0x3DCC, 0x0000], dtype=np.uint16))
    assert got.tolist() == [1.0, -2.0, 0.099609375, 0.0]


def test_round_to_bf16_is_nearest_even():
    # spacing in [1, 2) is 2^-7; 1 + 2^-8 is a tie -> even mantissa (1.0); 1 + 3*2^-8 -> 1 + 2^-6
    assert O.round_to_bf16(np.array([1.0 + 2.0 ** -8]))[0] == 1.0
    assert O.round_to_bf16(np.array([1.0 + 3 * 2.0 ** -8]))[0] == 1.0 + 2.0 ** -6
    assert O.round_to_bf16(np.array([1.0 + 2.0 ** -8 + 2.0 ** -30]))[0] == 1.0 + 2.0 ** -7
    assert O.round_to_bf16(np.array([-0.3]))[0] == -0.30078125
    # agrees with torch's float32 -> bfloat16 cast on float32-representable inputs
    import torch
    x = rng(0).standard_normal(4096).astype(np.float32) * np.float32(0.05)
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(O.round_to_bf16(x.astype(np.float64)), ref)
    # idempotent
    assert np.array_equal(O.round_to_bf16(ref), ref)


# ------------------------------------------------------------------ Eq. 1 / Eq. 3 score terms
def test_uniform_attention_ties_everything():
    """Uniform P = 1/n: every token receives the same -> all scores tie -> the filter
    discards the lowest indices (Eq. 1 + top-K with the lower-index tie rule)."""
    H, n = 3, 13
    A = np.full((H, n, n), 1.0 / n)
    P = O.head_mean(A)
    vis = np.arange(1, n)
    R = O.received_attention(P, vis, vis)
    G = O.cls_attention(P, 0, vis)
    assert np.all(R == R[0]) and np.all(G == G[0])
    assert abs(R[0] - 1.0 / n) < 1e-15          # (N rows * 1/n) / N
    s = O.combine_score(R, G, 0.35)
    S, T = O.filter_tokens(s, 5)
    assert S.tolist() == list(range(7)) and T.tolist() == list(range(7, 12))


def test_one_hot_column_receives_everything():
    """Every query attends only token c: R_c = 1 (N rows each give 1, divided by N), others 0."""
    n, c = 9, 4
    A = np.zeros((2, n, n))
    A[:, :, c] = 1.0
    P = O.head_mean(A)
    vis = np.arange(1, n)
    R = O.received_attention(P, vis, vis)
    expect = np.zeros(n - 1)
    expect[c - 1] = 1.0
    assert np.array_equal(R, expect)
    assert np.array_equal(O.cls_attention(P, 0, vis), expect)


def test_column_sums_of_row_stochastic_map():
    """sum_i N*R_i + (mass the visual queries put on the [CLS] column) = number of visual
    query rows, because each row of a softmax sums to one."""
    r = rng(1)
    H, n = 4, 21
    A = softmax_rows(r.standard_normal((H, n, n)))
    P = O.head_mean(A)
    vis = np.arange(1, n)
    R = O.received_attention(P, vis, vis)
    total = (n - 1) * R.sum() + P[1:, 0].sum()
    assert abs(total - (n - 1)) < 1e-12


def test_received_is_column_not_row_mean():
    """A transposed operand must fail: with P = outer(ones, p) every ROW is the same
    distribution p; the received attention of token i is then p_i, whereas a row mean
    would be the constant 1/N'."""
    p = np.array([0.1, 0.2, 0.3, 0.4])
    P = np.tile(p, (4, 1))
    idx = np.arange(4)
    assert np.allclose(O.received_attention(P, idx, idx), p, rtol=0, atol=1e-16)


def test_head_mean_is_mean_over_heads():
    r = rng(2)
    A = r.random((5, 6, 7))
    assert np.allclose(O.head_mean(A), A.mean(axis=0), rtol=1e-15, atol=0)
    assert np.allclose(O.head_mean_vector(A[:, 0]), A[:, 0].mean(axis=0), rtol=1e-15, atol=0)


def test_score_isolates_terms_and_sign():
    """Eq. 1: lambda = 1 leaves the received term, lambda = 0 leaves MINUS the [CLS] term."""
    R = np.array([0.1, 0.4, 0.2])
    G = np.array([0.3, 0.1, 0.5])
    assert np.array_equal(O.combine_score(R, G, 1.0), R)
    assert np.array_equal(O.combine_score(R, G, 0.0), -G)
    s = O.combine_score(R, G, 0.25)
    assert np.allclose(s, 0.25 * R - 0.75 * G, rtol=1e-15)
    # Eq. 3 task term: mean over text rows
    P = np.array([[0.2, 0.8], [0.6, 0.4], [0.1, 0.9]])
    assert np.allclose(O.text_attention(P, [1, 2], np.array([0, 1])), [0.35, 0.65], rtol=1e-15)


# ------------------------------------------------------------------ self-attention from Q, K
def test_attention_from_qk_closed_forms_and_library_softmax():
    """Sec. "Self-Attention": rows are softmaxes.  Identical keys (or zero queries) give the
    uniform map 1/nk exactly-ish; a key that every query is aligned with takes the whole row as
    the scale grows; the general case equals a library log-sum-exp evaluation; and a step fed
    Q, K equals the step fed the map they define (nothing else changes)."""
    from scipy.special import logsumexp
    r = rng(70)
    H, n, d = 3, 9, 4
    Q = r.standard_normal((H, n, d))
    K = np.tile(r.standard_normal((H, 1, d)), (1, n, 1))          # all keys of a head identical
    A = O.attention_from_qk(Q, K, 0.5)
    assert A.shape == (H, n, n) and np.allclose(A, 1.0 / n, rtol=0, atol=1e-15)
    assert np.allclose(O.attention_from_qk(np.zeros((H, n, d)), r.standard_normal((H, n, d)), 0.5), 1.0 / n, atol=1e-15)
    # one-hot limit: key 2 = 50 * e0, queries = e0  ->  logits 50 * scale on key 2, 0 elsewhere
    Q1 = np.zeros((1, 5, d)); Q1[0, :, 0] = 1.0
    K1 = np.zeros((1, 5, d)); K1[0, 2, 0] = 50.0
    A1 = O.attention_from_qk(Q1, K1, 1.0)
    want = np.exp(50.0) / (np.exp(50.0) + 4.0)
    assert np.allclose(A1[0, :, 2], want, rtol=1e-14) and np.allclose(A1[0, :, 0], (1 - want) / 4, rtol=1e-10)
    # general case against log-sum-exp; rows sum to one; the scale crosses as float32
    K = r.standard_normal((H, n + 2, d))
    A = O.attention_from_qk(Q, K, 0.3)
    sc = float(np.float32(0.3))
    for h in range(H):
        L = (Q[h] @ K[h].T) * sc
        assert np.allclose(A[h], np.exp(L - logsumexp(L, axis=1, keepdims=True)), rtol=1e-13)
    assert np.allclose(A.sum(axis=2), 1.0, rtol=0, atol=1e-14)
    # transposing the roles of Q and K is NOT the same map (a transposed operand must fail)
    assert not np.allclose(O.attention_from_qk(Q, Q[:, ::-1], 0.3), O.attention_from_qk(Q[:, ::-1], Q, 0.3))


def test_step_from_qk_equals_step_from_the_map_it_defines():
    r = rng(71)
    H, g, D, d = 2, 4, 6, 4
    n = g * g + 1
    X = r.standard_normal((n, D))
    Q, K = r.standard_normal((H, n, d)), r.standard_normal((H, n, d))
    A = O.attention_from_qk(Q, K, 0.5)
    kw = dict(cls_index=0, vis_begin=1, N=n - 1, n_keep=9, grid=(1, g, g))
    a, b = O.v_step(X, A, **kw), O.v_step_qk(X, Q, K, 0.5, **kw)
    assert np.array_equal(a["S"], b["S"]) and np.array_equal(a["X_out"], b["X_out"])
    assert all(np.array_equal(x, y) for x, y in zip(a["J"], b["J"]))


def test_causal_attention_from_qk():
    """The decoder's causal maps: row r is the unmasked softmax over keys 0 .. r alone (computed
    here row by row with a library log-sum-exp on the truncated key set), zero above the diagonal,
    the first row is (1, 0, ...), identical keys give 1 / (r + 1); and a FiCoCo-L step fed Q, K
    equals the step fed the visual and text blocks of the maps they define."""
    from scipy.special import logsumexp
    r = rng(72)
    H, n, d = 2, 11, 4
    Q, K = r.standard_normal((H, n, d)), r.standard_normal((H, n, d))
    A = O.attention_from_qk(Q, K, 0.4, causal=True)
    sc = float(np.float32(0.4))
    for h in range(H):
        for q in range(n):
            L = (K[h, :q + 1] @ Q[h, q]) * sc
            assert np.allclose(A[h, q, :q + 1], np.exp(L - logsumexp(L)), rtol=1e-13)
            assert np.all(A[h, q, q + 1:] == 0.0)
    assert np.all(A[:, 0, 0] == 1.0)
    same = O.attention_from_qk(Q, np.tile(K[:, :1], (1, n, 1)), 0.4, causal=True)
    for q in range(n):
        assert np.allclose(same[:, q, :q + 1], 1.0 / (q + 1), rtol=0, atol=1e-15)
    # the step: 2 system tokens, 6 visual, 3 text
    n_sys, N, M, D = 2, 6, 3, 5
    X = r.standard_normal((n, D))
    kw = dict(n_keep=3, beta=0.6, gamma=0.6)
    vis, txt = slice(n_sys, n_sys + N), slice(n_sys + N, n)
    a = O.l_step(X, A[:, vis, vis], A[:, txt, vis], vis_begin=n_sys, N=N, **kw)
    b = O.l_step_qk(X, Q, K, 0.4, vis_begin=n_sys, N=N, M=M, **kw)
    assert np.array_equal(a["S"], b["S"]) and np.array_equal(a["X_out"], b["X_out"])
    assert all(np.array_equal(x, y) for x, y in zip(a["J"], b["J"]))


# ------------------------------------------------------------------ equivalent token / mean cosine
def test_equivalent_token_closed_forms():
    """a^Eq = -cos(mu, F_i): identical tokens -> -1; F = {e1, e2} -> mu = (.5,.5), cos = 1/sqrt2."""
    F = np.tile(np.array([1.0, 2.0, -3.0]), (5, 1))
    assert np.allclose(O.equivalent_token_term(F), -1.0, rtol=0, atol=1e-15)
    F = np.eye(2)
    assert np.allclose(O.equivalent_token_term(F), -1 / math.sqrt(2), rtol=0, atol=1e-15)
    # a textbook evaluation
    r = rng(3)
    F = r.standard_normal((7, 5))
    mu = F.mean(axis=0)
    ref = -(F @ mu) / (np.linalg.norm(F, axis=1) * np.linalg.norm(mu))
    assert np.allclose(O.equivalent_token_term(F), ref, rtol=1e-13)
    # a common positive scale changes nothing
    assert np.allclose(O.equivalent_token_term(3.5 * F), ref, rtol=1e-13)


def test_mean_cosine_closed_forms():
    """Orthonormal tokens: each has cosine 1 with itself and 0 with the others -> 1/N.
    Identical tokens -> 1.  It is the row mean of the full cosine matrix."""
    assert np.allclose(O.mean_cosine_term(np.eye(6)), 1.0 / 6.0, rtol=0, atol=1e-16)
    assert np.allclose(O.mean_cosine_term(np.tile([3.0, 4.0], (4, 1))), 1.0, atol=1e-15)
    r = rng(4)
    F = r.standard_normal((9, 4))
    ref = np.array([np.mean([np.dot(F[i], F[j]) / (np.linalg.norm(F[i]) * np.linalg.norm(F[j]))
                             for j in range(9)]) for i in range(9)])
    assert np.allclose(O.mean_cosine_term(F), ref, rtol=1e-13)


def test_cosine_terms_tie_exactly_where_the_features_are_collinear():
    """Both cosine-derived score terms are sums in a fixed index order, so tokens that differ by
    a sign-preserving power of two -- and every token when there is one feature -- get the very
    same float64 (the filter then ranks them by index).  With one feature the values are the
    closed forms (n_same - n_opposite)/N and -sign(mu) sign(F_i)."""
    F = np.array([[0.75], [-2.5], [3.0], [0.125], [-7.0]])
    R = O.mean_cosine_term(F)
    assert np.array_equal(R, np.array([0.2, -0.2, 0.2, 0.2, -0.2]))
    G = O.equivalent_token_term(F)                       # mu = -5.625 / 5 < 0
    assert np.array_equal(G, np.array([1.0, -1.0, 1.0, 1.0, -1.0]))
    r = rng(41)
    base = r.standard_normal((6, 24)).astype(np.float32).astype(np.float64)
    F = np.concatenate([base, 4.0 * base[:3], 0.5 * base[3:]])
    R, G = O.mean_cosine_term(F), O.equivalent_token_term(F)
    assert np.array_equal(R[6:9], R[:3]) and np.array_equal(R[9:], R[3:6])
    assert np.array_equal(G[6:9], G[:3]) and np.array_equal(G[9:], G[3:6])
    # the cosine matrix against a library matrix product of the unit rows
    U = F / np.linalg.norm(F, axis=1)[:, None]
    assert np.allclose(O.cosine_matrix(F), U @ U.T, rtol=0, atol=1e-14)
    assert np.allclose(np.diag(O.cosine_matrix(F)), 1.0, rtol=0, atol=1e-14)


# ------------------------------------------------------------------ local penalty
def test_local_penalty_golden_4x4():
    """Hand-computed example (tests/golden/local_penalty_4x4.txt): 4x4 grid, 2x2 windows,
    coefficient 2.  One maximum per window is doubled, negative maxima become more negative."""
    rows = [l.split() for l in open(os.path.join(GOLDEN, "local_penalty_4x4.txt"))
            if l.strip() and not l.startswith("#")]
    s = np.array([float(v) for v in rows[0]])
    want = np.array([float(v) for v in rows[1]])
    got = O.local_penalty(s, np.arange(16), 1, 4, 4, 2, 2.0)
    assert np.array_equal(got, want)


def test_local_penalty_properties():
    r = rng(5)
    s = r.standard_normal(2 * 6 * 6)
    pos = np.arange(72)
    # coefficient 1 = no penalty (the paper's "w/o local penalty" ablation row)
    assert np.array_equal(O.local_penalty(s, pos, 2, 6, 6, 2, 1.0), s)
    assert np.array_equal(O.local_penalty(s, pos, 2, 6, 6, 0, 2.0), s)
    out = O.local_penalty(s, pos, 2, 6, 6, 2, 2.0)
    changed = np.nonzero(out != s)[0]
    assert len(changed) == 2 * 3 * 3                       # exactly one per window
    assert np.array_equal(out[changed], 2.0 * s[changed])
    for t in changed:                                       # each is its window's maximum
        sub, cell = divmod(t, 36)
        rr, cc = divmod(cell, 6)
        win = [sub * 36 + (rr // 2 * 2 + a) * 6 + (cc // 2 * 2 + b) for a in (0, 1) for b in (0, 1)]
        assert s[t] == max(s[win])
    # padding: drop three cells of the first window; the survivor is multiplied even if it
    # was not the window maximum before; windows emptied entirely change nothing.
    keep = np.array([t for t in range(72) if t not in (0, 1, 6)])
    out2 = O.local_penalty(s[keep], pos[keep], 2, 6, 6, 2, 2.0)
    assert out2[list(keep).index(7)] == 2.0 * s[7]
    # ragged grid: 3x3 with 2x2 windows has 4 windows (partial ones allowed)
    s9 = np.arange(9.0)
    out9 = O.local_penalty(s9, np.arange(9), 1, 3, 3, 2, 2.0)
    # windows {0,1,3,4} {2,5} {6,7} {8}: maxima at cells 4, 5, 7, 8
    assert np.array_equal(out9, [0, 1, 2, 3, 2 * 4, 2 * 5, 6, 2 * 7, 2 * 8])
    # ties: lowest cell wins
    out_t = O.local_penalty(np.ones(4), np.array([3, 2, 1, 0]), 1, 2, 2, 2, 2.0)
    assert out_t.tolist() == [1.0, 1.0, 1.0, 2.0]


# ------------------------------------------------------------------ filter
def test_filter_invariants_and_bruteforce():
    r = rng(6)
    for trial in range(50):
        n = int(r.integers(1, 40))
        s = r.integers(-3, 4, size=n).astype(np.float64) if trial % 2 else r.standard_normal(n)
        n_keep = int(r.integers(0, n + 1))
        S, T = O.filter_tokens(s, n_keep)
        assert len(T) == n_keep and len(S) == n - n_keep
        assert sorted(S.tolist() + T.tolist()) == list(range(n))
        assert np.all(np.diff(S) > 0) and np.all(np.diff(T) > 0)
        if len(S) and len(T):
            assert s[S].min() >= s[T].max()
            worst = max((-s[i], i) for i in S)          # last discarded in (score desc, index asc)
            best = min((-s[j], j) for j in T)
            assert worst < best
        S2, T2 = BF.split(s.tolist(), n_keep)
        assert S.tolist() == S2 and T.tolist() == T2


# ------------------------------------------------------------------ correlate
def test_v_correlation_is_a_gather_with_received_orientation():
    """C[i, j] = P[query j, key i]: asymmetric map so a transposed gather fails."""
    P = np.arange(36, dtype=np.float64).reshape(6, 6)
    vis = np.arange(1, 6)
    S, T = np.array([0, 3]), np.array([1, 2, 4])
    C = O.correlation_attention(P, S, T, vis, vis)
    for a, i in enumerate(S):
        for b, j in enumerate(T):
            assert C[a, b] == P[1 + j, 1 + i]


def test_materialise_f32_rounds_once():
    x = np.array([1.0 + 2.0 ** -30, 0.1])
    assert O.materialise_f32(x).tolist() == [1.0, float(np.float32(0.1))]


def test_l_correlation_special_cases():
    """Eq. 4: gamma = 1 is the direct (V) correlation; gamma = 0 with one-hot text profiles
    gives (1/M) * [number of text tokens that attend both i and j]."""
    r = rng(7)
    N, M = 7, 3
    direct = r.random((2, 5))
    bridge = r.random((2, 5))
    assert np.array_equal(O.correlation_l(direct, bridge, 1.0), direct)
    assert np.array_equal(O.correlation_l(direct, bridge, 0.0), bridge)
    g = float(np.float32(0.6))
    assert np.allclose(O.correlation_l(direct, bridge, 0.6), g * direct + (1 - g) * bridge, rtol=1e-15)
    Pt = np.zeros((M, N))
    owner = [0, 1, 2, 0, 1, 2, 0]                 # text token k attends visual tokens with owner k
    for i, k in enumerate(owner):
        Pt[k, i] = 1.0
    S, T = np.array([0, 1]), np.array([2, 3, 4, 5, 6])
    Bm = O.text_bridge(Pt, S, T)
    for a, i in enumerate(S):
        for b, j in enumerate(T):
            assert Bm[a, b] == (1.0 / M if owner[i] == owner[j] else 0.0)
    # general case against a textbook matrix product
    Pt = r.random((M, N))
    assert np.allclose(O.text_bridge(Pt, S, T), (Pt[:, S].T @ Pt[:, T]) / M, rtol=1e-14)


def test_cosine_correlation_properties():
    r = rng(8)
    F = r.standard_normal((12, 64))
    idx = np.arange(12)
    G = O.correlation_cosine(F, idx, idx)
    assert np.array_equal(G, G.T)
    assert np.all(np.abs(np.diag(G) - 1.0) < 2.0 ** -7)       # unit rows up to bf16 rounding
    assert G.min() >= 0.0 and G.max() <= 1.0 + 2.0 ** -6
    Un = F / np.linalg.norm(F, axis=1, keepdims=True)
    assert np.max(np.abs(G - np.maximum(Un @ Un.T, 0))) < 2.0 ** -7
    # every operand really is a bfloat16 value
    Uh = O.round_to_bf16(O.unit_rows(F))
    assert np.array_equal(O.round_to_bf16(Uh), Uh)
    # zero row -> zero correlation, no NaN
    F[3] = 0.0
    G = O.correlation_cosine(F, idx, idx)
    assert np.all(G[3] == 0.0) and np.all(np.isfinite(G))
    # rectangular block is the sub-matrix
    S, T = np.array([1, 5]), np.array([0, 2, 7])
    assert np.array_equal(O.correlation_cosine(F, S, T), G[np.ix_(S, T)])


# ------------------------------------------------------------------ threshold and weights
def test_quantile_matches_library_and_closed_form():
    r = rng(9)
    for n in (1, 2, 3, 17, 144, 192, 384, 640, 1152):
        row = r.standard_normal(n)
        for eps in (0.0, 0.25, 0.5, 0.9, 0.998, 1.0):
            e32 = float(np.float32(eps))
            ref = np.quantile(row, e32, method="linear")
            assert abs(O.quantile_threshold(row, eps) - ref) <= 1e-14 * max(1.0, abs(ref))
    # type-7 quantile of 0..n-1 is eps*(n-1)
    for n in (5, 384, 1152):
        e32 = float(np.float32(0.998))
        assert abs(O.quantile_threshold(np.arange(n, dtype=np.float64), 0.998) - e32 * (n - 1)) < 1e-12


@pytest.mark.parametrize("n,expect", [(144, 1), (192, 1), (256, 1), (384, 1), (640, 2), (1152, 3)])
def test_adaptive_k_closed_form(n, expect):
    """With distinct values |J_i| = n-1-floor(p) (fractional p = eps(n-1)) at eps = 0.998."""
    r = rng(10 + n)
    C = r.random((3, n))
    J, alpha, tau = O.correlated_targets(C, 0.998)
    for i in range(3):
        assert len(J[i]) == expect
        top = np.argsort(-C[i])[:expect]
        assert sorted(J[i].tolist()) == sorted(top.tolist())
        assert abs(alpha[i].sum() - 1.0) < 1e-15 and np.all(alpha[i] >= 0)
        assert np.allclose(alpha[i], C[i, J[i]] / C[i, J[i]].sum(), rtol=1e-15)


def test_threshold_edge_cases():
    r = rng(11)
    C = r.random((4, 10))
    J, alpha, _ = O.correlated_targets(C, 1.0)                 # eps = 1: arg-max set
    for i in range(4):
        assert J[i].tolist() == [int(np.argmax(C[i]))] and alpha[i].tolist() == [1.0]
    J, alpha, _ = O.correlated_targets(C, 0.0)                 # eps = 0: every target
    for i in range(4):
        assert J[i].tolist() == list(range(10))
        assert np.allclose(alpha[i], C[i] / C[i].sum(), rtol=1e-15)
    # ties at the top are all selected (C >= tau), weights split equally
    Ct = np.array([[0.1, 0.7, 0.7, 0.2], [0.0, 0.0, 0.0, 0.0]])
    J, alpha, _ = O.correlated_targets(Ct, 0.998)
    assert J[0].tolist() == [1, 2] and alpha[0].tolist() == [0.5, 0.5]
    assert len(J[1]) == 0                                      # all-zero row: pruned (reading R9)
    J, alpha, _ = O.correlated_targets(np.zeros((2, 0)), 0.998)
    assert len(J[0]) == 0


# ------------------------------------------------------------------ compress (Eq. 2)
def _random_plan(r, N, n_keep):
    s = r.standard_normal(N)
    S, T = O.filter_tokens(s, n_keep)
    C = r.random((len(S), len(T)))
    return S, T, C


def test_compress_zero_discards_is_identity():
    r = rng(12)
    X = r.standard_normal((9, 5))
    out = O.compress(X, 1, np.zeros(0, np.int64), np.arange(8), [], [])
    assert np.array_equal(out, X)
    res = O.v_step(X, softmax_rows(r.standard_normal((2, 9, 9))), cls_index=0, vis_begin=1, N=8,
                   n_keep=8, grid=(1, 2, 4))
    assert np.array_equal(res["X_out"], X) and len(res["S"]) == 0


def test_compress_mass_conservation_and_convexity():
    """sum_j (1+a_j) X'_j = sum_{j in T} X_j + sum_{i in S, J_i != {}} X_i  and the mixing
    weights of every preserved token are >= 0 and sum to 1."""
    r = rng(13)
    N, D, vb = 30, 6, 2
    X = r.standard_normal((vb + N + 3, D))
    for eps in (0.3, 0.9, 0.998):
        S, T, C = _random_plan(r, N, 11)
        C[0] = 0.0                                            # one pruned row
        J, alpha, _ = O.correlated_targets(C, eps)
        out = O.compress(X, vb, S, T, J, alpha)
        assert out.shape == (X.shape[0] - len(S), D)
        a = np.zeros(len(T))
        for i in range(len(S)):
            for jj, w in zip(J[i], alpha[i]):
                a[jj] += w
        lhs = ((1 + a)[:, None] * out[vb:vb + len(T)]).sum(axis=0)
        live = [i for i in range(len(S)) if len(J[i])]
        rhs = X[vb + T].sum(axis=0) + X[vb + S[live]].sum(axis=0)
        assert np.allclose(lhs, rhs, rtol=1e-12, atol=1e-12)
        assert abs((1 + a).sum() - (len(T) + len(live))) < 1e-12
        # pass-through rows are bit-exact, order preserved
        assert np.array_equal(out[:vb], X[:vb]) and np.array_equal(out[vb + len(T):], X[vb + N:])
        # outputs lie inside the per-dimension range of the inputs (convex combination)
        assert np.all(out.max(axis=0) <= X.max(axis=0) + 1e-12)
        assert np.all(out.min(axis=0) >= X.min(axis=0) - 1e-12)


def test_compress_k1_is_pairwise_average():
    """eps = 1 and each target hit by at most one source: X'_j = (X_j + X_i) / 2 (the K = 1,
    ToMe-like case the paper mentions under "Correlate")."""
    X = np.arange(24, dtype=np.float64).reshape(6, 4)
    S, T = np.array([0, 3]), np.array([1, 2, 4, 5])
    C = np.array([[0.1, 0.9, 0.2, 0.3], [0.8, 0.1, 0.1, 0.2]])
    J, alpha, _ = O.correlated_targets(C, 1.0)
    out = O.compress(X, 0, S, T, J, alpha)
    assert np.array_equal(out[1], (X[2] + X[0]) / 2) and np.array_equal(out[0], (X[1] + X[3]) / 2)
    assert np.array_equal(out[2:], X[[4, 5]])
    # two sources on the same target: (X_j + X_a + X_b) / 3, sources added in ascending order
    C2 = np.array([[0.1, 0.9, 0.2, 0.3], [0.1, 0.8, 0.1, 0.2]])
    J, alpha, _ = O.correlated_targets(C2, 1.0)
    out = O.compress(X, 0, S, T, J, alpha)
    assert np.array_equal(out[1], ((X[2] + X[0]) + X[3]) / 3.0)


def test_compress_matches_dense_weight_matrix_form():
    r = rng(14)
    N, D = 14, 5
    X = r.standard_normal((N + 1, D))
    S, T, C = _random_plan(r, N, 6)
    for eps in (0.5, 0.998):
        J, alpha, _ = O.correlated_targets(C, eps)
        out = O.compress(X, 1, S, T, J, alpha)
        W = np.array(BF.dense_weights(C.tolist(), eps))
        ref = (X[1 + T] + W.T @ X[1 + S]) / (1 + W.sum(axis=0))[:, None]
        assert np.allclose(out[1:], ref, rtol=1e-13, atol=1e-14)


# ------------------------------------------------------------------ whole step, brute force on tiny N
def _tiny_v_case(r, n_side, D, H, ties):
    N = n_side * n_side
    n = N + 1
    A = softmax_rows(r.standard_normal((H, n, n)))
    if ties:                                   # duplicate key columns and query rows -> exact ties
        A[:, :, 3] = A[:, :, 2]
        A[:, 3, :] = A[:, 2, :]
        A[:, :, 7] = A[:, :, 5]
        A = A / A.sum(axis=-1, keepdims=True)
        A[:, :, 3] = A[:, :, 2]
        A[:, :, 7] = A[:, :, 5]
    X = r.standard_normal((n, D))
    return X, A


@pytest.mark.parametrize("seed", range(12))
def test_v_step_against_brute_force(seed):
    r = rng(100 + seed)
    n_side = [2, 3, 4][seed % 3]
    N = n_side * n_side
    X, A = _tiny_v_case(r, n_side, 3, 2, ties=(seed % 2 == 1 and n_side >= 3))
    n_keep = int(r.integers(1, N + 1))
    eps = [0.998, 0.5, 1.0, 0.0][seed % 4]
    pos = r.permutation(n_side * n_side + 5)[:N] if seed % 5 == 0 else np.arange(N)
    gh, gw = (n_side, n_side) if seed % 5 else (1, n_side * n_side + 5)
    res = O.v_step(X, A, cls_index=0, vis_begin=1, N=N, n_keep=n_keep, lam=0.35, eps=eps,
                   pos=pos, grid=(1, gh, gw), window=2, coef=2.0)
    P = O.head_mean(A)
    out, S, T, W, s = BF.v_step(X.tolist(), P.tolist(), 0, 1, N, n_keep, 0.35, eps,
                                [int(p) for p in pos], gh, gw, 2, 2.0)
    assert res["S"].tolist() == S and res["T"].tolist() == T
    assert np.allclose(res["scores"], s, rtol=1e-14, atol=0)
    for a in range(len(S)):
        hit = [b for b in range(len(T)) if W[a][b] != 0.0]
        assert res["J"][a].tolist() == hit
        assert np.allclose(res["alpha"][a], [W[a][b] for b in hit], rtol=1e-14)
    assert np.allclose(res["X_out"], np.array(out).reshape(res["X_out"].shape), rtol=1e-13, atol=1e-15)
    assert res["X_out"].shape[0] == X.shape[0] - (N - n_keep)      # Algorithm 1 "Ensure"


@pytest.mark.parametrize("seed", range(8))
def test_l_step_against_brute_force(seed):
    r = rng(200 + seed)
    n_sys, N, M, D, H = 2, 9, 3, 4, 2
    n_tot = n_sys + N + M
    X = r.standard_normal((n_tot, D))
    full = r.standard_normal((H, n_tot, n_tot))
    causal = np.tril(np.ones((n_tot, n_tot), dtype=bool))
    full = np.where(causal, full, -np.inf)
    P = softmax_rows(full)
    A_vv = P[:, n_sys:n_sys + N, n_sys:n_sys + N]
    A_tv = P[:, n_sys + N:, n_sys:n_sys + N]
    n_keep = int(r.integers(1, N + 1))
    eps = [0.998, 0.6][seed % 2]
    res = O.l_step(X, A_vv, A_tv, vis_begin=n_sys, N=N, n_keep=n_keep, beta=0.6, gamma=0.6, eps=eps)
    out, S, T, W, s = BF.l_step(X.tolist(), O.head_mean(A_vv).tolist(), O.head_mean(A_tv).tolist(),
                                n_sys, N, n_keep, 0.6, 0.6, eps)
    assert res["S"].tolist() == S and res["T"].tolist() == T
    assert np.allclose(res["scores"], s, rtol=1e-14)
    for a in range(len(S)):
        hit = [b for b in range(len(T)) if W[a][b] != 0.0]
        assert res["J"][a].tolist() == hit
    assert np.allclose(res["X_out"], np.array(out).reshape(res["X_out"].shape), rtol=1e-13, atol=1e-15)
    assert res["X_out"].shape[0] == n_tot - (N - n_keep)           # Algorithm 2 "Ensure"
    # system and text tokens are untouched
    assert np.array_equal(res["X_out"][:n_sys], X[:n_sys])
    assert np.array_equal(res["X_out"][-M:], X[-M:])


def test_tie_orderings_enumerated():
    """All scores equal: whatever order the tokens come in, the discarded set is the lowest
    indices; permuting the attention columns permutes nothing in the outcome."""
    n = 5
    X = np.arange(6 * 2, dtype=np.float64).reshape(6, 2)
    A = np.full((1, 6, 6), 1.0 / 6)
    for perm in itertools.permutations(range(n)):
        pos = np.array(perm)
        res = O.v_step(X, A, cls_index=0, vis_begin=1, N=n, n_keep=2, pos=pos, grid=(1, 1, 5),
                       window=0)
        assert res["S"].tolist() == [0, 1, 2] and res["T"].tolist() == [3, 4]
        assert res["pos_out"].tolist() == [perm[3], perm[4]]


def test_v_step_modes_vector_and_cosine():
    """Config-4 style inputs: pre-reduced vectors + cosine correlation; the step must equal
    the same step fed an attention map whose column statistics are those vectors."""
    r = rng(15)
    N, D, H = 16, 8, 2
    X = r.standard_normal((N, D))
    recv = r.random((H, N))
    sem = r.random((H, N))
    res = O.v_step(X, None, cls_index=-1, vis_begin=0, N=N, n_keep=6, recv_vec=recv, sem_vec=sem,
                   red_src="vector", sem_src="vector", corr_src="cosine", grid=(1, 4, 4))
    lam = float(np.float32(0.35))
    s = lam * recv.mean(axis=0) - (1 - lam) * sem.mean(axis=0)
    s = O.local_penalty(s, np.arange(N), 1, 4, 4, 2, 2.0)
    assert np.allclose(res["scores"], s, rtol=1e-14)
    S, T = res["S"], res["T"]
    assert np.array_equal(res["C"], O.correlation_cosine(X, S, T))
    assert res["X_out"].shape == (6, D)


# ------------------------------------------------------------------ ablation variants (readings R11-R14)
def test_fixed_k_closed_forms():
    C = np.array([[0.1, 0.7, 0.7, 0.2],      # tie at the top: positions 1 and 2
                  [0.0, 0.0, 0.0, 0.0],      # nothing to recycle (R9)
                  [0.5, 0.25, 0.125, 0.125]])
    J0, a0 = O.fixed_k_targets(C, 0)
    assert all(len(j) == 0 for j in J0)                                   # K = 0 is pruning
    J1, a1 = O.fixed_k_targets(C, 1)
    assert J1[0].tolist() == [1] and a1[0].tolist() == [1.0]              # tie -> lower position
    assert len(J1[1]) == 0
    assert J1[2].tolist() == [0]
    J2, a2 = O.fixed_k_targets(C, 2)
    assert J2[0].tolist() == [1, 2] and np.allclose(a2[0], [0.5, 0.5])
    assert J2[2].tolist() == [0, 1] and np.allclose(a2[2], [2 / 3, 1 / 3])
    J3, a3 = O.fixed_k_targets(C, 3)
    assert J3[2].tolist() == [0, 1, 2]                                    # tie at the cut: lower position
    J9, a9 = O.fixed_k_targets(C, 9)
    assert J9[2].tolist() == [0, 1, 2, 3] and abs(a9[2].sum() - 1.0) < 1e-15


def test_fixed_k1_is_argmax_and_gap_matches_sorted_row():
    r = rng(77)
    C = r.random((9, 6))
    J, a = O.fixed_k_targets(C, 1)
    assert [int(j[0]) for j in J] == np.argmax(C, axis=1).tolist()
    srt = np.sort(C, axis=1)
    assert np.array_equal(O.correlation_gap(C), srt[:, -1] - srt[:, -2])
    C[0, :] = 0.25
    assert O.correlation_gap(C)[0] == 0.0                                 # tie at the top
    assert O.correlation_gap(np.ones((3, 1))).tolist() == [0.0, 0.0, 0.0]  # fewer than two preserved tokens


def test_average_compression_closed_form():
    r = rng(78)
    X = r.standard_normal((6, 4))
    S, T = np.array([1, 3, 4]), np.array([0, 2, 5])
    J = [np.array([0]), np.array([0, 2]), np.array([], dtype=np.int64)]
    alpha = [np.array([1.0]), np.array([0.9, 0.1]), np.array([])]
    out = O.compress(X, 0, S, T, J, alpha, average=True)
    assert np.allclose(out[0], (X[0] + X[1] + X[3]) / 3.0, rtol=1e-15)    # two sources, weights ignored
    assert np.array_equal(out[1], X[2])                                   # no source
    assert np.allclose(out[2], (X[5] + X[3]) / 2.0, rtol=1e-15)
    ref = O.compress(X, 0, S, T, J, alpha)
    assert np.allclose(ref[0], (X[0] + X[1] + 0.9 * X[3]) / 2.9, rtol=1e-15)


def test_convergent_token_and_layout():
    r = rng(79)
    X = r.standard_normal((9, 3))            # 2 leading + 5 visual + 2 trailing tokens
    S, T = np.array([0, 3]), np.array([1, 2, 4])
    none = [np.zeros(0, np.int64)] * 2
    extra = O.convergent_token(X, 2, S)
    assert np.allclose(extra, X[[2, 5]].mean(axis=0), rtol=1e-15)
    out = O.compress(X, 2, S, T, none, [np.zeros(0)] * 2, extra=extra)
    assert out.shape == (8, 3)                                            # N^S rows leave, one comes
    assert np.array_equal(out[[0, 1, 2, 3, 4, 6, 7]], X[[0, 1, 3, 4, 6, 7, 8]])
    assert np.array_equal(out[5], extra)                                  # directly behind the last preserved visual token


@pytest.mark.parametrize("seed", range(9))
def test_v_step_ablations_against_brute_force(seed):
    r = rng(300 + seed)
    n_side = [3, 4, 2][seed % 3]
    N = n_side * n_side
    X, A = _tiny_v_case(r, n_side, 3, 2, ties=(seed % 2 == 1 and n_side >= 3))
    n_keep = int(r.integers(1, N + 1))
    mode = ["fixed0", "fixed1", "fixed2", "average", "convergent"][seed % 5]
    kw = dict(fixed0=dict(k_mode="fixed", fixed_k=0), fixed1=dict(k_mode="fixed", fixed_k=1),
              fixed2=dict(k_mode="fixed", fixed_k=2), average=dict(average=True),
              convergent=dict(k_mode="convergent"))[mode]
    res = O.v_step(X, A, cls_index=0, vis_begin=1, N=N, n_keep=n_keep, lam=0.35, eps=0.5,
                   grid=(1, n_side, n_side), window=2, coef=2.0, **kw)
    P = O.head_mean(A)
    bkw = dict(fixed0=dict(fixed_k=0), fixed1=dict(fixed_k=1), fixed2=dict(fixed_k=2),
               average=dict(average=True), convergent=dict(convergent=True))[mode]
    out, S, T, W, s = BF.v_step(X.tolist(), P.tolist(), 0, 1, N, n_keep, 0.35, 0.5,
                                list(range(N)), n_side, n_side, 2, 2.0, **bkw)
    assert res["S"].tolist() == S and res["T"].tolist() == T
    if mode.startswith("fixed"):
        for a in range(len(S)):
            hit = [b for b in range(len(T)) if W[a][b] != 0.0]
            assert res["J"][a].tolist() == hit
            assert np.allclose(res["alpha"][a], [W[a][b] for b in hit], rtol=1e-14)
    n_rows = X.shape[0] - (N - n_keep) + (1 if mode == "convergent" and n_keep < N else 0)
    assert res["X_out"].shape[0] == n_rows
    assert np.allclose(res["X_out"], np.array(out).reshape(res["X_out"].shape), rtol=1e-13, atol=1e-15)
    if mode == "fixed0":                     # pruning: the preserved tokens are untouched
        keep_rows = [0] + [1 + j for j in T]
        assert np.array_equal(res["X_out"], X[keep_rows])


def test_gather_tokens_layout():
    t = np.arange(9 * 2).reshape(9, 2)       # 2 leading + 5 visual + 2 trailing tokens
    out = O.gather_tokens(t, 2, 5, np.array([1, 2, 4]))
    assert out[:, 0].tolist() == [0, 2, 6, 8, 12, 14, 16]     # rows 0 1 | 3 4 6 | 7 8
    assert O.gather_tokens(t, 2, 5, np.arange(5)).shape == (9, 2)
    ids = np.arange(9)
    assert O.gather_tokens(ids, 0, 9, np.array([0, 8])).tolist() == [0, 8]
