"""FiCoCo filter / correlate / compress step -- plain CPU oracle (TEST INFRASTRUCTURE).

This module is the checker, not the product.  It states, in slow and obvious float64
numpy, what one FiCoCo token-reduction step computes, following the paper
"Filter, Correlate, Compress" (arxiv 2411.17686): Algorithm 1 (FiCoCo-V),
Algorithm 2 (FiCoCo-L), Eq. 1 (integrated redundancy score), Eq. 2 (self-preserving
compression), Eq. 3 (FiCoCo-L score), Eq. 4 (FiCoCo-L correlation) and the appendix
section "Implementation of the Equivalent Token".

Only tests, the smoke check and the benchmark's CPU-baseline leg may import it.  It shares
no code with the HIP library and never calls it.  There is no blocking, fusion or
reordering here beyond what the definitions state.

Index convention (the paper's own is not self-consistent, see "readings" below).
`P[q, k]` is the usual row-stochastic attention map, row = query, column = key.  The
paper's A_{i,j} for visual token i is read as the attention token i RECEIVES from token j,
i.e. P[j, i]: Sec. "Redundancy-based Token Discard" describes the first score term as the
attention the token receives and the appendix section on the sign of vision-aware redundancy
as its incoming attention; a literal row sum of a softmax is the constant 1 and could not
rank anything.

Readings (where the paper is silent, ambiguous or garbled):
  R1  multi-head maps are reduced to one map by the head mean, heads added in order.
  R2  first score term = column mean over the N visual query rows (diagonal included).
  R3  second score term = the [CLS] query row (V) / mean over the M text query rows (L);
      Eq. 3 keeps the 1/M that Algorithm 2 drops.
  R4  local penalty: 2-D grid of cells, -inf padding for absent cells, non-overlapping
      W x W windows anchored at (0,0) of each sub-grid; the maximum of a window (ties: the
      lowest cell index) is multiplied by the coefficient, whatever its sign.
  R5  filter: discard the N^S largest by (score descending, index ascending).
  R6  V correlation C[i, j] = head-mean attention P[j, i] (preserved query j on discarded
      key i), read from the map materialised in single precision.
  R7  L indirect term = (1/M) sum_k P[k, i] P[k, j] over text queries k (co-attention of
      the two visual tokens by the text); Eq. 4 keeps the 1/M that Algorithm 2 drops.
  R8  the epsilon-quantile is the linear-interpolation order statistic
      v[f] + g (v[f+1] - v[f]),  p = eps (n-1), f = floor(p), g = p - f.
  R9  a row whose selected correlations sum to <= 0 recycles nothing (pure pruning).
  R10 extension (not in the paper): cosine correlation max(0, xh_i . xh_j) with the
      normalised rows xh rounded to bfloat16, and the mean-cosine first score term.
  R11 ablation "fixed K" (ablation tables, rows "fixed K=0/1/2"; Sec. "Correlation-based
      Information Recycling"): J_i = the K preserved tokens with the largest C_ij, ties to
      the lower position; weights as in Eq. 2; K = 0 is pruning.
  R12 ablation "convergent correlation" (same tables; the sentence on merging all discarded
      tokens into an additional token): the preserved tokens stay as they are and ONE extra
      token, the plain mean of the discarded tokens (added in ascending index), is placed
      directly behind the last preserved visual token.  The paper gives no weights for it.
  R13 ablation "average compression" (same tables; Sec. "Compress"): a preserved token is
      averaged with the discarded tokens correlated to it, all with weight one; the
      correlated sets are still those of the adaptive threshold.
  R14 "pairwise token correlation gap" (same section): top-1 minus top-2 value of a row of C,
      counted with multiplicity (a tie at the top gives 0); a row with fewer than two
      preserved tokens has gap 0.

  R16 queries and keys instead of the map (Sec. "Self-Attention", A = Softmax(Q K^T / sqrt(D))):
      the map of every head is the row softmax of that head's logits over all keys of the block,
      unmasked; it is used unrounded (the caller's model would have stored it in its own
      precision, which the step never sees in this form).  Everything after it is unchanged.

  R15 schedule utility (appendix "Theoretical FLOPs Calculation", Sec. "Implementation
      Details"): a layer over n visual tokens costs 4 p D^2 + 2 p^2 D + 2 p D F with p = n (V)
      or n + M (L); a reducing layer is charged with its tokens AFTER the reduction plus the
      method's own work; every layer from the start layer on discards the same count, never
      below a minimum; the schedule is the smallest such count within the budget.  The
      appendix's printed differences (Delta) do not equal before - after as printed (the
      vision form lacks a factor 2 on N N^S, the decoder form drops M); the before / after
      expressions are followed.

All decisions (window maxima, the top-K filter, the threshold test) are taken on float64
values; scalar hyper-parameters cross the library boundary as float32 and are widened
from that value here too.
"""
import math

import numpy as np

F64 = np.float64


# --------------------------------------------------------------------------- input decoding
def widen(buf):
    """Exact float64 view of an input buffer: float32 array, or bfloat16 bits as uint16."""
    buf = np.asarray(buf)
    if buf.dtype == np.uint16:
        return (buf.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(F64)
    if buf.dtype in (np.float32, np.float64):
        return buf.astype(F64)
    raise TypeError("expected float32 values or bfloat16 bit patterns (uint16)")


def f32(x):
    """The float64 value of a scalar that crossed the boundary as float32."""
    return float(np.float32(x))


def round_to_bf16(x):
    """Round float64 values to the nearest bfloat16 (ties to even); result kept as float64.

    bfloat16 has 8 significant bits and float32's exponent range, so the spacing at a value
    with binary exponent e is 2^(max(e, -126) - 7).
    """
    x = np.asarray(x, dtype=F64)
    _, e = np.frexp(x)                     # x = m * 2^e with 0.5 <= |m| < 1  ->  exponent e-1
    q = np.ldexp(1.0, np.maximum(e - 1, -126) - 7)
    return np.where(x == 0.0, 0.0, np.rint(x / q) * q)


def round_to_dtype(x, dtype):
    """Round a float64 array to the storage type of the tokens ('f32' or 'bf16')."""
    if dtype == "f32":
        return np.asarray(x, dtype=F64).astype(np.float32).astype(F64)
    if dtype == "bf16":
        return round_to_bf16(x)
    raise ValueError(dtype)


# --------------------------------------------------------------------------- self-attention
def attention_from_qk(Q, K, scale, causal=False):
    """Sec. "Self-Attention": A = Softmax(Q K^T / sqrt(D)) per head, for a caller that hands over
    the projected queries and keys instead of the map.  Q [H, nq, d], K [H, nk, d] float64;
    `scale` (the 1/sqrt(D) of the equation) crosses the boundary as float32.  Returns [H, nq, nk]:
    every row a softmax over all nk keys (no mask: the vision encoder attends everywhere), or,
    with causal=True (the decoder of FiCoCo-L; nq == nk, row r is sequence position r), over
    keys 0 .. r only, the others exactly 0.  The logits are a float64 matrix product, the
    exponentials are taken relative to the row maximum and the row is divided by its sum, keys
    added in order."""
    Q = np.asarray(Q, dtype=F64)
    K = np.asarray(K, dtype=F64)
    sc = f32(scale)
    A = np.empty((Q.shape[0], Q.shape[1], K.shape[1]), dtype=F64)
    later = np.triu(np.ones((Q.shape[1], K.shape[1]), dtype=bool), 1) if causal else None
    for h in range(Q.shape[0]):
        logits = (Q[h] @ K[h].T) * sc
        if causal:
            logits = np.where(later, -np.inf, logits)
        e = np.exp(logits - logits.max(axis=1, keepdims=True))
        den = np.zeros(e.shape[0], dtype=F64)
        for k in range(e.shape[1]):
            den = den + e[:, k]
        A[h] = e / den[:, None]
    return A


# --------------------------------------------------------------------------- filter: score
def head_mean(A):
    """Reading R1: (1/H) sum_h A[h], heads added in order.  A: [H, Nq, Nk] float64."""
    A = np.asarray(A, dtype=F64)
    acc = np.zeros(A.shape[1:], dtype=F64)
    for h in range(A.shape[0]):
        acc = acc + A[h]
    return acc * (1.0 / A.shape[0])


def received_attention(P, query_rows, key_cols):
    """First term of Eq. 1 / Eq. 3 (reading R2): for each visual token (a key column) the
    mean over the visual query rows of the attention it receives; rows added in order,
    divided by the number of visual tokens N = len(key_cols)."""
    acc = np.zeros(len(key_cols), dtype=F64)
    for q in query_rows:
        acc = acc + P[q, key_cols]
    return acc / float(len(key_cols))


def cls_attention(P, cls_row, key_cols):
    """Semantic term of Eq. 1: the [CLS] query's attention weight on each patch."""
    return P[cls_row, key_cols].astype(F64)


def text_attention(P, text_rows, key_cols):
    """Task term of Eq. 3 (reading R3): mean over the M text queries of the attention each
    visual token receives from them."""
    acc = np.zeros(len(key_cols), dtype=F64)
    for k in text_rows:
        acc = acc + P[k, key_cols]
    return acc / float(len(text_rows))


def head_mean_vector(V):
    """Pre-reduced per-head score vectors [H, N] -> head mean [N], heads added in order."""
    V = np.asarray(V, dtype=F64)
    acc = np.zeros(V.shape[1], dtype=F64)
    for h in range(V.shape[0]):
        acc = acc + V[h]
    return acc * (1.0 / V.shape[0])


def l2_norms(F):
    """Euclidean norm of each row, squares added in order along the feature axis."""
    F = np.asarray(F, dtype=F64)
    acc = np.zeros(F.shape[0], dtype=F64)
    for d in range(F.shape[1]):
        acc = acc + F[:, d] * F[:, d]
    return np.sqrt(acc)


def unit_rows(F):
    """Rows divided by their Euclidean norm; a zero row stays zero (its cosines are 0)."""
    F = np.asarray(F, dtype=F64)
    nrm = l2_norms(F)
    safe = np.where(nrm > 0.0, nrm, 1.0)
    return np.where(nrm[:, None] > 0.0, F / safe[:, None], 0.0)


def equivalent_token_term(F):
    """Appendix "Implementation of the Equivalent Token": mu = mean of the patch features
    (the caller supplies head-mean keys), a_i^Eq = -cos(mu, F_i).  Replaces a^CLS in Eq. 1.
    Every sum runs in index order (tokens for mu, features for the dot product and the norms),
    products and sums rounded separately, so the value is one definite float64."""
    F = np.asarray(F, dtype=F64)
    mu = np.zeros(F.shape[1], dtype=F64)
    for i in range(F.shape[0]):
        mu = mu + F[i]
    mu = mu / float(F.shape[0])
    mm = 0.0
    for d in range(F.shape[1]):
        mm = mm + float(mu[d]) * float(mu[d])
    mu_n = math.sqrt(mm)
    nrm = l2_norms(F)
    dots = np.zeros(F.shape[0], dtype=F64)
    for d in range(F.shape[1]):
        dots = dots + mu[d] * F[:, d]
    out = np.zeros(F.shape[0], dtype=F64)
    for i in range(F.shape[0]):
        if mu_n > 0.0 and nrm[i] > 0.0:
            out[i] = -(dots[i] / (mu_n * nrm[i]))
    return out


def cosine_matrix(F):
    """cos(F_i, F_j) for all pairs: the dot product of the two unit rows, features added in
    order, products and sums rounded separately.  (Rows are taken 32 at a time only so that the
    running sums stay in the CPU's cache; every entry is the same in-order sum either way.)"""
    U = unit_rows(F)
    n = U.shape[0]
    Ut = np.ascontiguousarray(U.T)                  # Ut[d] = feature d of every unit row
    G = np.zeros((n, n), dtype=F64)
    for i0 in range(0, n, 32):
        Ub = np.ascontiguousarray(U[i0:i0 + 32].T)  # Ub[d] = feature d of these rows
        acc = np.zeros((Ub.shape[1], n), dtype=F64)
        prod = np.empty_like(acc)
        for d in range(U.shape[1]):
            np.multiply(Ub[d][:, None], Ut[d][None, :], out=prod)
            acc += prod
        G[i0:i0 + 32] = acc
    return G


def mean_cosine_term(F):
    """Reading R10 (extension): (1/N) sum_j cos(F_i, F_j), j = i included -- the plain
    definition through the full cosine matrix, the cosines of a token added in order of j."""
    G = cosine_matrix(F)
    acc = np.zeros(G.shape[0], dtype=F64)
    for j in range(G.shape[1]):
        acc = acc + G[:, j]
    return acc / float(G.shape[0])


def combine_score(R, G, w):
    """Eq. 1 (w = lambda) and Eq. 3 (w = beta):  s = w R - (1 - w) G."""
    w = f32(w)
    return w * np.asarray(R, F64) - (1.0 - w) * np.asarray(G, F64)


def local_penalty(s, pos, grid_g, grid_h, grid_w, window, coef):
    """Local penalty of Sec. "Redundancy-based Token Discard" (reading R4).

    s[t] is the score of visual token t, pos[t] its cell in `grid_g` stacked grid_h x grid_w
    grids (row-major).  Cells of tokens discarded by earlier steps are padding.  In every
    non-overlapping window that holds at least one token the largest score (first in cell
    order on ties) is multiplied by `coef`.  window <= 0 switches the penalty off."""
    s = np.asarray(s, dtype=F64)
    out = s.copy()
    if window <= 0:
        return out
    coef = f32(coef)
    cells = grid_g * grid_h * grid_w
    owner = np.full(cells, -1, dtype=np.int64)
    for t in range(len(s)):
        assert 0 <= pos[t] < cells and owner[pos[t]] < 0, "pos must be distinct grid cells"
        owner[pos[t]] = t
    for sub in range(grid_g):
        for r0 in range(0, grid_h, window):
            for c0 in range(0, grid_w, window):
                best = -1
                for r in range(r0, min(r0 + window, grid_h)):
                    for c in range(c0, min(c0 + window, grid_w)):
                        t = owner[(sub * grid_h + r) * grid_w + c]
                        if t >= 0 and (best < 0 or s[t] > s[best]):
                            best = t
                if best >= 0:
                    out[best] = coef * s[best]
    return out


# --------------------------------------------------------------------------- filter: top-K
def filter_tokens(s, n_keep):
    """Stage 1 of Algorithms 1 and 2 (reading R5): the N^S = N - n_keep tokens with the
    highest redundancy form the source set S, the rest the target set T.  Both are returned
    in ascending index order."""
    s = np.asarray(s, dtype=F64)
    assert np.all(np.isfinite(s)), "scores must be finite"
    n = len(s)
    n_s = n - n_keep
    assert 0 <= n_s <= n
    order = sorted(range(n), key=lambda i: (-s[i], i))
    S = np.array(sorted(order[:n_s]), dtype=np.int64)
    T = np.array(sorted(order[n_s:]), dtype=np.int64)
    return S, T


# --------------------------------------------------------------------------- correlate
def materialise_f32(P):
    """The head-mean map as the step stores it between its two passes: single precision."""
    return np.asarray(P, dtype=F64).astype(np.float32).astype(F64)


def correlation_attention(P32, S, T, key_cols, query_rows):
    """Stage 2 of Algorithm 1 (reading R6): C[i, j] = P[query j in T, key i in S].
    key_cols / query_rows map a visual token index to its column / row of P32."""
    S = np.asarray(S, dtype=np.int64)
    T = np.asarray(T, dtype=np.int64)
    rows = np.asarray(query_rows)[T]
    cols = np.asarray(key_cols)[S]
    return P32[np.ix_(rows, cols)].T.astype(F64)       # a pure gather: C[a, b] = P32[rows[b], cols[a]]


def text_bridge(Ptext, S, T):
    """Indirect term of Eq. 4 (reading R7).  Ptext: [M, N] head-mean attention of the M text
    queries on the N visual tokens.  B[i, j] = (1/M) sum_k Ptext[k, i] Ptext[k, j], text
    tokens added in order."""
    M = Ptext.shape[0]
    Bm = np.zeros((len(S), len(T)), dtype=F64)
    for k in range(M):
        Bm = Bm + np.outer(Ptext[k, S], Ptext[k, T])
    return Bm / float(M)


def correlation_cosine(F, S, T):
    """Reading R10 (extension): unit rows rounded to bfloat16, C[i, j] = max(0, xh_i . xh_j)
    (a float64 matrix product of the rounded rows)."""
    Uh = round_to_bf16(unit_rows(F))
    C = Uh[np.asarray(S, dtype=np.int64)] @ Uh[np.asarray(T, dtype=np.int64)].T
    return np.maximum(C, 0.0)


def correlation_l(direct, bridge, gamma):
    """Eq. 4:  C = gamma * direct + (1 - gamma) * indirect."""
    g = f32(gamma)
    return g * direct + (1.0 - g) * bridge


# --------------------------------------------------------------------------- compress
def quantile_threshold(row, eps):
    """tau = epsilon-quantile of one row of C (Algorithm 1, stage 3; reading R8)."""
    v = np.sort(np.asarray(row, dtype=F64))
    n = len(v)
    p = f32(eps) * float(n - 1)
    f = int(math.floor(p))
    g = p - float(f)
    f1 = min(f + 1, n - 1)
    return v[f] + g * (v[f1] - v[f])


def correlated_targets(C, eps):
    """Token-adaptive K (Sec. "Correlation-based Information Recycling") and the weights of
    Eq. 2.  Returns, per discarded row i: J_i (positions in T, ascending) and alpha_i."""
    J, alpha, tau = [], [], []
    for i in range(C.shape[0]):
        if C.shape[1] == 0:
            J.append(np.zeros(0, np.int64)); alpha.append(np.zeros(0, F64)); tau.append(0.0)
            continue
        t = quantile_threshold(C[i], eps)
        sel = np.nonzero(C[i] >= t)[0]
        d = 0.0
        for j in sel:
            d = d + C[i, j]
        if d > 0.0:
            J.append(sel.astype(np.int64))
            alpha.append(np.array([C[i, j] / d for j in sel], dtype=F64))
        else:                                       # reading R9
            J.append(np.zeros(0, np.int64))
            alpha.append(np.zeros(0, F64))
        tau.append(t)
    return J, alpha, np.array(tau, dtype=F64)


def fixed_k_targets(C, K):
    """Ablation "fixed K" (reading R11): per discarded row the K preserved tokens with the
    largest correlation, ties to the lower position; weights alpha as in Eq. 2."""
    J, alpha = [], []
    for i in range(C.shape[0]):
        order = sorted(range(C.shape[1]), key=lambda j: (-C[i, j], j))
        sel = np.array(sorted(order[:max(int(K), 0)]), dtype=np.int64)
        d = 0.0
        for j in sel:
            d = d + C[i, j]
        if len(sel) and d > 0.0:
            J.append(sel)
            alpha.append(np.array([C[i, j] / d for j in sel], dtype=F64))
        else:                                       # reading R9
            J.append(np.zeros(0, np.int64))
            alpha.append(np.zeros(0, F64))
    return J, alpha


def correlation_gap(C):
    """Pairwise token correlation gap of every discarded row (reading R14)."""
    gap = np.zeros(C.shape[0], dtype=F64)
    for i in range(C.shape[0]):
        if C.shape[1] >= 2:
            v = np.sort(np.asarray(C[i], dtype=F64))
            gap[i] = v[-1] - v[-2]
    return gap


def convergent_token(X, vis_begin, S):
    """The additional token of the "convergent" ablation (reading R12)."""
    X = np.asarray(X, dtype=F64)
    acc = np.zeros(X.shape[1], dtype=F64)
    for i in S:
        acc = acc + X[vis_begin + int(i)]
    return acc / float(len(S))


def compress(X, vis_begin, S, T, J, alpha, average=False, extra=None):
    """Eq. 2 and the last stage of Algorithms 1 and 2.

    X: [n_tot, D] float64 tokens of the whole sequence; S, T index the visual span that
    starts at vis_begin.  Every preserved visual token j becomes
        (X_j + sum_{i in I_j} alpha_ij X_i) / (1 + sum_{i in I_j} alpha_ij),
    sources added in ascending order of i; the discarded tokens are then removed and all
    other tokens of the sequence keep their order.
    average=True: every weight is one (ablation "average compression", reading R13).
    extra: a row placed directly behind the last preserved visual token (the additional
    token of the "convergent" ablation, reading R12)."""
    X = np.asarray(X, dtype=F64)
    num = {int(j): X[vis_begin + int(j)].copy() for j in T}
    den = {int(j): 1.0 for j in T}
    for a, i in enumerate(S):                       # S ascending -> ascending i per target
        for jj, w in zip(J[a], alpha[a]):
            j = int(T[jj])
            if average:
                w = 1.0
            num[j] = num[j] + w * X[vis_begin + int(i)]
            den[j] = den[j] + w
    gone = set(vis_begin + int(i) for i in S)
    last_kept = vis_begin + int(max(T)) if len(T) else None
    rows = []
    if extra is not None and last_kept is None:     # no preserved visual token: the extra one opens the span
        for t in range(vis_begin):
            rows.append(X[t].copy())
        rows.append(np.asarray(extra, dtype=F64).copy())
        for t in range(vis_begin, X.shape[0]):
            if t not in gone:
                rows.append(X[t].copy())
        return np.array(rows, dtype=F64).reshape(len(rows), X.shape[1])
    for t in range(X.shape[0]):
        if t in gone:
            continue
        j = t - vis_begin
        if j in num:
            rows.append(num[j] / den[j])
        else:
            rows.append(X[t].copy())
        if extra is not None and t == last_kept:
            rows.append(np.asarray(extra, dtype=F64).copy())
    return np.array(rows, dtype=F64).reshape(len(rows), X.shape[1])


# --------------------------------------------------------------------------- whole steps
def _finish(X, vis_begin, s, n_keep, C_of, eps, pos, k_mode="adaptive", fixed_k=1, average=False):
    """k_mode: 'adaptive' (the method), 'fixed' (top-fixed_k per row) or 'convergent'."""
    S, T = filter_tokens(s, n_keep)
    C = C_of(S, T)
    tau = None
    extra = None
    if k_mode == "adaptive":
        J, alpha, tau = correlated_targets(C, eps)
    elif k_mode == "fixed":
        J, alpha = fixed_k_targets(C, fixed_k)
    elif k_mode == "convergent":
        J = [np.zeros(0, np.int64) for _ in S]
        alpha = [np.zeros(0, F64) for _ in S]
        extra = convergent_token(X, vis_begin, S) if len(S) else None
    else:
        raise ValueError(k_mode)
    X_out = compress(X, vis_begin, S, T, J, alpha, average=average, extra=extra)
    pos_out = None if pos is None else np.asarray(pos)[T]
    return dict(X_out=X_out, S=S, T=T, J=J, alpha=alpha, tau=tau, scores=s, C=C,
                pos_out=pos_out, gap=correlation_gap(C))


def v_step(X, A, *, cls_index, vis_begin, N, n_keep, lam=0.35, eps=0.998,
           pos=None, grid=(1, 0, 0), window=2, coef=2.0,
           recv_vec=None, sem_vec=None, F=None,
           red_src="attn", sem_src="cls", corr_src="attn",
           k_mode="adaptive", fixed_k=1, average=False):
    """Algorithm 1 for one image.

    X [n_tot, D]; A [H, n_tot, n_tot] or None; visual span [vis_begin, vis_begin+N).
    red_src: 'attn' | 'vector' | 'sim_mean';  sem_src: 'cls' | 'vector' | 'eq_token';
    corr_src: 'attn' | 'cosine'.  F: features for the cosine-based terms (default: the
    visual rows of X).  k_mode / fixed_k / average: the ablation variants (R11-R13)."""
    X = np.asarray(X, dtype=F64)
    vis = np.arange(vis_begin, vis_begin + N)
    Fv = X[vis] if F is None else np.asarray(F, dtype=F64)
    P = head_mean(A) if A is not None else None
    if red_src == "attn":
        R = received_attention(P, vis, vis)
    elif red_src == "vector":
        R = head_mean_vector(recv_vec)
    elif red_src == "sim_mean":
        R = mean_cosine_term(Fv)
    else:
        raise ValueError(red_src)
    if sem_src == "cls":
        G = cls_attention(P, cls_index, vis)
    elif sem_src == "vector":
        G = head_mean_vector(sem_vec)
    elif sem_src == "eq_token":
        G = equivalent_token_term(Fv)
    else:
        raise ValueError(sem_src)
    s = combine_score(R, G, lam)
    if pos is None:
        pos = np.arange(N)
    s = local_penalty(s, pos, grid[0], grid[1], grid[2], window, coef)
    if corr_src == "attn":
        P32 = materialise_f32(P)
        C_of = lambda S, T: correlation_attention(P32, S, T, vis, vis)
    elif corr_src == "cosine":
        C_of = lambda S, T: correlation_cosine(Fv, S, T)
    else:
        raise ValueError(corr_src)
    return _finish(X, vis_begin, s, n_keep, C_of, eps, pos, k_mode, fixed_k, average)


def v_step_qk(X, Q, K, scale, **kw):
    """Algorithm 1 for a caller that supplies the layer's projected queries and keys
    (Q, K: [H, n_tot, d]) instead of the attention map (reading R16)."""
    return v_step(X, attention_from_qk(Q, K, scale), **kw)


def l_step(X, A_vv, A_tv, *, vis_begin, N, n_keep, beta=0.6, gamma=0.6, eps=0.998,
           F=None, red_src="attn", corr_src="attn", k_mode="adaptive", fixed_k=1, average=False):
    """Algorithm 2 for one sequence.

    X [n_tot, D] (system + visual + text tokens); A_tv [H, M, N]: attention of the M text
    queries on the N visual keys; A_vv [H, N, N]: attention among the visual tokens (None
    when the caller has no such map -- then red_src='sim_mean' and corr_src='cosine', the
    extension of reading R10, stand in for it).  No local penalty in FiCoCo-L."""
    X = np.asarray(X, dtype=F64)
    vis = np.arange(vis_begin, vis_begin + N)
    loc = np.arange(N)
    Fv = X[vis] if F is None else np.asarray(F, dtype=F64)
    Pt = head_mean(A_tv)
    Pv = head_mean(A_vv) if A_vv is not None else None
    if red_src == "attn":
        R = received_attention(Pv, loc, loc)
    elif red_src == "sim_mean":
        R = mean_cosine_term(Fv)
    else:
        raise ValueError(red_src)
    G = text_attention(Pt, np.arange(Pt.shape[0]), loc)
    s = combine_score(R, G, beta)
    if corr_src == "attn":
        P32 = materialise_f32(Pv)
        direct = lambda S, T: correlation_attention(P32, S, T, loc, loc)
    elif corr_src == "cosine":
        direct = lambda S, T: correlation_cosine(Fv, S, T)
    else:
        raise ValueError(corr_src)
    C_of = lambda S, T: correlation_l(direct(S, T), text_bridge(Pt, S, T), gamma)
    return _finish(X, vis_begin, s, n_keep, C_of, eps, None, k_mode, fixed_k, average)


def l_step_qk(X, Q, K, scale, *, vis_begin, N, M, **kw):
    """Algorithm 2 for a caller that supplies the decoder layer's projected queries and keys
    (Q, K: [H, n_tot, d], causal attention) instead of the maps: the M text tokens follow the
    visual span, A_tv is their attention on the visual keys and A_vv the visual block of the
    same maps (reading R16)."""
    A = attention_from_qk(Q, K, scale, causal=True)
    vis = slice(vis_begin, vis_begin + N)
    txt = slice(vis_begin + N, vis_begin + N + M)
    return l_step(X, A[:, vis, vis], A[:, txt, vis], vis_begin=vis_begin, N=N, **kw)


def gather_tokens(t, vis_begin, N, T):
    """Rows of another per-token tensor of the sequence (key / value cache, position ids) that
    remain after the step: the sequence in order without the discarded visual tokens
    (Algorithm 2 removes them from what the following layers see)."""
    t = np.asarray(t)
    keep = set(vis_begin + int(j) for j in T)
    rows = [r for r in range(t.shape[0]) if not (vis_begin <= r < vis_begin + N) or r in keep]
    return t[rows]


# --------------------------------------------------------------------------- FLOPs model (reading R15)
def layer_flops(tokens, D, F):
    """Appendix "Theoretical FLOPs Calculation": one transformer layer over `tokens` tokens."""
    t = float(tokens)
    return 4.0 * t * D * D + 2.0 * t * t * D + 2.0 * t * D * F


def step_flops(variant, n, s, D):
    """The method's own work in a layer that reduces n visual tokens by s (same appendix)."""
    n, s = float(n), float(s)
    first = n * n + 2.0 * n
    if variant == "L":
        first = 2.0 * first
    return first + s * ((n - s) + 2.0 * D + 1.0) + D


def schedule_cost(variant, layers, start_layer, N, M, D, F, min_keep, s):
    """Total cost and per-layer discard counts when every layer from start_layer on discards s."""
    n = N
    total = 0.0
    drops = []
    for l in range(layers):
        drop = 0
        if l >= start_layer:
            drop = s if n - s >= min_keep else n - min_keep
            drop = max(drop, 0)
        if drop > 0:
            total += step_flops(variant, n, drop, D)
        n -= drop
        total += layer_flops(n + (M if variant == "L" else 0), D, F)
        drops.append(drop)
    return total, drops


def schedule_uniform(variant, layers, start_layer, N, M, D, F, min_keep, budget):
    """Smallest uniform per-layer discard count within the budget (counts tried in ascending
    order).  Returns (reachable, drops, total)."""
    for s in range(0, N - min_keep + 1):
        total, drops = schedule_cost(variant, layers, start_layer, N, M, D, F, min_keep, s)
        if total <= budget:
            return True, drops, total
    total, drops = schedule_cost(variant, layers, start_layer, N, M, D, F, min_keep, N - min_keep)
    return False, drops, total
