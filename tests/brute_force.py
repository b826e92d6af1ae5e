"""Independent brute-force statement of the FiCoCo step for tiny inputs (N <= 16).

Written separately from `oracle/`: plain Python floats and lists, repeated arg-max instead
of a sort for the filter, a library quantile routine for the threshold, and the dense
weight-matrix form  X' = diag(1 + W^T 1)^-1 (X_T + W^T X_S)  for the compression
(Eq. 2 of the paper).  It follows Algorithm 1 / Algorithm 2 for a single head-averaged
map and exists only to pin the oracle."""
import numpy as np


def v_scores(P, cls, vis, lam, pos, gh, gw, window, coef):
    """P: list-of-lists [n_tot][n_tot] head-mean map. Returns penalised Eq. 1 scores."""
    N = len(vis)
    lam = float(np.float32(lam))
    s = []
    for i in vis:
        received = 0.0
        for q in vis:
            received += P[q][i]
        s.append(lam * (received / N) - (1.0 - lam) * P[cls][i])
    if window > 0:
        coef = float(np.float32(coef))
        groups = {}
        for t in range(N):
            r, c = divmod(pos[t] % (gh * gw), gw)
            key = (pos[t] // (gh * gw), r // window, c // window)
            groups.setdefault(key, []).append(t)
        boosted = {}
        for members in groups.values():
            top = max(s[t] for t in members)
            first = min((pos[t], t) for t in members if s[t] == top)[1]
            boosted[first] = coef * s[first]
        for t, v in boosted.items():
            s[t] = v
    return s


def l_scores(Pvv, Ptv, beta):
    N = len(Pvv)
    M = len(Ptv)
    beta = float(np.float32(beta))
    s = []
    for i in range(N):
        recv = 0.0
        for q in range(N):
            recv += Pvv[q][i]
        task = 0.0
        for k in range(M):
            task += Ptv[k][i]
        s.append(beta * (recv / N) - (1.0 - beta) * (task / M))
    return s


def split(s, n_keep):
    """Discard one token at a time: always the largest remaining score, lowest index first."""
    alive = list(range(len(s)))
    S = []
    for _ in range(len(s) - n_keep):
        best = alive[0]
        for i in alive:
            if s[i] > s[best]:
                best = i
        S.append(best)
        alive.remove(best)
    return sorted(S), alive


def dense_weights(C, eps):
    """W[a][b] = alpha_ab for b in J_a, else 0 (rows: discarded, columns: preserved)."""
    W = [[0.0] * len(C[0]) for _ in C] if len(C) and len(C[0]) else [[] for _ in C]
    for a, row in enumerate(C):
        if not row:
            continue
        tau = float(np.quantile(np.array(row, dtype=np.float64), float(np.float32(eps)),
                                method="linear"))
        hit = [b for b, v in enumerate(row) if v >= tau]
        tot = 0.0
        for b in hit:
            tot += row[b]
        if tot > 0.0:
            for b in hit:
                W[a][b] = row[b] / tot
    return W


def top_k_weights(C, K):
    """Ablation "fixed K": K rounds of "take the largest remaining value of the row, first
    position on ties"; weights = value / sum of the taken values."""
    W = [[0.0] * len(C[0]) for _ in C] if len(C) and len(C[0]) else [[] for _ in C]
    for a, row in enumerate(C):
        left = list(range(len(row)))
        took = []
        for _ in range(min(K, len(row))):
            best = left[0]
            for b in left:
                if row[b] > row[best]:
                    best = b
            took.append(best)
            left.remove(best)
        tot = 0.0
        for b in sorted(took):
            tot += row[b]
        if tot > 0.0:
            for b in took:
                W[a][b] = row[b] / tot
    return W


def merge(X, vis_begin, S, T, W, average=False, convergent=False):
    """average: every non-zero weight counts as one.  convergent: W is ignored, the preserved
    tokens stay, and the mean of the discarded tokens follows the last preserved one."""
    D = len(X[0])
    out = []
    gone = {vis_begin + i for i in S}
    slot = {vis_begin + j: b for b, j in enumerate(T)}
    extra_after = vis_begin + max(T) if (convergent and S and T) else None
    extra = None
    if convergent and S:
        extra = [sum(X[vis_begin + i][d] for i in S) / len(S) for d in range(D)]
    for t, row in enumerate(X):
        if convergent and S and not T and t == vis_begin:
            out.append(extra)
        if t in gone:
            continue
        if t in slot and not convergent:
            b = slot[t]
            col = [W[a][b] for a in range(len(S))]
            num = list(row)
            den = 1.0
            for a, w in enumerate(col):
                if w != 0.0:
                    if average:
                        w = 1.0
                    src = X[vis_begin + S[a]]
                    num = [num[d] + w * src[d] for d in range(D)]
                    den += w
            out.append([v / den for v in num])
        else:
            out.append(list(row))
        if t == extra_after:
            out.append(extra)
    return out


def v_step(X, P, cls, vis_begin, N, n_keep, lam, eps, pos, gh, gw, window, coef,
           fixed_k=None, average=False, convergent=False):
    vis = list(range(vis_begin, vis_begin + N))
    s = v_scores(P, cls, vis, lam, pos, gh, gw, window, coef)
    S, T = split(s, n_keep)
    P32 = [[float(np.float32(v)) for v in row] for row in P]
    C = [[P32[vis_begin + j][vis_begin + i] for j in T] for i in S]
    W = dense_weights(C, eps) if fixed_k is None else top_k_weights(C, fixed_k)
    return merge(X, vis_begin, S, T, W, average, convergent), S, T, W, s


def l_step(X, Pvv, Ptv, vis_begin, N, n_keep, beta, gamma, eps):
    s = l_scores(Pvv, Ptv, beta)
    S, T = split(s, n_keep)
    M = len(Ptv)
    g = float(np.float32(gamma))
    P32 = [[float(np.float32(v)) for v in row] for row in Pvv]
    C = []
    for i in S:
        row = []
        for j in T:
            ind = 0.0
            for k in range(M):
                ind += Ptv[k][i] * Ptv[k][j]
            row.append(g * P32[j][i] + (1.0 - g) * (ind / M))
        C.append(row)
    W = dense_weights(C, eps)
    return merge(X, vis_begin, S, T, W), S, T, W, s
