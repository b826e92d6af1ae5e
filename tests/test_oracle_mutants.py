"""The pins must FAIL when a plausible mistake is planted in the oracle (on the CPU):
a dropped term, a wrong sign or index, a transposed operand.  Each mutant replaces one
oracle function; at least one pin test has to notice."""
import numpy as np
import pytest

from oracle import ficoco_oracle as O
from tests import test_oracle_pins as pins

PIN_TESTS = [getattr(pins, n) for n in dir(pins) if n.startswith("test_")]


def _run_pins():
    """Names of the pin tests that fail against the current (possibly mutated) oracle."""
    failed = []
    for t in PIN_TESTS:
        marks = [m for m in getattr(t, "pytestmark", []) if m.name == "parametrize"]
        cases = [()]
        if marks:
            names, values = marks[0].args[0], marks[0].args[1]
            n_args = len([a for a in names.split(",")])
            cases = [v if n_args > 1 else (v,) for v in values]
        for c in cases:
            try:
                t(*c)
            except AssertionError:
                failed.append(t.__name__)
                break
            except Exception:
                failed.append(t.__name__)
                break
    return failed


def test_pins_pass_on_the_real_oracle():
    assert _run_pins() == []


def _m_row_mean(P, query_rows, key_cols):          # transposed operand
    acc = np.zeros(len(key_cols))
    for q in query_rows:
        acc = acc + P[key_cols, q]
    return acc / float(len(key_cols))


def _m_score_sign(R, G, w):                         # wrong sign of the semantic term
    w = O.f32(w)
    return w * np.asarray(R) + (1.0 - w) * np.asarray(G)


def _m_corr_transposed(P32, S, T, key_cols, query_rows):
    rows = np.asarray(query_rows)[np.asarray(S)]
    cols = np.asarray(key_cols)[np.asarray(T)]
    return P32[np.ix_(rows, cols)].astype(np.float64)


def _m_quantile_off_by_one(row, eps):               # wrong index
    v = np.sort(np.asarray(row, dtype=np.float64))
    n = len(v)
    p = O.f32(eps) * float(n)
    f = min(int(np.floor(p)), n - 1)
    g = p - np.floor(p)
    return v[f] + g * (v[min(f + 1, n - 1)] - v[f])


def _m_bridge_no_mean(Ptext, S, T):                 # dropped 1/M
    return Ptext[:, S].T @ Ptext[:, T]


def _m_filter_ascending(s, n_keep):                 # keeps the most redundant tokens
    s = np.asarray(s, dtype=np.float64)
    n = len(s)
    order = sorted(range(n), key=lambda i: (s[i], i))
    return (np.array(sorted(order[:n - n_keep]), dtype=np.int64),
            np.array(sorted(order[n - n_keep:]), dtype=np.int64))


def _m_compress_no_self(X, vis_begin, S, T, J, alpha, average=False, extra=None):   # dropped the "1 +" of Eq. 2
    if average or extra is not None:
        return O._real_compress(X, vis_begin, S, T, J, alpha, average=average, extra=extra)
    out = O._real_compress(X, vis_begin, S, T, J, alpha)
    a = np.zeros(len(T))
    for i in range(len(S)):
        for jj, w in zip(J[i], alpha[i]):
            a[jj] += w
    for b, j in enumerate(T):
        if a[b] > 0:
            out[vis_begin + b] = out[vis_begin + b] * (1 + a[b]) / a[b]
    return out


def _m_penalty_min(s, pos, g, h, w, window, coef):  # multiplies the window minimum
    out = -O._real_penalty(-np.asarray(s, dtype=np.float64), pos, g, h, w, window, coef)
    return out


def _m_head_mean_first(A):                          # ignores all heads but the first
    return np.asarray(A, dtype=np.float64)[0].copy()


def _m_fixed_k_high_index(C, K):                    # ties go to the higher position
    J, alpha = [], []
    for i in range(C.shape[0]):
        order = sorted(range(C.shape[1]), key=lambda j: (-C[i, j], -j))
        sel = np.array(sorted(order[:max(int(K), 0)]), dtype=np.int64)
        d = sum(C[i, j] for j in sel)
        if len(sel) and d > 0.0:
            J.append(sel); alpha.append(np.array([C[i, j] / d for j in sel]))
        else:
            J.append(np.zeros(0, np.int64)); alpha.append(np.zeros(0))
    return J, alpha


def _m_average_keeps_weights(X, vis_begin, S, T, J, alpha, average=False, extra=None):   # "average" still weighted
    return O._real_compress(X, vis_begin, S, T, J, alpha, average=False, extra=extra)


def _m_convergent_sum(X, vis_begin, S):             # dropped the division by N^S
    return O._real_convergent(X, vis_begin, S) * float(len(S))


def _m_gap_top1(C):                                 # forgot to subtract the runner-up
    return np.max(C, axis=1) if C.shape[1] >= 2 else np.zeros(C.shape[0])


MUTANTS = [
    ("received_attention", _m_row_mean),
    ("combine_score", _m_score_sign),
    ("correlation_attention", _m_corr_transposed),
    ("quantile_threshold", _m_quantile_off_by_one),
    ("text_bridge", _m_bridge_no_mean),
    ("filter_tokens", _m_filter_ascending),
    ("compress", _m_compress_no_self),
    ("local_penalty", _m_penalty_min),
    ("head_mean", _m_head_mean_first),
    ("fixed_k_targets", _m_fixed_k_high_index),
    ("compress", _m_average_keeps_weights),
    ("convergent_token", _m_convergent_sum),
    ("correlation_gap", _m_gap_top1),
]


@pytest.mark.parametrize("name,mutant", MUTANTS, ids=["%s-%s" % (m[0], m[1].__name__) for m in MUTANTS])
def test_planted_mistake_is_caught(monkeypatch, name, mutant):
    monkeypatch.setattr(O, "_real_compress", O.compress, raising=False)
    monkeypatch.setattr(O, "_real_penalty", O.local_penalty, raising=False)
    monkeypatch.setattr(O, "_real_convergent", O.convergent_token, raising=False)
    monkeypatch.setattr(O, name, mutant)
    failed = _run_pins()
    assert failed, "no pin noticed the mutated %s" % name
