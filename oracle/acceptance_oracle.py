"""fp64 CPU oracle for the acceptance rates of the OTLP solvers (App. C).

THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT (see mpv_oracle.py): only the tests,
the smoke check and the benchmark's cpu_baseline leg may import it; it shares no
code with the HIP library and never calls it.

Acceptance rate (Sec. 3.2): for a node with target distribution p, draft
distribution q and k draft tokens drawn i.i.d. from q, the probability, over the
draft tokens and the solver's own randomness, that the solver's output token is
one of the draft tokens.  The listings of App. C, written out with explicit
length-V vectors:

    NSS        sum_t p(t) (1 - (1 - q(t))^k)
    Naive      sum_t min(p(t), q(t)) + sum_t (p(t) - q(t))_+ (1 - (1 - q(t))^(k-1))
    SpecTr     rho*, beta, p_acc, gamma as in the solver;  p_res = norm (p - gamma min(p/rho*, q))_+,
               r = (q - p/rho*)_+ / (1 - beta);  p_acc + (1 - p_acc) sum_t p_res(t) (1 - (1 - r(t))^k)
    SpecInfer  k rounds: r = sum min(p, q), p_rej *= 1 - r, m *= 1 - (q - p)_+/(1 - r), p <- norm (p - q)_+;
               (1 - p_rej) + p_rej sum_t p(t) (1 - m(t))

(Khisti has no exact listing in the paper and its subroutines are defined elsewhere;
Traversal Verification is not an OTLP solver.)
"""

from __future__ import annotations

import numpy as np

from . import mpv_oracle as base


def nss_acceptance(P, Q, k):
    P = np.asarray(P, dtype=np.float64)
    Q = np.asarray(Q, dtype=np.float64)
    return float(np.sum(P * (1.0 - (1.0 - Q) ** k)))


def naive_acceptance(P, Q, k):
    P = np.asarray(P, dtype=np.float64)
    Q = np.asarray(Q, dtype=np.float64)
    return float(np.sum(np.minimum(P, Q)) + np.sum(np.maximum(P - Q, 0.0) * (1.0 - (1.0 - Q) ** (k - 1))))


def spectr_acceptance(P, Q, k):
    P = np.asarray(P, dtype=np.float64)
    Q = np.asarray(Q, dtype=np.float64)
    rho = base.spectr_division_factor(P, Q, k)
    beta = base.spectr_beta(P, Q, rho)
    p_acc = 1.0 - (1.0 - beta) ** k
    gamma = p_acc / beta if beta > 0.0 else 0.0
    res = np.maximum(P - np.minimum(P / rho, Q) * gamma, 0.0)
    if np.sum(res) > 0.0:
        res = res / np.sum(res)
    if beta >= 1.0:                                 # p = q: every draft token is accepted
        return 1.0
    r = np.maximum(Q - P / rho, 0.0) / (1.0 - beta)
    return float(p_acc + (1.0 - p_acc) * np.sum(res * (1.0 - (1.0 - r) ** k)))


def specinfer_acceptance(P, Q, k):
    P = np.array(P, dtype=np.float64)
    Q = np.asarray(Q, dtype=np.float64)
    p_rej = 1.0
    m = np.ones(len(P))
    for _ in range(k):
        r = float(np.sum(np.minimum(P, Q)))
        nxt = np.maximum(P - Q, 0.0)
        if r >= 1.0 or not (np.sum(nxt) > 0.0):     # p = q: this round accepts whatever is drawn
            p_rej = 0.0
            break
        p_rej *= 1.0 - r
        m = m * (1.0 - np.maximum(Q - P, 0.0) / (1.0 - r))
        P = nxt / np.sum(nxt)
    return float((1.0 - p_rej) + p_rej * np.sum(P * (1.0 - m)))


_ACCEPTANCE = {base.SPECINFER: specinfer_acceptance, base.NSS: nss_acceptance, base.NAIVE: naive_acceptance,
               base.SPECTR: spectr_acceptance}


def acceptance_rates(method, parent, target_logits, draft_logits, T):
    """Acceptance rate of every internal node of one tree given its stored logits [N, V], with k = the
    node's number of children; leaves get 0.  Returns float64 [N]."""
    children = base.children_lists(parent)
    out = np.zeros(len(parent))
    for n, ch in enumerate(children):
        if ch:
            out[n] = _ACCEPTANCE[method](base.softmax_T(target_logits[n], T), base.softmax_T(draft_logits[n], T), len(ch))
    return out
