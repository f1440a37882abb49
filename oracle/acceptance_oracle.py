"""fp64 CPU oracle for the acceptance rates of the OTLP solvers (Sec. 3.2, Def. 5.1).

THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT (see mpv_oracle.py): only the tests,
the smoke check and the benchmark's cpu_baseline leg may import it; it shares no
code with the HIP library and never calls it.

Acceptance rate of a node with target distribution p, draft distribution q and k draft
tokens X_1..X_k drawn i.i.d. from q: the probability, over the draft tokens and the solver's
own randomness, that the solver's output token is one of the draft tokens.

It is put together here from what each solver of App. B does, round by round, by the law of
total probability.  A solver is described by
  * one vector per draft token, in the order the tokens are looked at: test[i][t] is the
    probability that X_i is accepted if it is the token t and no earlier one was accepted
    (all zeros for a token the solver never tests), and
  * the distribution `fallback` the output is drawn from when no draft token was accepted.
Given that round i is reached, X_i is still distributed as q (the earlier rounds did not look
at it), so round i accepts with probability  h_i = sum_t q(t) test[i][t], and a token that
was looked at and not accepted is distributed as  q (1 - test[i]) / (1 - h_i).  The draft
tokens that were passed over are independent of each other and of the fallback draw, hence

    rate = sum_i  (prod_{j<i} (1 - h_j)) h_i
         + (prod_j (1 - h_j)) sum_t fallback(t) (1 - prod_i (1 - passed_i(t))).

The closed forms the paper prints (App. C) are not used here; the tests hold them as pins,
next to a brute-force enumeration over all draft tuples with the solvers of mpv_oracle.py.
(Khisti has no exact listing in the paper; Traversal Verification is not an OTLP solver.)
"""

from __future__ import annotations

import numpy as np

from . import mpv_oracle as base


def _test_probabilities(numerator, denominator):
    """min(1, numerator/denominator) for every token, with mpv_oracle._ratio's guard for a
    denominator that has underflowed to zero."""
    numerator = np.asarray(numerator, dtype=np.float64)
    denominator = np.asarray(denominator, dtype=np.float64)
    safe = np.where(denominator > 0.0, denominator, 1.0)
    with_den = np.minimum(1.0, numerator / safe)
    without = np.where(numerator > 0.0, 1.0, 0.0)
    return np.where(denominator > 0.0, with_den, without)


def _normalised(v, otherwise):
    s = float(np.sum(v))
    return v / s if s > 0.0 else otherwise


def describe_nss(P, Q, k):
    """App. B, Alg. 1: nothing is tested, the output is drawn from p."""
    return [np.zeros(len(P)) for _ in range(k)], P


def describe_naive(P, Q, k):
    """App. B, Alg. 2: the first draft token is tested against p/q; the output is otherwise
    drawn from the normalised excess of p over q."""
    tests = [_test_probabilities(P, Q)] + [np.zeros(len(P)) for _ in range(k - 1)]
    return tests[:k], _normalised(np.maximum(P - Q, 0.0), P)


def describe_specinfer(P, Q, k):
    """App. B, Alg. 4: every draft token in turn against the current distribution, which a
    rejection replaces by the normalised excess over q."""
    tests = []
    current = P
    for _ in range(k):
        tests.append(_test_probabilities(current, Q))
        current = _normalised(np.maximum(current - Q, 0.0), current)
    return tests, current


def describe_spectr(P, Q, k):
    """App. B, Alg. 3 (K-SEQ): every draft token against p / (rho* q); the fallback is what is
    left of p after the accepted mass has been taken out."""
    rho = base.spectr_division_factor(P, Q, k)
    beta = base.spectr_beta(P, Q, rho)
    accepted_somewhere = 1.0 - (1.0 - beta) ** k
    share = accepted_somewhere / beta if beta > 0.0 else 0.0
    test = _test_probabilities(P, rho * Q)
    left = np.maximum(P - share * np.minimum(P / rho, Q), 0.0)
    return [test for _ in range(k)], _normalised(left, P)


_DESCRIPTIONS = {base.NSS: describe_nss, base.NAIVE: describe_naive, base.SPECINFER: describe_specinfer,
                 base.SPECTR: describe_spectr}


def acceptance_rate(method, P, Q, k):
    """Acceptance rate of one node (see the module text)."""
    P = np.asarray(P, dtype=np.float64)
    Q = np.asarray(Q, dtype=np.float64)
    tests, fallback = _DESCRIPTIONS[method](P, Q, k)
    reached = 1.0                        # no draft token accepted so far
    nobody_is = np.ones(len(P))          # given that: none of the tokens passed over so far is t
    rate = 0.0
    for test in tests:
        h = float(np.sum(Q * test))
        rate += reached * h
        if h >= 1.0:                     # this round accepts whatever comes (p = q)
            return float(min(rate, 1.0))
        nobody_is = nobody_is * (1.0 - Q * (1.0 - test) / (1.0 - h))
        reached *= 1.0 - h
    rate += reached * float(np.sum(fallback * (1.0 - nobody_is)))
    return float(rate)


def nss_acceptance(P, Q, k):
    return acceptance_rate(base.NSS, P, Q, k)


def naive_acceptance(P, Q, k):
    return acceptance_rate(base.NAIVE, P, Q, k)


def spectr_acceptance(P, Q, k):
    return acceptance_rate(base.SPECTR, P, Q, k)


def specinfer_acceptance(P, Q, k):
    return acceptance_rate(base.SPECINFER, P, Q, k)


def acceptance_rates(method, parent, target_logits, draft_logits, T):
    """Acceptance rate of every internal node of one tree given its stored logits [N, V], with k = the
    node's number of children; leaves get 0.  Returns float64 [N]."""
    children = base.children_lists(parent)
    out = np.zeros(len(parent))
    for n, ch in enumerate(children):
        if ch:
            out[n] = acceptance_rate(method, base.softmax_T(target_logits[n], T), base.softmax_T(draft_logits[n], T), len(ch))
    return out
