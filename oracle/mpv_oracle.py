"""fp64 CPU oracle for lossless multi-path verification of draft token trees.

THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only the tests, the smoke check
and the benchmark's cpu_baseline leg may import it.  It shares no code with the
HIP library and never calls it.  It is deliberately plain and slow: every
distribution is an explicit length-V float64 vector, every residual is formed
and normalised as written, nothing is fused, blocked or reordered.

What it computes (citations are to the paper's sections / algorithms):

* node distributions: p = softmax(z_target / T), q = softmax(z_draft / T)
  (Sec. 3: p(.|c), q(.|c) are next-token distributions; Sec. 4.1: sampling at a
  temperature; the paper does not say what the draft row is divided by: the
  same T, a reading).
* SpecInfer verification: the top-down walk of Sec. 3.2 ("OT-based algorithms")
  driving the SpecInfer OTLP solver of Appendix B, Algorithm 4, with children
  taken in ascending node index instead of uniformly at random.
* Traversal Verification: the bottom-up method cited in Sec. 3.2; the paper
  gives no listing, so this follows a reading of its description:
  chain weights w = min(1, w_parent * p/q) (the block-verification recursion of
  Sec. 3.1), leaves tested first in depth-first order, and on the rejection of a
  whole child subtree the parent's weight a and target distribution P are
  replaced by  S/(S+1-a)  and  (a*P - q)_+/S  with  S = sum (a*P - q)_+.
  It is pinned by exact losslessness (enumeration), by its K=1 reduction to
  block verification and by its depth-1 agreement with SpecInfer; its fidelity
  to the original Traversal paper beyond these properties is PARITY UNPINNED.
* bonus token: inverse-CDF sample from the final residual (Algorithm 4, last
  two lines; Sec. 2 step 3 "correction token").
* NSS and NaiveTree verification: the same top-down walk of Sec. 3.2 with the
  NSS solver (App. B, Alg. 1: Y ~ p, draft tokens ignored) or the Naive solver
  (App. B, Alg. 2: the first child is tested with min(1, p/q); otherwise
  Y ~ (p-q)_+).  With these solvers the token the solver outputs can be one of
  the other draft tokens: the walk then moves to the child carrying it and ends
  if no child does (Sec. 3.2, the top-down walk); with equal-token siblings, to
  the first of them in list order.
* SpecTr verification: the same walk with the K-SEQ solver (App. B, Alg. 3):
  division factor rho* = root of p_acc(rho) - rho*beta(rho) on [1,k] by binary
  search (64 halvings: the paper gives no stopping rule), children tested in
  list order with min(1, p/(rho* q)), then Y ~ (p - gamma*min(p/rho*, q))_+.

Conventions (each a reading where the paper is silent or loose):
* accept iff u < a (strict), u in [0,1): a = 0 never accepts, a = 1 always.
* inverse CDF: smallest t with cumsum(r)[t] > u * sum(r); never a zero-mass t.
* zero residual mass: the distribution is left unchanged; in Traversal the
  parent's weight becomes 1 if it was 1, else 0.
* one uniform per node: u[n] (n >= 1) is used only for the test of node n;
  u[0] draws the bonus token.  NSS and NaiveTree draw a token at every node
  they visit: the draw at node n uses u_draw[n], a second array.

Three drivers share the same step functions:
* verify_tree(...)          sample mode: consumes the uniforms.
* enumerate_outcomes(...)   probability mode: branches on every test with its
                            exact probability; used by the losslessness pins.
* all_test_probs(...)       the probability each node would be tested with if
                            it were reached (used to compare debug outputs).
"""

from __future__ import annotations

import numpy as np

SPECINFER = 0
TRAVERSAL = 1
NSS = 2
NAIVE = 3
SPECTR = 4


# --------------------------------------------------------------------------
# small helpers
# --------------------------------------------------------------------------

def children_lists(parent):
    """Ordered child lists (ascending node index) of a parent array.

    Sec. 3, Definition 3.1: a draft tree with ordered child lists.  parent[0]
    must be -1 and parent[n] < n for n >= 1.
    """
    parent = [int(x) for x in parent]
    n_nodes = len(parent)
    if n_nodes == 0 or parent[0] != -1:
        raise ValueError("parent[0] must be -1")
    ch = [[] for _ in range(n_nodes)]
    for n in range(1, n_nodes):
        if not (0 <= parent[n] < n):
            raise ValueError("parent[n] must satisfy 0 <= parent[n] < n")
        ch[parent[n]].append(n)
    return ch


def node_depths(parent):
    d = [0] * len(parent)
    for n in range(1, len(parent)):
        d[n] = d[int(parent[n])] + 1
    return d


def path_to(parent, n):
    """Nodes from the first non-root ancestor down to n (empty for the root)."""
    out = []
    n = int(n)
    while n > 0:
        out.append(n)
        n = int(parent[n])
    return out[::-1]


def softmax_T(z, T):
    """softmax(z / T) in float64 (Sec. 3; temperature of Sec. 4.1)."""
    x = np.asarray(z, dtype=np.float64) / float(T)
    x = x - np.max(x)
    e = np.exp(x)
    return e / np.sum(e)


def sample_index(r, u):
    """Inverse-CDF draw from the unnormalised non-negative vector r.

    Returns (t, gap): t is the smallest index with cumsum(r)[t] > u*sum(r);
    gap is the distance from u*sum(r) to the nearest CDF step, divided by
    sum(r) (how close the draw was to flipping to a neighbouring token).
    """
    r = np.asarray(r, dtype=np.float64)
    cdf = np.cumsum(r)
    total = cdf[-1]
    if not (total > 0.0):
        raise ValueError("cannot sample from a zero-mass vector")
    x = float(u) * total
    t = int(np.searchsorted(cdf, x, side="right"))
    if t >= len(r):  # rounding exhausted the CDF: last index with mass
        t = int(np.nonzero(r > 0)[0][-1])
    lo = cdf[t - 1] if t > 0 else 0.0
    gap = min(abs(x - lo), abs(cdf[t] - x)) / total
    return t, float(gap)


def _ratio(num, den):
    """min(1, num/den) with the guard for an underflowed denominator."""
    if den > 0.0:
        return min(1.0, num / den)
    return 1.0 if num > 0.0 else 0.0


# --------------------------------------------------------------------------
# the two verification rules, written against a `decide(node, a)` callback
# --------------------------------------------------------------------------

def specinfer_solver(P, Q, xs, decide, on_update=None):
    """SpecInfer OTLP solver (App. B, Alg. 4), children in list order.

    P, Q: target / draft distribution at the node; xs: the child tokens
    X_1..X_k; decide(i, a): is child i, tested with probability a, accepted?
    Returns (i, P): the accepted child's position (None if every child was
    rejected) and the current distribution, from which Y is drawn when i is
    None.  on_update(i, s), if given, is told the mass s of (p - q)_+ after the
    rejection of child i (reporting only).
    """
    P = np.array(P, dtype=np.float64)
    for i, x in enumerate(xs):
        a = _ratio(P[x], Q[x])                  # Alg. 4: U <= p(x)/q(x)
        if decide(i, a):
            return i, P
        r = np.maximum(P - Q, 0.0)              # Alg. 4: p <- norm (p-q)_+
        s = np.sum(r)
        if on_update is not None:
            on_update(i, float(s))
        if s > 0.0:
            P = r / s
    return None, P


def specinfer_rule(children, tokens, p_of, q_of, decide):
    """Top-down walk (Sec. 3.2) with the SpecInfer solver at every node.

    p_of(n), q_of(n) return node n's target / draft distribution (float64
    vectors).  decide(c, a) says whether child node c, tested with acceptance
    probability a, is accepted.  Returns (stop_node, P) where P is the
    distribution the bonus token is drawn from.
    """
    n = 0
    while True:
        ch = children[n]
        if not ch:
            return n, np.array(p_of(n), dtype=np.float64)
        i, P = specinfer_solver(p_of(n), np.asarray(q_of(n), dtype=np.float64),
                                [int(tokens[c]) for c in ch],
                                lambda i, a: decide(ch[i], a))
        if i is None:
            return n, P                         # Alg. 4: sample Y ~ p
        n = ch[i]                               # the walk goes on at the accepted child


def traversal_rule(children, tokens, p_of, q_of, decide, observe=None, on_update=None):
    """Bottom-up Traversal Verification (reading stated in the module header).

    Same callback protocol as specinfer_rule.  The root is accepted with
    probability 1 when the traversal comes back to it.  observe(n, a, P), if
    given, is called just before node n is tested.  on_update(n, c, a, S), if
    given, is told the weight a node n had and the mass S of (a P - q)_+ when the
    subtree of its child c was rejected (reporting only).
    """
    result = {}

    def process(n, a):
        P = np.array(p_of(n), dtype=np.float64)
        if children[n]:
            Q = np.asarray(q_of(n), dtype=np.float64)
            for c in children[n]:
                x = int(tokens[c])
                a_c = _chain_weight(a, P[x], Q[x])
                if process(c, a_c):
                    return True
                # the whole subtree of c was rejected: delete it, update n
                r = np.maximum(a * P - Q, 0.0)
                S = np.sum(r)
                if on_update is not None:
                    on_update(n, c, float(a), float(S))
                if S > 0.0:
                    P = r / S
                    a = S / (S + (1.0 - a))
                else:
                    a = 1.0 if a >= 1.0 else 0.0
        if observe is not None:
            observe(n, a, P)
        if n == 0 or decide(n, a):
            result["node"] = n
            result["P"] = P
            return True
        return False

    process(0, 1.0)
    return result["node"], result["P"]


def _chain_weight(a, num, den):
    """min(1, a * num/den): the block-verification weight recursion (Sec. 3.1),
    with the guards for a zero weight, a zero numerator and an underflowed
    denominator."""
    if a <= 0.0 or num <= 0.0:
        return 0.0
    if den > 0.0:
        return min(1.0, a * num / den)
    return 1.0


_RULES = {SPECINFER: specinfer_rule, TRAVERSAL: traversal_rule}


# --------------------------------------------------------------------------
# solvers whose output token can be another draft token: NSS and Naive, and the
# walk that follows the drawn token (Sec. 3.2)
# --------------------------------------------------------------------------

def nss_solver(P, Q, xs, decide):
    """NSS OTLP solver (App. B, Alg. 1): no test; Y is drawn from p."""
    return None, np.array(P, dtype=np.float64)


def naive_solver(P, Q, xs, decide):
    """Naive OTLP solver (App. B, Alg. 2): only the first draft token is tested,
    with min(1, p/q); otherwise Y is drawn from (p - q)_+ (normalised by the draw)."""
    P = np.array(P, dtype=np.float64)
    if xs:
        x = xs[0]
        if decide(0, _ratio(P[x], Q[x])):
            return 0, P
        r = np.maximum(P - Q, 0.0)
        if np.sum(r) > 0.0:                     # zero mass: p = q, the test above cannot fail
            P = r
    return None, P


def spectr_beta(P, Q, rho):
    """beta(rho) = sum_x min(p(x)/rho, q(x))  (App. B, SpecTr)."""
    return float(np.sum(np.minimum(P / rho, Q)))


def spectr_division_factor(P, Q, k):
    """rho*: the root of rho -> p_acc(rho) - rho*beta(rho), p_acc = 1-(1-beta)^k, on [1,k].

    The map is monotone decreasing with a value >= 0 at 1 and <= 0 at k (App. B); binary
    search as the paper says, run until float64 is exhausted.  The function is evaluated as
        sum (p - rho q)_+  -  (sum (q - p/rho)_+)^k ,
    which is the same number: rho*beta = sum min(p, rho q) = 1 - sum (p - rho q)_+ and
    1 - beta = sum (q - p/rho)_+.  Written with beta itself, both halves are 1 - (something
    tiny) when p is close to q and the difference drowns in rounding."""
    P = np.asarray(P, dtype=np.float64)
    Q = np.asarray(Q, dtype=np.float64)
    lo, hi = 1.0, float(k)
    for _ in range(64):
        mid = 0.5 * (lo + hi)
        excess = float(np.sum(np.maximum(P - mid * Q, 0.0)))
        deficit = float(np.sum(np.maximum(Q - P / mid, 0.0)))
        if excess - deficit ** k > 0.0:
            lo = mid
        else:
            hi = mid
    return 0.5 * (lo + hi)


def spectr_solver(P, Q, xs, decide):
    """SpecTr OTLP solver, K-SEQ (App. B, Alg. 3), children in list order."""
    P = np.array(P, dtype=np.float64)
    k = len(xs)
    if k == 0:
        return None, P
    rho = spectr_division_factor(P, Q, k)
    beta = spectr_beta(P, Q, rho)
    p_acc = 1.0 - (1.0 - beta) ** k
    gamma = p_acc / beta if beta > 0.0 else 0.0
    for i, x in enumerate(xs):
        if decide(i, _ratio(P[x], rho * Q[x])):     # Alg. 3: rho* U <= p(x)/q(x)
            return i, P
    r = np.maximum(P - np.minimum(P / rho, Q) * gamma, 0.0)
    if np.sum(r) > 0.0:
        P = r
    return None, P


_SOLVERS = {NSS: nss_solver, NAIVE: naive_solver, SPECTR: spectr_solver}


def token_walk(solver, children, tokens, p_of, q_of, decide, draw, node_of=None):
    """Top-down walk (Sec. 3.2) for solvers whose output can be any token.

    At node n the solver either accepts a child or hands back the (unnormalised)
    vector Y is drawn from; draw(n, r) returns the drawn token.  If that token is
    the token of a child (the first such child in list order) the walk moves
    there, otherwise it ends.  A leaf has no draft tokens: Y ~ p, and the walk
    ends.  Returns (stop_node, final_token, r_last): the node the walk ended in,
    the token drawn there and the vector it was drawn from.

    node_of (Def. 3.1: a child list can name one node several times, each entry
    with a number and a uniform of its own): node_of[c] is the node that entry c
    stands for, where the walk goes on when c is accepted; None: c itself.
    """
    n = 0
    while True:
        ch = children[n]
        xs = [int(tokens[c]) for c in ch]
        i, r = solver(p_of(n), np.asarray(q_of(n), dtype=np.float64) if ch else None, xs,
                      lambda i, a: decide(ch[i], a))
        if i is not None:
            n = ch[i] if node_of is None else int(node_of[ch[i]])
            continue
        y = draw(n, r)
        match = [c for c, x in zip(ch, xs) if x == y]
        if not match:
            return n, int(y), r
        n = match[0]


# --------------------------------------------------------------------------
# drivers
# --------------------------------------------------------------------------

class _RowCache:
    """softmax rows computed on first use, from logits of shape [N, V]."""

    def __init__(self, logits, T):
        self.logits = logits
        self.T = T
        self.rows = {}

    def __call__(self, n):
        if n not in self.rows:
            self.rows[n] = softmax_T(self.logits[n], self.T)
        return self.rows[n]


def verify_tree(method, parent, tokens, target_logits, draft_logits, T, u, u_draw=None, node_of=None):
    """Sample mode for ONE tree.

    parent: [N] ints; tokens: [N] ints (tokens[0] ignored); target_logits,
    draft_logits: [N, V] arrays holding the exact stored logit values;
    u: [N] uniforms in [0,1); u_draw: [N] more uniforms, needed by NSS, NAIVE and
    SPECTR only (the draw at node n); node_of: see token_walk (those methods only).
    Returns a dict with
      stop_node, accept_len, path_nodes, path_tokens, bonus_token,
      residual (float64 [V], normalised), decisions [(node, a, u, accepted)],
      min_margin (smallest |a - u| over decisions with a < 1, or inf),
      bonus_gap (see sample_index; the smallest over the draws of the walk),
      draws [(node, token, gap)] (NSS and NAIVE: every draw of the walk).
    """
    children = children_lists(parent)
    p_of = _RowCache(target_logits, T)
    q_of = _RowCache(draft_logits, T)
    decisions = []
    draws = []

    def decide(c, a):
        ok = bool(float(u[c]) < a)
        decisions.append((int(c), float(a), float(u[c]), ok))
        return ok

    if method in _SOLVERS:
        def draw(n, r):
            t, g = sample_index(r, u_draw[n])
            draws.append((int(n), int(t), float(g)))
            return t

        stop, bonus, P = token_walk(_SOLVERS[method], children, tokens, p_of, q_of, decide, draw, node_of)
        gap = min(g for (_, _, g) in draws)
    else:
        stop, P = _RULES[method](children, tokens, p_of, q_of, decide)
        bonus, gap = sample_index(P, u[0])
    nodes = path_to(parent, stop)
    margins = [abs(a - uu) for (_, a, uu, _) in decisions]
    return {
        "stop_node": int(stop),
        "accept_len": len(nodes),
        "path_nodes": nodes,
        "path_tokens": [int(tokens[n]) for n in nodes],
        "bonus_token": int(bonus),
        "residual": P / np.sum(P),
        "decisions": decisions,
        "min_margin": min(margins) if margins else float("inf"),
        "bonus_gap": gap,
        "draws": draws,
    }


def verify_batch(method, parent, tokens, target_logits, draft_logits, T, u, u_draw=None):
    """Sample mode for a batch: tokens [B,N], logits [B,N,V], u [B,N] (u_draw likewise)."""
    return [
        verify_tree(method, parent, tokens[b], target_logits[b], draft_logits[b], T, u[b],
                    None if u_draw is None else u_draw[b])
        for b in range(len(tokens))
    ]


def enumerate_outcomes(method, parent, tokens, p_of, q_of, node_of=None):
    """Probability mode: every reachable (stop_node, P) with its probability.

    Each test of a node with acceptance probability a is branched into
    "accepted" (weight a) and "rejected" (weight 1-a).  Returns a list of
    (prob, stop_node, P) whose probs sum to 1.
    """
    children = children_lists(parent)
    if method in _SOLVERS:
        return _enumerate_token_walk(_SOLVERS[method], children, tokens, p_of, q_of, node_of)
    rule = _RULES[method]
    outcomes = []
    pending = [[]]                      # decision scripts still to run
    while pending:
        script = pending.pop()
        taken = []                      # (a, decision) actually made

        def decide(c, a, script=script, taken=taken):
            i = len(taken)
            d = script[i] if i < len(script) else True
            taken.append((float(a), d))
            return d

        stop, P = rule(children, tokens, p_of, q_of, decide)
        prob = 1.0
        for a, d in taken:
            prob *= a if d else (1.0 - a)
        if prob > 0.0:
            outcomes.append((prob, int(stop), np.array(P)))
        for i in range(len(script), len(taken)):
            if taken[i][0] < 1.0:       # the opposite branch has weight > 0
                pending.append([d for (_, d) in taken[:i]] + [False])
    return outcomes


def _enumerate_token_walk(solver, children, tokens, p_of, q_of, node_of=None):
    """Probability mode of token_walk: every test is branched as in
    enumerate_outcomes, every draw into one branch per token of positive mass.
    Returns (prob, stop_node, final_token) triples (the final token in place of
    a distribution: here the draws are part of the walk)."""
    outcomes = []
    pending = [[]]                      # scripts of choices: booleans for tests, tokens for draws
    while pending:
        script = pending.pop()
        made = []                       # (choice, its probability, choices not explored yet)

        def decide(c, a, script=script, made=made):
            i = len(made)
            d = script[i] if i < len(script) else True
            others = [False] if (i >= len(script) and a < 1.0) else []
            made.append((d, float(a) if d else 1.0 - float(a), others))
            return d

        def draw(n, r, script=script, made=made):
            i = len(made)
            r = np.asarray(r, dtype=np.float64)
            support = [int(t) for t in np.nonzero(r > 0)[0]]
            y = script[i] if i < len(script) else support[0]
            others = [t for t in support if t != y] if i >= len(script) else []
            made.append((y, float(r[y] / np.sum(r)), others))
            return y

        stop, y, _ = token_walk(solver, children, tokens, p_of, q_of, decide, draw, node_of)
        prob = 1.0
        for _, w, _ in made:
            prob *= w
        if prob > 0.0:
            outcomes.append((prob, int(stop), int(y)))
        prefix = [m[0] for m in made]
        for i in range(len(script), len(made)):
            for other in made[i][2]:
                pending.append(prefix[:i] + [other])
    return outcomes


def all_test_probs(method, parent, tokens, target_logits, draft_logits, T, updates=None, rows=None):
    """Probability with which each node would be tested if it were reached.

    Because a node is only ever tested after one fixed history (SpecInfer:
    parent reached, earlier siblings rejected; Traversal: everything earlier in
    the depth-first order rejected), that probability does not depend on the
    uniforms.  Entry 0 (the root) is 1.  Also returns, for every node, the
    normalised distribution a bonus token would be drawn from if the rule
    stopped there.  updates, if a list, receives one (node, child, weight, mass)
    per residual update made on the way: after the rejection of `child` (of its
    whole subtree, Traversal) node `node`, of weight `weight` (1 for SpecInfer), had
    the residual mass `mass`.  rows, if given, is a pair of callables (p_of, q_of) that
    supply the node distributions in place of the softmax of the logits (the tests use it
    to see how far the results move when the distributions are slightly off).
    """
    children = children_lists(parent)
    n_nodes = len(parent)
    p_of, q_of = rows if rows is not None else (_RowCache(target_logits, T), _RowCache(draft_logits, T))
    probs = np.full(n_nodes, np.nan)
    probs[0] = 1.0
    stop_dist = [None] * n_nodes

    if method == TRAVERSAL:
        # Reject everything: the traversal then tests every node exactly once.
        def observe(n, a, P):
            if n != 0:
                probs[n] = a
            stop_dist[n] = P / np.sum(P)

        on_update = None if updates is None else (lambda n, c, a, S: updates.append((n, c, a, S)))
        traversal_rule(children, tokens, p_of, q_of, lambda c, a: False, observe, on_update)
        return probs, stop_dist

    # SpecInfer: run the solver at every node, rejecting every child.
    for n in range(n_nodes):
        ch = children[n]
        if not ch:
            stop_dist[n] = np.array(p_of(n))
            continue

        def decide(i, a, ch=ch):
            probs[ch[i]] = a
            return False

        on_update = None if updates is None else (lambda i, m, n=n, ch=ch: updates.append((n, ch[i], 1.0, m)))
        _, P = specinfer_solver(p_of(n), q_of(n), [int(tokens[c]) for c in ch], decide, on_update)
        stop_dist[n] = P / np.sum(P)
    return probs, stop_dist


# --------------------------------------------------------------------------
# counter-based uniforms (the oracle's own copy of the generator the library
# documents: SplitMix64 finaliser of seed + (index+1)*golden-ratio increment,
# top 24 bits scaled by 2^-24)
# --------------------------------------------------------------------------

def uniforms_from_seed(seed, count):
    """count float32 uniforms in [0,1), element i from counter i."""
    mask = (1 << 64) - 1
    out = np.empty(count, dtype=np.float32)
    for i in range(count):
        z = (int(seed) + (i + 1) * 0x9E3779B97F4A7C15) & mask
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & mask
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & mask
        z = z ^ (z >> 31)
        out[i] = np.float32((z >> 40) * (1.0 / 16777216.0))
    return out
