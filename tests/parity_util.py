"""Element-by-element comparison of the HIP library's outputs with the oracle.

Bars (written here so every parity test uses the same ones):
* integer outputs (accepted length, path nodes, path tokens, bonus token) must be
  identical, except that a tree whose oracle walk contains a test with
  |a - u| < DECISION_BAND may take the other branch, and a bonus token may
  differ when u*R lies within BONUS_BAND (relative to R) of a CDF step.  Such
  trees are counted and returned, never silently accepted beyond the band.
  For the methods that draw a token at every node they visit (NSS, Naive, SpecTr) any
  of the walk's draws within BONUS_BAND of a CDF step may send the walk elsewhere.
* probabilities (edge probabilities, per-node test probabilities, the final
  normalised residual) must agree within PROB_ATOL absolute.  Two kinds of test probability are
  treated apart, both counted in the report:
  - "remote": the test can only be performed after events of total probability <= DECISION_BAND
    (say, after a sibling that is accepted with probability 1 was rejected).  Such a number
    cannot influence any output beyond the decision band, and it is the quotient of two residual
    masses that may both be tiny.  It is still compared, against PROB_ATOL plus the error float32
    terms leave on a residual mass W after c draft rows have been subtracted, SUM_REL_ERR (1 + c)/W
    times a small factor (see remote_tolerance); where that exceeds SPECTR_SLACK_CAP the mass is
    below float32 resolution and the number is counted as noise instead ("noise_tests").
  - "fragile": it follows a residual update at the rule's one discontinuity (see fragile_tests).
    Left out; the five benchmark configurations must have none.
* row maxima must be identical; ln-sum-exp statistics within PROB_ATOL.
"""

import numpy as np

from oracle import mpv_oracle as orc

DECISION_BAND = 1e-6
BONUS_BAND = 1e-6
PROB_ATOL = 1e-5
# SpecTr's division factor is the root of a function of V-wide sums; a relative error e in those
# sums moves the root, and with it every test probability p/(rho* q), by up to kappa * e,
# kappa = oracle.spectr_conditioning (large only where the function is flat on one side of the
# root).  The paper gives no stopping rule for its binary search; the library's root is exact up
# to the accuracy of its float32 sums, taken as 3e-7 relative here (three times the 1e-7 that one
# v_exp_f32 and the rounding of its argument give a term).
SUM_REL_ERR = 3e-7
# The slack never opens a bar further than this, however flat the root function is.
SPECTR_SLACK_CAP = 1e-3
# A residual mass below this, next to a weight within this of 1, is the rule's discontinuity.
FRAGILE_MASS = 1e-6


def spectr_conditioning(P, Q, k, rho):
    """How far relative errors of size e in the V-wide sums move SpecTr's division factor:
    |d ln rho*| <= kappa * e  (first order; pinned by tests/test_parity_util_pins.py, which perturbs
    P and Q and solves the printed equation again).

    With W = sum (p - rho q)_+, D = sum (q - p/rho)_+ = (W + rho - 1)/rho and f = W - D^k (the root
    function of App. B's SpecTr solver with beta eliminated): an error e in W and in the normalisation
    of p and q changes f by at most e * (W + k D^(k-1) (W + 2)/rho), and
    f' = -sum_{p > rho q} q - k D^(k-1) sum_{p < rho q} p/rho^2.
    The root often sits on, or within 1e-7 of, a kink of f (the ratio p/q of a dominant token), where
    the slopes to the left and right differ by orders of magnitude: the slopes are taken 1e-6 to
    either side (closer than float32 sums can tell apart) and the flatter one counts.
    Test-side tolerance model only: neither the oracle nor the library uses it.
    """
    if k <= 1:
        return 0.0
    P = np.asarray(P, dtype=np.float64)
    Q = np.asarray(Q, dtype=np.float64)
    W = float(np.sum(np.maximum(P - rho * Q, 0.0)))
    D = float(np.sum(np.maximum(Q - P / rho, 0.0)))
    df = W + k * D ** (k - 1) * (W + 2.0) / rho
    slopes = []
    for r in (rho * (1.0 - 1e-6), rho * (1.0 + 1e-6)):       # just left and just right of the root
        up = P > r * Q
        slopes.append(float(np.sum(Q[up])) + k * D ** (k - 1) * float(np.sum(P[~up])) / (r * r))
    slope = min(slopes)
    if slope <= 0.0:
        return float("inf")
    return df / (slope * rho)


def spectr_slack(host, b, node_parent, T, k, capped=None):
    """Extra tolerance on the test probabilities of the children of node_parent (SpecTr): the
    conditioning of the root times the accuracy of float32 sums, never more than SPECTR_SLACK_CAP
    (a flat root function would otherwise open the bar without limit).  capped, if a list, gets
    one entry per slack that hit the cap."""
    P = orc.softmax_T(host["target"][b][node_parent], T)
    Q = orc.softmax_T(host["draft"][b][node_parent], T)
    rho = orc.spectr_division_factor(P, Q, k)
    slack = SUM_REL_ERR * spectr_conditioning(P, Q, k, rho)
    if not (slack <= SPECTR_SLACK_CAP):                       # also inf and nan
        if capped is not None:
            capped.append((b, node_parent, slack))
        slack = SPECTR_SLACK_CAP
    return slack


def node_tolerances(method, host, b, T):
    """Per-node bar on the reach probability."""
    parent = host["parent"]
    N = len(parent)
    tol = np.full(N, PROB_ATOL)
    if method != orc.SPECTR:
        return tol
    children = orc.children_lists(parent)
    slack = np.zeros(N)                       # of the step from a node to any of its children
    for n in range(N):
        if len(children[n]) > 1:
            # every test probability moves by at most the slack; a step combines up to k of them
            slack[n] = (len(children[n]) + 1) * spectr_slack(host, b, n, T, len(children[n]))
    for n in range(1, N):
        m = parent[n]
        while m >= 0:
            tol[n] += slack[m]
            m = parent[m] if m > 0 else -1
    return tol


def fragile_tests(method, parent, children, updates):
    """Which nodes' test probabilities sit behind the rule's discontinuity (oracle numbers only).

    `updates` are the residual updates of orc.all_test_probs: (node, child, weight, mass), one per
    rejected child (subtree).  The update is continuous except in one corner: where the mass S of
    (a P - q)_+ vanishes, a weight of exactly 1 stays 1 while any weight below 1 drops to 0 (zero-mass
    rule), and S/(S + 1 - a) swings between the two as S and 1 - a trade places.  Only an update with
    S < FRAGILE_MASS and 1 - a < FRAGILE_MASS is that corner (SpecInfer: a = 1 throughout, so S alone).
    What it taints: the node's state from then on, i.e. the tests of the node's later children
    (and, Traversal, of everything below them, whose weights descend from the node's) and the
    node's own test.  Everything else is compared with the ordinary bar."""
    N = len(parent)
    fragile = np.zeros(N, dtype=bool)

    def taint_subtree(n):
        fragile[n] = True
        if method == orc.TRAVERSAL:
            for c in children[n]:
                taint_subtree(c)

    for node, child, weight, mass in updates:
        if mass < FRAGILE_MASS and 1.0 - weight < FRAGILE_MASS:
            for c in children[node]:
                if c > child:
                    taint_subtree(c)
            if method == orc.TRAVERSAL and node != 0:
                fragile[node] = True
                # the node's own final weight feeds nothing else: its parent's update uses the
                # parent's weight, not this one
    fragile[0] = False
    return fragile


def reach_of_tests(method, parent, children, probs):
    """Probability that each node's test is performed at all, given that the walk has got as far as
    it must (SpecInfer: the parent is reached and every earlier sibling was rejected; Traversal:
    everything earlier in depth-first post-order was rejected).  Oracle numbers."""
    N = len(parent)
    reach = np.ones(N)
    if method == orc.SPECINFER:
        for n in range(N):
            none_before = 1.0
            for c in children[n]:
                reach[c] = none_before
                none_before *= 1.0 - probs[c]
        return reach
    order = []

    def visit(n):
        for c in children[n]:
            visit(c)
        order.append(n)

    visit(0)
    none_before = 1.0
    for n in order:
        reach[n] = none_before
        none_before *= 1.0 - (1.0 if n == 0 else probs[n])
    reach[0] = 1.0
    return reach


# A float32 term 2^(z k - A) is good to about 1e-7 relative, so a residual mass, kept as the sum
# W(c) = sum (p - c q)_+ of differences of such terms over the ORIGINAL rows (the residual vector is
# never stored and never renormalised), carries an absolute error of up to SUM_REL_ERR (1 + c): each
# positive difference p_v - c q_v is off by up to SUM_REL_ERR (p_v + c q_v).  Whatever is computed
# from the state (c, W) then inherits a relative error of SUM_REL_ERR (1 + c) / W: nothing while the
# mass W of what is left of the target distribution is of order one, everything once it is of the
# order of the rounding itself.  REMOTE_FACTOR covers the handful of such terms that enter one test
# probability (the masses of the earlier rounds through c, the current one, the gathered term).
REMOTE_FACTOR = 8.0


def state_amplification(method, parent, children, updates):
    """For every node, the largest (1 + c) / W over the residual states its test probability is
    computed from, in the unnormalised form the kernels keep (c: what has been subtracted from the
    node's target row in units of its draft row; W: the mass left).  From the oracle's reported
    updates: a rejection at a node of weight a with relative mass S moves (c, W) to (c + W/a, S W/a).
    SpecInfer: each node's solver starts from (0, 1); a child's test uses the state after its earlier
    siblings.  Traversal: the same, a node's own test uses the state after all its children, and a
    child inherits what its starting weight was computed from."""
    N = len(parent)
    by_node = {}
    for node, child, weight, mass in updates:
        by_node.setdefault(node, {})[child] = (weight, mass)
    amp = np.ones(N)

    def walk(n, inherited):
        worst, c, W = inherited, 0.0, 1.0
        for child in children[n]:
            amp[child] = max(amp[child], worst)
            walk(child, worst if method == orc.TRAVERSAL else 1.0)
            if child in by_node.get(n, {}):
                a, S = by_node[n][child]
                if S > 0.0 and a > 0.0:
                    c, W = c + W / a, S * W / a
                    worst = max(worst, (1.0 + c) / W)
        if method == orc.TRAVERSAL:
            amp[n] = max(amp[n], worst)

    walk(0, 1.0)
    return amp


def remote_tolerance(method, parent, children, updates):
    """Bar for the "remote" test probabilities: PROB_ATOL + REMOTE_FACTOR * SUM_REL_ERR * (1 + c)/W
    (see above).  Where that exceeds SPECTR_SLACK_CAP the number is rounding noise of a mass far
    below float32 resolution: returned as inf (not compared, counted by the caller)."""
    tol = PROB_ATOL + REMOTE_FACTOR * SUM_REL_ERR * state_amplification(method, parent, children, updates)
    tol[tol > SPECTR_SLACK_CAP] = np.inf
    return tol


def result_to_host(res):
    out = {}
    for name in ("accept_len", "path_nodes", "path_tokens", "bonus_token", "counters",
                 "stats", "edge_probs", "accept_prob", "final_residual"):
        t = getattr(res, name)
        out[name] = None if t is None else t.cpu().numpy()
    return out


def compare_with_oracle(method, host, T, got, trees=None, check_debug=True):
    """host: dict from workloads.to_host; got: dict from result_to_host.

    Returns a report dict; raises AssertionError on any out-of-band difference.
    """
    parent = host["parent"]
    N = len(parent)
    B = host["tokens"].shape[0]
    trees = range(B) if trees is None else trees
    depth = orc.node_depths(parent)
    children = orc.children_lists(parent)
    report = {"trees": 0, "near_tie_paths": 0, "near_tie_bonus": 0, "fragile_tests": 0, "remote_tests": 0,
              "remote_over_flat_bar": 0, "noise_tests": 0, "max_prob_err": 0.0,
              "max_resid_err": 0.0, "max_stat_err": 0.0, "mean_accept_len": 0.0}
    for b in trees:
        tok = host["tokens"][b]
        zt, zd, u = host["target"][b], host["draft"][b], host["uniforms"][b]
        token_walk = method in (orc.NSS, orc.NAIVE, orc.SPECTR)
        ref = orc.verify_tree(method, parent, tok, zt, zd, T, u,
                              host["draw_uniforms"][b] if token_walk else None,
                              node_of=host.get("node_of"))     # trees of distinct contexts: see merged_tree_oracle
        report["trees"] += 1
        report["mean_accept_len"] += ref["accept_len"]
        g_len = int(got["accept_len"][b])
        g_nodes = [int(x) for x in got["path_nodes"][b][:g_len]]
        g_toks = [int(x) for x in got["path_tokens"][b][:g_len]]
        # structural validity of whatever the library returned
        assert all(int(x) == -1 for x in got["path_nodes"][b][g_len:]), f"tree {b}: padding"
        assert all(int(x) == -1 for x in got["path_tokens"][b][g_len:]), f"tree {b}: padding"
        stop_g = g_nodes[-1] if g_nodes else 0
        assert g_nodes == orc.path_to(parent, stop_g), f"tree {b}: path is not root-to-node"
        assert g_toks == [int(tok[n]) for n in g_nodes], f"tree {b}: path tokens"
        assert depth[stop_g] == g_len
        same_path = (g_nodes == ref["path_nodes"])
        slack = {}
        if method == orc.SPECTR:
            capped = []
            for node, _, _, _ in ref["decisions"]:
                par = parent[node]
                if par not in slack:
                    slack[par] = spectr_slack(host, b, par, T, len(children[par]), capped)
            report["capped_slacks"] = report.get("capped_slacks", 0) + len(capped)
        close_call = any(abs(a_ref - uu) < DECISION_BAND + slack.get(parent[node], 0.0)
                         for node, a_ref, uu, _ in ref["decisions"])
        worst_slack = max(slack.values(), default=0.0)
        if not same_path and token_walk and ref["bonus_gap"] < BONUS_BAND + worst_slack:
            report["near_tie_bonus"] += 1           # a draw on the way was within the band of a CDF step
        elif not same_path and close_call:
            report["near_tie_paths"] += 1
        elif not same_path:
            assert ref["min_margin"] < DECISION_BAND, (
                f"tree {b}: path {g_nodes} != oracle {ref['path_nodes']} and no oracle decision within "
                f"{DECISION_BAND} of its uniform (closest {ref['min_margin']:.3e})")
            report["near_tie_paths"] += 1
        else:
            g_bonus = int(got["bonus_token"][b])
            if g_bonus != ref["bonus_token"]:
                assert ref["bonus_gap"] < BONUS_BAND + worst_slack, (
                    f"tree {b}: bonus {g_bonus} != oracle {ref['bonus_token']}, "
                    f"gap to CDF step {ref['bonus_gap']:.3e}")
                report["near_tie_bonus"] += 1
            if check_debug and got.get("final_residual") is not None:
                err = float(np.max(np.abs(got["final_residual"][b].astype(np.float64) - ref["residual"])))
                report["max_resid_err"] = max(report["max_resid_err"], err)
                assert err <= PROB_ATOL + worst_slack, f"tree {b}: final residual differs by {err:.3e}"
        if not check_debug:
            continue
        if token_walk:
            # only the nodes the walk tested have a test probability
            if got.get("accept_prob") is not None and same_path:
                for node, a_ref, _, _ in ref["decisions"]:
                    err = abs(float(got["accept_prob"][b][node]) - a_ref)
                    tol = PROB_ATOL + slack.get(parent[node], 0.0)
                    report["max_prob_err"] = max(report["max_prob_err"], err)
                    assert err <= tol, (f"tree {b} node {node}: test probability differs by {err:.3e} "
                                        f"(allowed {tol:.3e})")
            continue
        if got.get("accept_prob") is not None:
            updates = []
            probs, _ = orc.all_test_probs(method, parent, tok, zt, zd, T, updates)
            fragile = fragile_tests(method, parent, children, updates)
            remote = (reach_of_tests(method, parent, children, probs) <= DECISION_BAND) & ~fragile
            plain = ~fragile & ~remote
            report["fragile_tests"] += int(np.count_nonzero(fragile))
            report["remote_tests"] += int(np.count_nonzero(remote))
            diff = np.abs(got["accept_prob"][b].astype(np.float64) - probs)
            err = float(np.max(diff[plain]))
            report["max_prob_err"] = max(report["max_prob_err"], err)
            assert err <= PROB_ATOL, (
                f"tree {b}: test probabilities differ by {err:.3e}\n got {got['accept_prob'][b]}\n ref {probs}")
            if np.any(remote):
                tol = remote_tolerance(method, parent, children, updates)
                report["noise_tests"] += int(np.count_nonzero(remote & np.isinf(tol)))
                report["remote_over_flat_bar"] += int(np.count_nonzero(remote & np.isfinite(tol) & (diff > PROB_ATOL)))
                bad = remote & (diff > tol)
                assert not np.any(bad), (
                    f"tree {b}: remote test probabilities of nodes {np.nonzero(bad)[0].tolist()} differ by "
                    f"{diff[bad].tolist()} (allowed {tol[bad].tolist()})")
        if got.get("edge_probs") is not None:
            for n in range(1, N):
                par = parent[n]
                p = orc.softmax_T(zt[par], T)[int(tok[n])]
                q = orc.softmax_T(zd[par], T)[int(tok[n])]
                e = got["edge_probs"][b][n].astype(np.float64)
                err = max(abs(e[0] - p), abs(e[1] - q))
                report["max_prob_err"] = max(report["max_prob_err"], float(err))
                assert err <= PROB_ATOL, f"tree {b} node {n}: edge probs {e} vs ({p}, {q})"
        if got.get("stats") is not None:
            for n in range(N):
                s = got["stats"][b][n].astype(np.float64)
                rows = [(zt[n], s[0], s[1])]
                if children[n]:
                    rows.append((zd[n], s[2], s[3]))
                else:
                    assert np.isnan(s[2]) and np.isnan(s[3])
                for z, m_g, lz_g in rows:
                    z = z.astype(np.float64)
                    m = z.max()
                    lz = np.log(np.sum(np.exp((z - m) / T)))
                    assert m_g == m, f"tree {b} node {n}: row maximum {m_g} vs {m}"
                    report["max_stat_err"] = max(report["max_stat_err"], abs(lz_g - lz))
                    assert abs(lz_g - lz) <= PROB_ATOL * max(1.0, abs(lz)), (
                        f"tree {b} node {n}: logZ {lz_g} vs {lz}")
    if report["trees"]:
        report["mean_accept_len"] /= report["trees"]
    return report


def check_properties(parent, V, got, tokens):
    """Size-independent validity checks for every tree of a batch (no oracle)."""
    depth = orc.node_depths(parent)
    maxd = max(depth)
    B = got["accept_len"].shape[0]
    al = got["accept_len"]
    assert al.min() >= 0 and al.max() <= maxd
    assert got["bonus_token"].min() >= 0 and got["bonus_token"].max() < V
    for b in range(B):
        ln = int(al[b])
        nodes = [int(x) for x in got["path_nodes"][b][:ln]]
        stop = nodes[-1] if nodes else 0
        assert nodes == orc.path_to(parent, stop)
        assert [int(x) for x in got["path_tokens"][b][:ln]] == [int(tokens[b][n]) for n in nodes]
        assert np.all(got["path_nodes"][b][ln:] == -1)
