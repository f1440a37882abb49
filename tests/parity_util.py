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
  normalised residual) must agree within PROB_ATOL absolute.  Test probabilities of nodes
  whose test cannot be reached with probability above DECISION_BAND are left out (see
  reachable_tests).
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


def spectr_slack(host, b, node_parent, T, k):
    """Extra tolerance on the test probabilities of the children of node_parent (SpecTr)."""
    P = orc.softmax_T(host["target"][b][node_parent], T)
    Q = orc.softmax_T(host["draft"][b][node_parent], T)
    rho = orc.spectr_division_factor(P, Q, k)
    return SUM_REL_ERR * orc.spectr_conditioning(P, Q, k, rho)


def reachable_tests(method, parent, children, probs):
    """Which nodes' tests can be reached with probability above DECISION_BAND (oracle numbers).

    A node is tested only after certain other tests have failed (SpecInfer: its earlier
    siblings; Traversal: everything before it in depth-first post-order).  If one of those has
    an acceptance probability within the band of 1, the node's own test probability is the
    rule's state after an event that (nearly) cannot happen, and there the rule is not
    continuous: with zero residual mass the weight stays 1 if it was exactly 1 and drops to 0
    otherwise, so a weight of 1 - 1e-7 on one side and 1 on the other give 0 and 1.  Such test
    probabilities are not compared (they are counted); the decisions still are."""
    N = len(parent)
    live = np.ones(N, dtype=bool)
    if method == orc.SPECINFER:
        for n in range(N):
            none_before = 1.0
            for c in children[n]:
                live[c] = none_before > DECISION_BAND
                none_before *= 1.0 - probs[c]
        return live
    order = []

    def visit(n):
        for c in children[n]:
            visit(c)
        order.append(n)

    visit(0)
    none_before = 1.0
    for n in order:
        live[n] = none_before > DECISION_BAND
        none_before *= 1.0 - (1.0 if n == 0 else probs[n])
    live[0] = True
    return live


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
    report = {"trees": 0, "near_tie_paths": 0, "near_tie_bonus": 0, "max_prob_err": 0.0,
              "max_resid_err": 0.0, "max_stat_err": 0.0, "mean_accept_len": 0.0}
    for b in trees:
        tok = host["tokens"][b]
        zt, zd, u = host["target"][b], host["draft"][b], host["uniforms"][b]
        token_walk = method in (orc.NSS, orc.NAIVE, orc.SPECTR)
        ref = orc.verify_tree(method, parent, tok, zt, zd, T, u,
                              host["draw_uniforms"][b] if token_walk else None)
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
            for node, _, _, _ in ref["decisions"]:
                par = parent[node]
                if par not in slack:
                    slack[par] = spectr_slack(host, b, par, T, len(children[par]))
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
            probs, _ = orc.all_test_probs(method, parent, tok, zt, zd, T)
            live = reachable_tests(method, parent, children, probs)
            report["unreachable_tests"] = report.get("unreachable_tests", 0) + int(np.count_nonzero(~live))
            diff = np.abs(got["accept_prob"][b].astype(np.float64) - probs)
            err = float(np.max(diff[live]))
            report["max_prob_err"] = max(report["max_prob_err"], err)
            assert err <= PROB_ATOL, (
                f"tree {b}: test probabilities differ by {err:.3e}\n got {got['accept_prob'][b]}\n ref {probs}")
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
