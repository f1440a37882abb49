"""Parent arrays of the two tree families the paper drafts.

Node numbering: trunk first, then chain by chain, depth-first, so parent[n] < n
and the order of siblings is the order of the chains.
"""


def delayed_tree(K, L1, L2):
    """(K, L1, L2) delayed tree (Sec. 5, Def. 5.2): a trunk of L1 nodes, then K
    chains of L2 nodes under the last trunk node.  N = 1 + L1 + K*L2."""
    if K < 1 or L1 < 0 or L2 < 0:
        raise ValueError("need K >= 1, L1 >= 0, L2 >= 0")
    parent = [-1]
    last = 0
    for _ in range(L1):
        parent.append(last)
        last = len(parent) - 1
    for _ in range(K):
        prev = last
        for _ in range(L2):
            parent.append(prev)
            prev = len(parent) - 1
    return parent


def root_tree(K, L):
    """K i.i.d. paths of length L from the root (Sec. 3.2).  N = 1 + K*L."""
    return delayed_tree(K, 0, L)


def tree_depth(parent):
    depth = [0] * len(parent)
    for n in range(1, len(parent)):
        depth[n] = depth[parent[n]] + 1
    return max(depth)
