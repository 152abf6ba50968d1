"""Oracle D: from rollout token sequences to the prefix tree, and the paper's
load-balanced DFS-contiguous partitioning.  TEST INFRASTRUCTURE ONLY (never
imported by the product path).  Integer work; results must match bit for bit.

Prefix tree (paper section 3, problem formulation): N rollouts whose shared
prefixes are merged; nodes are token segments, root-to-node paths are the
sequences.  Written here as the plain definition: put every sequence into a
token-by-token trie, then merge every chain of single-child, non-terminal trie
nodes into one segment.  A node therefore ends exactly where sequences branch
or where a sequence ends (a rollout contained in a longer one ends at an
interior node; the paper's algorithms assume leaves, see the notation block of
the pseudocode appendix).  Canonical numbering: DFS preorder with children in
ascending order of their first token, which is the lexicographic order of the
sequences (section 4: lexicographic order is a valid DFS order).

Partitioning (pseudocode appendix, algorithm "Load-Balanced DFS-Contiguous
Partitioning"; section 4): sequences in lexicographic order pi, the cost of a
contiguous group is the number of tree tokens it needs, |pi_a| + sum over the
rest of (|pi_i| - LCP(pi_{i-1}, pi_i)); binary search on the largest group cost
tau with a greedy feasibility scan, then groups are split until there are K.
The steps below are the algorithm's, in its order and notation; where it says
"split any non-singleton interval" the first such interval is split after its
first element.

Pinned in tests/test_oracle_pins.py: expanding the tree's root-to-node paths
gives back every input sequence; T equals the appendix's formula
|pi_1| + sum(|pi_i| - LCP); brute force over all contiguous K-partitions gives
the same largest group cost; the duplicated-token bound of section 4.
"""
from __future__ import annotations


def lcp(a, b):
    """Length of the longest common prefix of two sequences."""
    n = min(len(a), len(b))
    i = 0
    while i < n and a[i] == b[i]:
        i += 1
    return i


def lexicographic_order(seqs):
    """Indices of seqs in lexicographic order (a proper prefix sorts first;
    equal sequences keep their input order)."""
    return sorted(range(len(seqs)), key=lambda i: (tuple(seqs[i]), i))


def build_tree(seqs):
    """Returns dict(parent, seg_len, tokens, seq_node, order):
    parent[u], seg_len[u] in canonical DFS numbering; tokens = the packed token
    ids of all nodes in that order (length T); seq_node[i] = node at which input
    sequence i ends; order = lexicographic_order(seqs).  Sequences must be
    non-empty."""
    # token-by-token trie: node = [children dict, terminal flag]
    root = [{}, False]
    ends = []
    for s in seqs:
        if len(s) == 0:
            raise ValueError("empty sequence")
        cur = root
        for tok in s:
            cur = cur[0].setdefault(int(tok), [{}, False])
        cur[1] = True
        ends.append(cur)
    parent, seg_len, tokens = [], [], []
    node_of = {}          # id(trie node at which a segment ends) -> tree node

    def emit(trie_node, first_tok, par):
        """Segment starting with the edge `first_tok` into trie_node."""
        seg = [first_tok]
        while len(trie_node[0]) == 1 and not trie_node[1]:
            (tok, nxt), = trie_node[0].items()
            seg.append(tok)
            trie_node = nxt
        u = len(parent)
        parent.append(par)
        seg_len.append(len(seg))
        tokens.extend(seg)
        node_of[id(trie_node)] = u
        for tok in sorted(trie_node[0]):
            emit(trie_node[0][tok], tok, u)

    import sys
    sys.setrecursionlimit(max(10000, sys.getrecursionlimit()))
    for tok in sorted(root[0]):
        emit(root[0][tok], tok, -1)
    return dict(parent=parent, seg_len=seg_len, tokens=tokens,
                seq_node=[node_of[id(e)] for e in ends], order=lexicographic_order(seqs))


def group_cost(sorted_seqs, a, b):
    """Tree tokens needed by the contiguous group pi_a .. pi_b (inclusive, 0-based)."""
    c = len(sorted_seqs[a])
    for i in range(a + 1, b + 1):
        c += len(sorted_seqs[i]) - lcp(sorted_seqs[i - 1], sorted_seqs[i])
    return c


def partition(seqs, K):
    """Returns (order, cuts): cuts = K inclusive index ranges (a, b) into the
    lexicographic order.  Requires 1 <= K <= len(seqs)."""
    order = lexicographic_order(seqs)
    pi = [seqs[i] for i in order]
    N = len(pi)
    if not (1 <= K <= N):
        raise ValueError("need 1 <= K <= number of sequences")

    def feasible(tau):
        if max(len(s) for s in pi) > tau:
            return False, []
        m, a, c, cuts = 1, 0, len(pi[0]), []
        for i in range(1, N):
            delta = len(pi[i]) - lcp(pi[i - 1], pi[i])
            if c + delta > tau:
                cuts.append((a, i - 1))
                m, a, c = m + 1, i, len(pi[i])
            else:
                c += delta
        cuts.append((a, N - 1))
        return m <= K, cuts

    L = max(len(s) for s in pi)
    R = len(pi[0]) + sum(len(pi[i]) - lcp(pi[i - 1], pi[i]) for i in range(1, N))
    while L < R:
        tau = (L + R) // 2
        ok, _ = feasible(tau)
        if ok:
            R = tau
        else:
            L = tau + 1
    _, cuts = feasible(L)
    while len(cuts) < K:
        j = next(i for i, (a, b) in enumerate(cuts) if b > a)
        a, b = cuts[j]
        cuts[j:j + 1] = [(a, a), (a + 1, b)]
    return order, cuts
