"""CPU oracle (test infrastructure) for the multi-colour spanning trees of Section 4.2.

The paper: for each of the k colours the nodes are arranged in a k-ary BFS tree that spans
all nodes; the non-leaf nodes (root included) of different colours are disjoint; roots and
non-leaf nodes sum, leaves only send (Section 4.2 and Figure 2: 4 colours, 4-ary trees,
8 nodes; colour 0 rooted at node 0 with node 1 the only other non-leaf, colour 1 rooted at
node 2 with node 3).

The paper does not say how nodes are assigned to tree positions.  Reading taken: colour c
uses the node sequence rotated by c*s, where s is the number of non-leaf nodes one tree
needs; the tree is then filled breadth first, every parent taking the next k nodes of the
sequence.  A k-ary tree on n nodes has n-1 edges and at most k per parent, so it needs at
least ceil((n-1)/k) non-leaf nodes; disjoint sets for k colours therefore exist only if
k*ceil((n-1)/k) <= n, and this construction reaches that bound.

Only tests, the smoke check and the benchmark's CPU leg may import this module.
"""
from collections import deque
from typing import List, Optional


def non_leaves_needed(n_nodes: int, arity: int) -> int:
    """Fewest non-leaf nodes of any tree with n_nodes nodes and at most `arity` children each."""
    edges = n_nodes - 1
    return -(-edges // arity)


def feasible(n_nodes: int, k: int) -> bool:
    return n_nodes >= 1 and k >= 1 and k * non_leaves_needed(n_nodes, k) <= n_nodes


def colour_tree(n_nodes: int, k: int, c: int) -> List[int]:
    """parent[node] for colour c (-1 for the root), built by breadth-first filling."""
    s = non_leaves_needed(n_nodes, k)
    sequence = [(j + c * s) % n_nodes for j in range(n_nodes)]
    parent = [None] * n_nodes
    root = sequence[0]
    parent[root] = -1
    waiting = deque([root])           # nodes that may still take children, in BFS order
    nxt = 1
    while nxt < n_nodes:
        p = waiting.popleft()
        for _ in range(k):
            if nxt == n_nodes:
                break
            child = sequence[nxt]
            nxt += 1
            parent[child] = p
            waiting.append(child)
    return parent


def colour_trees(n_nodes: int, k: int) -> Optional[List[List[int]]]:
    """parent tables of all k colours, or None when disjoint non-leaf sets cannot exist."""
    if not feasible(n_nodes, k):
        return None
    return [colour_tree(n_nodes, k, c) for c in range(k)]


def children_of(parent: List[int], node: int) -> List[int]:
    return [r for r, p in enumerate(parent) if p == node]


def role(parent: List[int], node: int) -> str:
    if parent[node] == -1:
        return "root"
    return "inner" if children_of(parent, node) else "leaf"
