"""A whole multi-colour Allreduce + SGD step simulated rank by rank (Section 3, Algorithm 1
and Section 4.2), driven through a `roles_call` that is either the CPU oracle's or the GPU
library's per-rank operation.  Used to check that the per-rank pieces compose to the plain
sum of all contributions and to identical weights on every node."""
import numpy as np


def simulate(roles_call, parents, m, local, w0, v0, N, k, lr, mu, wd):
    """parents[c][node] = parent of node in colour c's tree (-1 root).
    local[node][j] = flat contribution of GPU j of that node (length N).
    Returns (g_total, w[node], v[node]) with g_total assembled from the roots' colours."""
    n = len(parents[0])
    kids = [[[r for r in range(n) if parents[c][r] == node] for c in range(k)] for node in range(n)]
    depth = [[0] * n for _ in range(k)]
    for c in range(k):
        for r in range(n):
            cur, d = r, 0
            while parents[c][cur] != -1:
                cur, d = parents[c][cur], d + 1
            depth[c][r] = d
    P = m + k                                   # m local replicas + up to k child buffers
    zero = np.zeros(N, np.float32)
    partial = [np.full(N, np.nan, np.float32) for _ in range(n)]   # what each node hands upward
    w = [w0.copy() for _ in range(n)]
    v = [v0.copy() for _ in range(n)]
    g_total = np.full(N, np.nan, np.float32)

    def order_for(node):
        rows = []
        for c in range(k):
            used = list(range(m)) + [m + j for j in range(len(kids[node][c]))]
            rows.append(used + [q for q in range(P) if q not in used])
        return np.array(rows, np.int32)

    # phase 1: every node, its leaf colours: sum of the m local replicas only
    for node in range(n):
        n_terms = [m if not kids[node][c] and parents[c][node] != -1 else 0 for c in range(k)]
        if any(n_terms):
            roles_call(local[node] + [zero] * k, n_terms, [0] * k, partial[node], None, None,
                       lr, mu, wd, order_for(node))
    # phase 2: inner nodes bottom-up, roots last (with the update)
    maxd = max(max(d) for d in depth)
    for d in range(maxd, -1, -1):
        for node in range(n):
            n_terms, upd = [0] * k, [0] * k
            for c in range(k):
                is_root = parents[c][node] == -1
                if depth[c][node] == d and (kids[node][c] or is_root):
                    if kids[node][c] or is_root:
                        n_terms[c] = m + len(kids[node][c])
                        upd[c] = 1 if is_root else 0
            if not any(n_terms):
                continue
            child_bufs = [zero] * k
            for c in range(k):
                if n_terms[c]:
                    child_bufs = [partial[ch] for ch in kids[node][c]] + [zero] * (k - len(kids[node][c]))
            assert sum(1 for c in range(k) if n_terms[c] and kids[node][c]) <= 1
            out = partial[node]
            roles_call(local[node] + child_bufs, n_terms, upd, out, w[node], v[node],
                       lr, mu, wd, order_for(node))
    # the roots hold the complete sums; "broadcast" them and update everywhere else
    bounds = roles_call.bounds
    for c in range(k):
        root = parents[c].index(-1)
        lo, hi = int(bounds[c]), int(bounds[c + 1])
        g_total[lo:hi] = partial[root][lo:hi]
    for node in range(n):
        n_terms = [0 if parents[c][node] == -1 else 1 for c in range(k)]
        if any(n_terms):
            scratch = np.empty(N, np.float32)
            roles_call([g_total] + [zero] * (P - 1), n_terms, [1] * k, scratch, w[node], v[node],
                       lr, mu, wd, None)
    return g_total, w, v


def tree_order_sum(parents_c, m, local, lo, hi):
    """Independent restatement in numpy: the value colour c's root ends up with when every
    node adds its m replicas left to right and then its children's partial sums in order."""
    n = len(parents_c)

    def partial(node):
        acc = local[node][0][lo:hi].copy()
        for j in range(1, m):
            acc = acc + local[node][j][lo:hi]
        for ch in [r for r in range(n) if parents_c[r] == node]:
            acc = acc + partial(ch)
        return acc
    return partial(parents_c.index(-1))
