"""TEST INFRASTRUCTURE.  Plain Python statements of the host-side steps that sit next to the hot
path: the partition of a computation DAG into sequential sub-graphs (Appendix B, Algorithm 2 of
the paper) taken step by step in the paper's order, and the Prefix / Random baseline strategies
of Sec. 3.1.  Imported by tests only; shares nothing with the library.

Readings of Algorithm 2 where the printed listing is loose:
  * "Run BFS and denote the longest path from the start to each vertex": a longest path needs the
    vertices in topological order, so path lengths are computed that way.
  * The frontier A is a set; the vertices picked for expansion in one sweep are those that were in
    A when the sweep began (the listing mutates A while iterating over it); next[v'] is added
    vertex by vertex.
"""


def longest_paths(n, edges):
    succ = [[] for _ in range(n)]
    indeg = [0] * n
    for a, b in edges:
        succ[a].append(b)
        indeg[b] += 1
    start = [v for v in range(n) if indeg[v] == 0]
    assert len(start) == 1
    order, plen = [start[0]], [0] * n
    deg = list(indeg)
    for v in order:
        for w in succ[v]:
            plen[w] = max(plen[w], plen[v] + 1)
            deg[w] -= 1
            if deg[w] == 0:
                order.append(w)
    assert len(order) == n, "cycle"
    return start[0], succ, plen


def partition_sequential(n, edges, quantizable=None):
    """Returns the list of groups (lists of vertices, quantisable ones only, in no particular order)."""
    start, succ, plen = longest_paths(n, edges)
    ends = [v for v in range(n) if not succ[v]]
    assert len(ends) == 1
    end = ends[0]
    groups = []
    v = start
    while v != end:
        group = set()
        cur_len = plen[v] + 1
        frontier = set(succ[v])
        while len(frontier) > 1:
            for w in sorted(frontier):                       # the sweep's snapshot of A
                if plen[w] <= cur_len:
                    frontier.discard(w)
                    group.add(w)
                    frontier.update(succ[w])
            cur_len += 1
        v = frontier.pop()
        group.add(v)
        if quantizable is not None:
            group = {w for w in group if quantizable[w]}
        if group:
            groups.append(sorted(group))
    return groups


def select_ordered(n_choices, gain, mse, budget, order=None):
    """Walk the groups in `order`; take a group's largest-gain choice while the budget holds; stop
    at the first group that does not fit.  Returns (choice, total_gain, total_mse) or None."""
    J = len(n_choices)
    off = [0]
    for nc in n_choices:
        off.append(off[-1] + nc)
    choice = [0] * J
    d = sum(mse[off[j]] for j in range(J))
    if d > budget:
        return None
    for j in (range(J) if order is None else order):
        best = 0
        for p in range(1, n_choices[j]):
            gp, gb = gain[off[j] + p], gain[off[j] + best]
            if gp > gb or (gp == gb and mse[off[j] + p] < mse[off[j] + best]):
                best = p
        nd = d - mse[off[j]] + mse[off[j] + best]
        if nd > budget:
            break
        d = nd
        choice[j] = best
    g = sum(gain[off[j] + choice[j]] for j in range(J))
    return choice, g, d
