"""TEST INFRASTRUCTURE.  Plain Python statements of the host-side steps that sit next to the hot
path: the partition of a computation DAG into sequential sub-graphs (Appendix B of the paper) and
the Prefix / Random baseline strategies of Sec. 3.1.  Imported by tests only; shares nothing with
the library.

The partition is written from what a sequential sub-graph is (Sec. 2.3.1 and Appendix B: a region
with a single entry and a single exit, so that everything before it is finished when it starts and
everything after it waits for its last vertex), not from the appendix's listing: a vertex closes a
group iff every path from the start vertex to the sink passes through it, which is decided here by
brute force (take the vertex out and see whether the sink can still be reached); every other vertex
belongs to the first closing vertex it leads to.
"""


def _reachable(succ, src, banned=None):
    """Vertices reachable from src (src included) without stepping on `banned`."""
    seen = {src}
    stack = [src]
    while stack:
        v = stack.pop()
        for w in succ[v]:
            if w != banned and w not in seen:
                seen.add(w)
                stack.append(w)
    return seen


def partition_sequential(n, edges, quantizable=None):
    """Returns the list of groups (sorted lists of vertices, quantisable ones only) in execution order."""
    succ = [[] for _ in range(n)]
    has_pred = [False] * n
    for a, b in edges:
        succ[a].append(b)
        has_pred[b] = True
    starts = [v for v in range(n) if not has_pred[v]]
    sinks = [v for v in range(n) if not succ[v]]
    assert len(starts) == 1 and len(sinks) == 1
    start, sink = starts[0], sinks[0]
    reach = [_reachable(succ, v) for v in range(n)]
    # closing vertices: without them the sink is cut off from the start (the sink itself is one)
    closing = [v for v in range(n)
               if v != start and (v == sink or sink not in _reachable(succ, start, banned=v))]
    # every path meets all of them, so they are totally ordered: c comes before c' iff c leads to c'
    closing.sort(key=lambda c: sum(1 for c2 in closing if c2 in reach[c]), reverse=True)
    groups = [[] for _ in closing]
    for v in range(n):
        if v == start:
            continue
        first = next(i for i, c in enumerate(closing) if c in reach[v])
        if quantizable is None or quantizable[v]:
            groups[first].append(v)
    return [sorted(g) for g in groups if g]


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
