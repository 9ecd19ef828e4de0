"""Makespan model of one MoE layer under a circuit schedule -- TEST INFRASTRUCTURE ONLY (CPU oracle).

Section 5 (Setup, "Execution time"): the completion time of a matching is its largest transfer
divided by the link bandwidth; expert computation of matching i begins when its dispatch has
completed, while the communication of matching i+1 proceeds; without overlap communication and
computation run strictly one after the other.  The idealised congestion-free all-to-all
completes in (largest row or column sum) / bandwidth.  Expert time comes either from a measured
table of time against rows ("profiling-based") or from a linear model.

Readings where the paper is silent (event order of its simulator is not given):
  * one circuit configuration is active at a time; every change of configuration costs `reconf`;
  * matching t ships min(remaining entry, duration_t) on each of its pairs (duration = cap of a
    circuit's hold time, in tokens);
  * tokens whose expert is local (the diagonal) need no circuit and are computed first;
  * what the (capped) schedule leaves is served as one conventional round that lasts
    (largest line sum of the residual) / bandwidth, after the matchings;
  * combine sends every result back over the same pairs: it costs what the dispatch cost and
    needs the network; with overlap the network first serves all dispatches in order, then the
    combines in order, each as soon as the network is free and every rank has finished that
    slice; a rank computes its slices in arrival order, one at a time;
  * the layer ends when the last combine ends.

Plain Python loops, float64.  Nothing here is shared with the library's own implementation.
"""
from __future__ import annotations

import numpy as np


def expert_time(rows: float, model: dict) -> float:
    """Seconds one rank needs for `rows` (token, expert) rows; 0 rows cost nothing."""
    if rows <= 0:
        return 0.0
    if model["kind"] == "linear":
        return model["fixed"] + model["per_row"] * rows
    xs, ys = model["rows"], model["seconds"]          # measured table, rows ascending
    if rows <= xs[0]:
        return ys[0]                                  # the floor of a small batch (Section 2.2, Figure 1)
    for a in range(len(xs) - 1):
        if rows <= xs[a + 1]:
            w = (rows - xs[a]) / (xs[a + 1] - xs[a])
            return ys[a] + w * (ys[a + 1] - ys[a])
    slope = (ys[-1] - ys[-2]) / (xs[-1] - xs[-2])     # beyond the table: continue the last segment
    return ys[-1] + slope * (rows - xs[-1])


def shipped_amounts(traffic, perms, durations):
    """(ship[t][j] = rows rank j receives in matching t, residual matrix, local rows per rank)."""
    A = np.array(traffic, dtype=np.int64)
    n = A.shape[0]
    local = np.diag(A).copy()
    R = A.copy()
    np.fill_diagonal(R, 0)
    ship = np.zeros((len(perms), n), dtype=np.int64)
    for t, sigma in enumerate(perms):
        for i in range(n):
            j = int(sigma[i])
            if i == j:
                continue
            s = min(int(R[i][j]), int(durations[t]))
            R[i][j] -= s
            ship[t][j] = s
    return ship, R, local


def makespan(traffic, perms, durations, bytes_per_row, bandwidth, reconf, model, order=None):
    """Returns dict(sequential, overlap, ideal, comm, compute) in seconds."""
    ship, R, local = shipped_amounts(traffic, perms, durations)
    n = len(local)
    K = len(perms)
    order = list(range(K)) if order is None else [int(o) for o in order]
    assert sorted(order) == list(range(K))
    # communication phases: the K matchings in the given order, then the residual round if anything is left
    comm = [reconf + float(durations[t]) * bytes_per_row / bandwidth for t in order]
    rows = [ship[t] for t in order]
    res_line = max(int(R.sum(axis=0).max()), int(R.sum(axis=1).max())) if n else 0
    if res_line > 0:
        comm.append(reconf + res_line * bytes_per_row / bandwidth)
        rows.append(R.sum(axis=0))
    P = len(comm)
    ctime = [[expert_time(float(rows[p][j]), model) for j in range(n)] for p in range(P)]
    ltime = [expert_time(float(local[j]), model) for j in range(n)]

    # ---- no overlap: local compute, then per phase dispatch -> compute -> combine
    seq = max(ltime) if n else 0.0
    for p in range(P):
        seq += comm[p] + max(ctime[p]) + comm[p]

    # ---- overlap
    net = 0.0
    ready = []
    for p in range(P):
        net += comm[p]
        ready.append(net)
    rank_free = list(ltime)
    done = []
    for p in range(P):
        finish = 0.0
        for j in range(n):
            if rows[p][j] > 0:
                start = max(ready[p], rank_free[j])
                rank_free[j] = start + ctime[p][j]
                finish = max(finish, rank_free[j])
            else:
                finish = max(finish, ready[p])
        done.append(finish)
    for p in range(P):
        net = max(net, done[p]) + comm[p]
    over = max([net] + rank_free) if n else 0.0

    # ---- idealised congestion-free all-to-all, no overlap
    A = np.array(traffic, dtype=np.int64)
    off = A.copy()
    np.fill_diagonal(off, 0)
    tstar = max(int(off.sum(axis=0).max()), int(off.sum(axis=1).max())) if n else 0
    a2a = tstar * bytes_per_row / bandwidth
    ideal = 2 * a2a + max(expert_time(float(A[:, j].sum()), model) for j in range(n)) if n else 0.0
    return dict(sequential=seq, overlap=over, ideal=ideal, comm=sum(comm), compute=sum(max(c) for c in ctime) + (max(ltime) if n else 0.0))


def johnson_order(traffic, perms, durations, bytes_per_row, bandwidth, reconf, model):
    """Order of the matchings by Johnson's rule for the two-stage flow shop dispatch -> compute
    (Section 4, "ordering of matchings" as a flow-shop problem): matchings whose dispatch is not
    longer than their compute first, by increasing dispatch time; the others after them, by
    decreasing compute time.  Ties keep the original order."""
    ship, _, _ = shipped_amounts(traffic, perms, durations)
    K = len(perms)
    a = [reconf + float(durations[t]) * bytes_per_row / bandwidth for t in range(K)]
    b = [max(expert_time(float(x), model) for x in ship[t]) for t in range(K)]
    first = sorted([t for t in range(K) if a[t] <= b[t]], key=lambda t: (a[t], t))
    second = sorted([t for t in range(K) if a[t] > b[t]], key=lambda t: (-b[t], t))
    return first + second
