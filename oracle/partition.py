"""Oracle for the partition structure and a naive partition-wise evaluator.

TEST INFRASTRUCTURE ONLY (see ``oracle/__init__.py``).

What the paper fixes and this file writes out:

* a partition owns its destination vertices; its gathered input ``GA_p`` is the union of the
  source vertices of all of them (Cache-(Re)Gather-Bypass section, "(Re)gather" item);
* the cross-partition part of that union is ordered by partition id, then vertex id
  (appendix "In-Partition Vertex Ordering for Sequential Accesses");
* expansion ratio ``alpha`` = required vertices / target vertices (appendix "Effect of
  Partitioning on Host<->GPU Traffic");
* forward of a partition: gather, aggregate along ``T_p``, transform; backward: regather,
  recompute the aggregate, produce the gradient of the gathered rows and scatter-accumulate
  it onto the owners, weight gradients summed over partitions (overall-procedure algorithm
  in the appendix);
* first/second preference of a vertex and the size penalty of the label-propagation
  partitioner (partitioning section and its appendix).

The paper's partitioner is multi-threaded and randomly initialised, so it defines no unique
assignment.  The two deterministic rules below are this build's reading; they are written so
that an independent implementation can reproduce them bit for bit.
"""
from __future__ import annotations

import numpy as np

MASK64 = (1 << 64) - 1


# ----------------------------------------------------------------------------------------
# assignment rules
# ----------------------------------------------------------------------------------------
def splitmix64(x: int) -> int:
    """One output of the SplitMix64 generator whose state before the step is ``x``."""
    z = (x + 0x9E3779B97F4A7C15) & MASK64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & MASK64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & MASK64
    return z ^ (z >> 31)


def assign_random(n: int, k: int, seed: int) -> np.ndarray:
    """Random-balanced rule: sort vertices by ``(key(v), v)`` with
    ``key(v) = splitmix64(seed xor splitmix64(v))``; the vertex at rank ``r`` goes to
    partition ``r mod k``.  Partition sizes differ by at most one."""
    keys = [(splitmix64((seed & MASK64) ^ splitmix64(v)), v) for v in range(n)]
    keys.sort()
    part = np.empty(n, dtype=np.int32)
    for r, (_, v) in enumerate(keys):
        part[v] = r % k
    return part


def preferences(neigh_parts, k: int):
    """Partitions ordered by how often they occur among a vertex's neighbours (most frequent
    first, lower id first among equals); partitions that do not occur are left out."""
    cnt = np.bincount(np.asarray(neigh_parts, dtype=np.int64), minlength=k)
    order = sorted((j for j in range(k) if cnt[j] > 0), key=lambda j: (-cnt[j], j))
    return order


def lp_targets(rowptr, colidx, part, k: int) -> np.ndarray:
    """Target partition of every vertex for one label-propagation round, from a frozen state.

    The paper scores partition ``j`` for vertex ``v`` with
    ``1 + #N(v,j)/#N(v,.) - |P_j| / (1.1 |V| / k)``.  Dropping the constant and multiplying
    by ``11 |V| #N(v,.)`` gives the integer key ``11 |V| #N(v,j) - 10 k #N(v,.) |P_j|``,
    which orders the partitions in the same way and makes ties exact.  ``N(v)`` is row ``v``
    of the CSR without ``v`` itself.  Ties go to the current partition if it is among the
    best, else to the lowest id.
    """
    n = len(rowptr) - 1
    sizes = np.bincount(part, minlength=k).astype(np.int64)
    target = np.array(part, dtype=np.int32, copy=True)
    for v in range(n):
        nb = colidx[rowptr[v]:rowptr[v + 1]]
        nb = nb[nb != v]
        deg = len(nb)
        cnt = np.bincount(part[nb], minlength=k).astype(np.int64)
        key = 11 * n * cnt - 10 * k * deg * sizes
        best = key.max()
        if key[part[v]] == best:
            target[v] = part[v]
        else:
            target[v] = int(np.flatnonzero(key == best)[0])
    return target


def lp_targets_fast(rowptr, colidx, part, k: int) -> np.ndarray:
    """Same result as :func:`lp_targets`, vectorised with a dense ``[n, k]`` count table so
    that mid-size graphs finish in seconds."""
    n = len(rowptr) - 1
    sizes = np.bincount(part, minlength=k).astype(np.int64)
    rows = np.repeat(np.arange(n, dtype=np.int64), np.diff(rowptr))
    cols = np.asarray(colidx, dtype=np.int64)
    keep = rows != cols
    rows, cols = rows[keep], cols[keep]
    cnt = np.bincount(rows * k + part[cols], minlength=n * k).reshape(n, k).astype(np.int64)
    deg = cnt.sum(axis=1)
    key = 11 * n * cnt - 10 * k * deg[:, None] * sizes[None, :]
    best = key.max(axis=1)
    first = np.argmax(key == best[:, None], axis=1)
    cur = np.asarray(part, dtype=np.int64)
    stay = key[np.arange(n), cur] == best
    return np.where(stay, cur, first).astype(np.int32)


def assign_lp(rowptr, colidx, k: int, seed: int, rounds: int = 10, fast: bool = True):
    """Edge-cut rule: start from :func:`assign_random`; each round computes every vertex's
    target from the frozen state, then one sweep in ascending vertex id moves ``v`` to its
    target when that partition currently holds fewer than ``floor(1.1 |V| / k)`` vertices
    (the paper's capacity limit with the balance factor 1.1)."""
    n = len(rowptr) - 1
    part = assign_random(n, k, seed) if n < 200_000 else assign_random_fast(n, k, seed)
    cap = (11 * n) // (10 * k)
    for _ in range(rounds):
        tgt = (lp_targets_fast if fast else lp_targets)(rowptr, colidx, part, k)
        sizes = np.bincount(part, minlength=k).astype(np.int64)
        for v in np.flatnonzero(tgt != part):
            j = int(tgt[v])
            if sizes[j] < cap:
                sizes[part[v]] -= 1
                sizes[j] += 1
                part[v] = j
    return part


def assign_random_fast(n: int, k: int, seed: int) -> np.ndarray:
    """:func:`assign_random` with numpy uint64 arithmetic (wraps modulo 2**64)."""
    def sm(x):
        with np.errstate(over="ignore"):
            z = x + np.uint64(0x9E3779B97F4A7C15)
            z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
            z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
            return z ^ (z >> np.uint64(31))
    v = np.arange(n, dtype=np.uint64)
    key = sm(np.uint64(seed & MASK64) ^ sm(v))
    order = np.lexsort((v, key))
    part = np.empty(n, dtype=np.int32)
    part[order] = (np.arange(n) % k).astype(np.int32)
    return part


# ----------------------------------------------------------------------------------------
# switching-aware partitioner, complete procedure (partitioning section; appendix "Insights
# and Details" of the partitioner; convergence table in the appendix)
# ----------------------------------------------------------------------------------------
FRAC_ONE = 1 << 20          # fixed-point scale of #N(v,j)/#N(v,.) in the exact objective


def switching_preferences(nb_parts, cur: int, n: int, k: int, sizes):
    """First and second preference of a vertex whose neighbours lie in ``nb_parts``.

    The partitions a vertex can prefer are those that occur among its neighbours, plus the
    one it is in.  They are ranked by the paper's score ``1 + #N(v,j)/#N(v,.) - Penalty_j``
    in the exact integer form used by :func:`lp_targets`; equal scores rank the current
    partition first, then the lower id.  The second preference is ``-1`` when only one
    partition can be preferred."""
    nb_parts = np.asarray(nb_parts, dtype=np.int64)
    deg = len(nb_parts)
    cnt = np.bincount(nb_parts, minlength=k)
    domain = sorted(set(int(j) for j in nb_parts) | {int(cur)})
    ranked = sorted(domain, key=lambda j: (-(11 * n * int(cnt[j]) - 10 * k * deg * int(sizes[j])),
                                           0 if j == cur else 1, j))
    return ranked[0], (ranked[1] if len(ranked) > 1 else -1)


def switching_objective(rowptr, colidx, part, k: int) -> int:
    """The partitioner's objective ``sum_v Score(v, partition_v)`` as an exact integer:
    ``11 |V| * sum_v (2^20 + floor(2^20 #N(v,p_v) / #N(v,.))) - 10 k 2^20 sum_j |P_j|^2``
    (the score times ``11 |V| 2^20``, the neighbour fraction rounded down to 20 fractional
    bits and taken as 0 for a vertex without neighbours)."""
    n = len(rowptr) - 1
    sizes = np.bincount(part, minlength=k)
    total = 0
    for v in range(n):
        nb = colidx[rowptr[v]:rowptr[v + 1]]
        nb = nb[nb != v]
        frac = 0
        if len(nb):
            frac = (FRAC_ONE * int(np.count_nonzero(part[nb] == part[v]))) // len(nb)
        total += FRAC_ONE + frac
    return 11 * n * total - 10 * k * FRAC_ONE * sum(int(x) * int(x) for x in sizes)


def worker_capacity(rc: int, workers: int, w: int) -> int:
    """Share of a partition's relocation capacity ``rc`` given to worker ``w``: an equal
    split, the remainder going to the first workers."""
    return rc // workers + (1 if w < rc % workers else 0)


def switching_iteration(rowptr, colidx, part, k: int, workers: int):
    """One iteration from the frozen state ``part``; returns the new assignment.

    Relocation capacity of partition ``j``: ``RC_j = floor(1.1 |V| / k) - |P_j|`` (not below
    zero).  The vertices are split into ``workers`` contiguous ranges
    ``[floor(w |V| / W), floor((w+1) |V| / W))``; each worker keeps, per partition ``j``, the
    list of its vertices whose first preference is ``j`` and differs from where they are,
    groups that list by second preference, and relocates the largest group (ties: the lower
    second preference, "none" lowest) in ascending vertex id, at most its share of ``RC_j``."""
    n = len(rowptr) - 1
    part = np.asarray(part, dtype=np.int32)
    sizes = np.bincount(part, minlength=k).astype(np.int64)
    cap = (11 * n) // (10 * k)
    new = part.copy()
    for w in range(workers):
        lo, hi = (w * n) // workers, ((w + 1) * n) // workers
        lists = [dict() for _ in range(k)]          # per target partition: second pref -> vertices
        for v in range(lo, hi):
            nb = colidx[rowptr[v]:rowptr[v + 1]]
            nb = nb[nb != v]
            first, second = switching_preferences(part[nb], int(part[v]), n, k, sizes)
            if first != part[v]:
                lists[first].setdefault(second, []).append(v)
        for j in range(k):
            if not lists[j]:
                continue
            room = worker_capacity(max(0, cap - int(sizes[j])), workers, w)
            g = min(lists[j], key=lambda sec: (-len(lists[j][sec]), sec))
            for v in lists[j][g][:room]:
                new[v] = j
    return new


def assign_switching(rowptr, colidx, k: int, seed: int, workers: int = 8, max_iters: int = 50,
                     window: int = 5, iteration=None, objective=None):
    """The complete partitioner: random start, iterations of :func:`switching_iteration`,
    halting when the objective has improved by less than 0.1 % of its previous value in
    ``window`` consecutive iterations, after ``max_iters`` iterations at the latest.
    Returns the assignment and the list of objective values (initial state first)."""
    iteration = iteration or switching_iteration
    objective = objective or switching_objective
    n = len(rowptr) - 1
    part = assign_random(n, k, seed) if n < 200_000 else assign_random_fast(n, k, seed)
    hist = [objective(rowptr, colidx, part, k)]
    streak = 0
    for _ in range(max_iters):
        part = iteration(rowptr, colidx, part, k, workers)
        hist.append(objective(rowptr, colidx, part, k))
        small = 1000 * (hist[-1] - hist[-2]) < abs(hist[-2])
        streak = streak + 1 if small else 0
        if streak == window:
            break
    return part, hist


def _count_table(rowptr, colidx, part, k):
    n = len(rowptr) - 1
    rows = np.repeat(np.arange(n, dtype=np.int64), np.diff(rowptr))
    cols = np.asarray(colidx, dtype=np.int64)
    keep = rows != cols
    rows, cols = rows[keep], cols[keep]
    return np.bincount(rows * k + part[cols], minlength=n * k).reshape(n, k).astype(np.int64)


def switching_iteration_fast(rowptr, colidx, part, k: int, workers: int):
    """Same result as :func:`switching_iteration` with a dense ``[n, k]`` count table."""
    n = len(rowptr) - 1
    part = np.asarray(part, dtype=np.int32)
    cur = part.astype(np.int64)
    sizes = np.bincount(part, minlength=k).astype(np.int64)
    cnt = _count_table(rowptr, colidx, part, k)
    deg = cnt.sum(axis=1)
    ar = np.arange(n)
    key = 11 * n * cnt - 10 * k * deg[:, None] * sizes[None, :]
    allowed = cnt > 0
    allowed[ar, cur] = True
    # rank by (key desc, current first, id asc): fold the tie-breaks into one sortable value
    lowest = key.min() - 1
    keyd = np.where(allowed, key, lowest)
    def best(keyd):
        m = keyd.max(axis=1)
        tie = keyd == m[:, None]
        pick = np.argmax(tie, axis=1)
        return np.where(tie[ar, cur], cur, pick), m
    first, _ = best(keyd)
    keyd2 = keyd.copy()
    keyd2[ar, first] = lowest
    allowed2 = allowed.copy()
    allowed2[ar, first] = False
    second, _ = best(keyd2)
    second = np.where(allowed2.any(axis=1), second, -1)
    cap = (11 * n) // (10 * k)
    new = part.copy()
    cand = np.flatnonzero(first != cur)
    wk = np.searchsorted(np.array([(w * n) // workers for w in range(1, workers + 1)]), cand, side="right")
    order = np.lexsort((cand, second[cand], first[cand], wk))
    cand = cand[order]
    grp = np.stack([wk[order], first[cand], second[cand]], axis=1)
    if len(cand) == 0:
        return new
    change = np.flatnonzero(np.any(grp[1:] != grp[:-1], axis=1)) + 1
    starts = np.concatenate([[0], change])
    ends = np.concatenate([change, [len(cand)]])
    bestg = {}
    for s0, e0 in zip(starts, ends):
        w, j, sec = (int(x) for x in grp[s0])
        b = bestg.get((w, j))
        if b is None or (e0 - s0) > b[0]:           # groups arrive in ascending `sec`
            bestg[(w, j)] = (e0 - s0, s0)
    for (w, j), (length, s0) in bestg.items():
        room = worker_capacity(max(0, cap - int(sizes[j])), workers, w)
        new[cand[s0:s0 + min(length, room)]] = j
    return new


def switching_objective_fast(rowptr, colidx, part, k: int) -> int:
    n = len(rowptr) - 1
    part = np.asarray(part, dtype=np.int32)
    cnt = _count_table(rowptr, colidx, part, k)
    deg = cnt.sum(axis=1)
    same = cnt[np.arange(n), part.astype(np.int64)]
    frac = np.where(deg > 0, (FRAC_ONE * same) // np.maximum(deg, 1), 0)
    total = int(n) * FRAC_ONE + int(frac.sum())
    sizes = np.bincount(part, minlength=k)
    return 11 * n * total - 10 * k * FRAC_ONE * sum(int(x) * int(x) for x in sizes)


# ----------------------------------------------------------------------------------------
# partition structure by set arithmetic
# ----------------------------------------------------------------------------------------
def owned(part, p: int) -> np.ndarray:
    return np.flatnonzero(np.asarray(part) == p).astype(np.int32)


def boundary(rowptr, colidx, part, p: int) -> np.ndarray:
    """Sources outside partition ``p`` that some vertex of ``p`` aggregates from, ordered by
    (partition id, vertex id)."""
    need = set()
    for v in owned(part, p):
        for u in colidx[rowptr[v]:rowptr[v + 1]]:
            if part[u] != p:
                need.add(int(u))
    return np.array(sorted(need, key=lambda u: (int(part[u]), u)), dtype=np.int32)


def required(rowptr, colidx, part, p: int, self_loops: bool) -> set:
    """All vertices whose activations partition ``p`` reads: the union of the sources of its
    destinations (with the implicit self-loop when the model adds one)."""
    need = set()
    for v in owned(part, p):
        need.update(int(u) for u in colidx[rowptr[v]:rowptr[v + 1]])
        if self_loops:
            need.add(int(v))
    return need


def dependent_partitions(rowptr, colidx, part, p: int) -> list:
    return sorted({int(part[u]) for u in boundary(rowptr, colidx, part, p)})


def alpha(rowptr, colidx, part, k: int, self_loops: bool) -> float:
    n = len(rowptr) - 1
    return sum(len(required(rowptr, colidx, part, p, self_loops)) for p in range(k)) / n


def reuse_order(rowptr, colidx, part, k: int) -> list:
    """Order in which the partitions are processed so that cached neighbours are reused
    (appendix on I/O optimisations: the next target partition is picked statically).  The
    paper gives no rule; this build's reading: start at partition 0, then always take the
    unprocessed partition with the most blocks (its own and its dependent partitions') in
    common with the one just processed, the lower id among equals."""
    deps = [set(dependent_partitions(rowptr, colidx, part, p)) | {p} for p in range(k)]
    order = [0]
    left = set(range(1, k))
    while left:
        cur = deps[order[-1]]
        nxt = min(left, key=lambda q: (-len(deps[q] & cur), q))
        order.append(nxt)
        left.remove(nxt)
    return order


# ----------------------------------------------------------------------------------------
# naive partition-wise evaluator (numpy, fp64)
# ----------------------------------------------------------------------------------------
def _operator_rows(model, rowptr, colidx):
    """Per destination: (sources, weights) of the aggregation operator, from the definition."""
    n = len(rowptr) - 1
    rows = []
    if model == "gcn":
        nbr = []
        for v in range(n):
            s = set(int(u) for u in colidx[rowptr[v]:rowptr[v + 1]])
            s.add(v)
            nbr.append(sorted(s))
        deg = np.array([len(s) for s in nbr], dtype=np.float64)
        for v in range(n):
            u = np.array(nbr[v], dtype=np.int64)
            rows.append((u, 1.0 / np.sqrt(deg[u] * deg[v])))
    else:
        for v in range(n):
            u = np.asarray(colidx[rowptr[v]:rowptr[v + 1]], dtype=np.int64)
            rows.append((u, np.full(len(u), 1.0 / max(len(u), 1))))
    return rows


def partitionwise_epoch(model, rowptr, colidx, dims, X, weights, labels, mask, part, k):
    """The paper's per-partition schedule, written naively.

    forward, layer by layer, partition by partition: gather ``GA_p`` (own rows then boundary
    rows), aggregate along ``T_p``, transform, write the partition's rows of ``A^l``;
    backward, layers ``L..1``: zero the gradient of ``A^{l-1}``, then per partition regather,
    recompute the aggregate, add the partition's share of the weight gradients, and for
    ``l >= 2`` scatter-accumulate the gradient of the gathered rows onto their owners.
    Returns the same dict layout as ``oracle.fullgraph.epoch``.
    """
    L = len(dims) - 1
    n = len(rowptr) - 1
    X = np.asarray(X, dtype=np.float64)
    rows = _operator_rows(model, rowptr, colidx)
    parts = []
    for p in range(k):
        own = owned(part, p).astype(np.int64)
        # boundary taken from the operator's rows (the GCN self-loop never leaves a partition)
        need = set()
        for v in own:
            need.update(int(u) for u in rows[v][0] if part[u] != p)
        bnd = np.array(sorted(need, key=lambda u: (int(part[u]), u)), dtype=np.int64)
        R = np.concatenate([own, bnd])
        local = {int(u): i for i, u in enumerate(R)}
        S = np.zeros((len(own), len(R)))
        for i, v in enumerate(own):
            u, w = rows[v]
            for uu, ww in zip(u, w):
                S[i, local[int(uu)]] += ww
        parts.append((own, R, S))

    Wn = [np.asarray(w["W"], dtype=np.float64) for w in weights]
    Wsf = [np.asarray(w["Ws"], dtype=np.float64) if model == "sage" else None for w in weights]
    bs = [np.asarray(w["b"], dtype=np.float64) if w.get("b") is not None else None
          for w in weights]
    act = []
    for l in range(L):
        Ain = X if l == 0 else act[l - 1]
        out = np.zeros((n, dims[l + 1]))
        for own, R, S in parts:
            GA = Ain[R]                       # gather
            Z = S @ GA                        # aggregate along T_p
            Y = Z @ Wn[l]
            if model == "sage":
                Y = Y + Ain[own] @ Wsf[l]
            if bs[l] is not None:
                Y = Y + bs[l]
            out[own] = np.maximum(Y, 0.0) if l < L - 1 else Y
        act.append(out)

    from . import fullgraph
    lossv, G = fullgraph.loss(act[-1], labels, mask)
    gW = [np.zeros_like(w) for w in Wn]
    gWs = [np.zeros_like(w) if w is not None else None for w in Wsf]
    gb = [np.zeros_like(b) if b is not None else None for b in bs]
    gact = [None] * L
    for l in range(L - 1, -1, -1):
        Ain = X if l == 0 else act[l - 1]
        gact[l] = G
        Gprev = np.zeros((n, dims[l]))        # initialisation of the write-back buffer
        for own, R, S in parts:
            dY = G[own] * (act[l][own] > 0) if l < L - 1 else G[own]
            GA = Ain[R]                       # regather
            Z = S @ GA                        # recompute the intermediate
            gW[l] += Z.T @ dY
            if gb[l] is not None:
                gb[l] += dY.sum(axis=0)
            if model == "sage":
                gWs[l] += Ain[own].T @ dY
            if l >= 1:
                dGA = S.T @ (dY @ Wn[l].T)    # gradient of the gathered rows
                np.add.at(Gprev, R, dGA)      # scatter-accumulate
                if model == "sage":
                    Gprev[own] += dY @ Wsf[l].T
        G = Gprev
    return {"act": act, "loss": lossv, "gW": gW, "gWs": gWs, "gb": gb, "gact": gact}
