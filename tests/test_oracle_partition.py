"""Pins for the partition-structure oracle and the partition-wise evaluator."""
import os
from fractions import Fraction

import numpy as np
import pytest

from helpers import random_weights, small_graph
from oracle import fullgraph as og
from oracle import partition as op
from synth import csr_from_edges, make_config

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def read_fixture(name):
    edges, facts, part = [], {}, None
    for line in open(os.path.join(GOLD, name)):
        line = line.split("#")[0].strip()
        if not line:
            continue
        key, _, rest = line.partition(" ")
        if key == "edge":
            edges.append(tuple(int(t) for t in rest.split()))
        elif key == "partition":
            part = np.array([int(t) for t in rest.split()], dtype=np.int32)
        else:
            facts[line.split(":")[0].strip() if ":" in line else key] = \
                [int(t) for t in line.split(":")[-1].split()] if ":" in line else \
                [int(t) for t in rest.split()]
    return edges, part, facts


def test_splitmix64_published_vector():
    # first outputs of the public-domain SplitMix64 reference seeded with 0
    assert op.splitmix64(0) == 0xE220A8397B1DCDAF
    s = 0x9E3779B97F4A7C15
    assert op.splitmix64(s) == 0x6E789E6AA1B965F4
    assert op.splitmix64((2 * s) & op.MASK64) == 0x06C45D188009454F


def test_nine_vertex_example_from_the_paper():
    edges, part, facts = read_fixture("nine_vertex_fixture.txt")
    s = np.array([e[0] for e in edges] + [e[1] for e in edges])
    t = np.array([e[1] for e in edges] + [e[0] for e in edges])
    rowptr, colidx = csr_from_edges(9, s, t)
    assert sorted(op.required(rowptr, colidx, part, 0, self_loops=True)) == facts["required 0"]
    assert sorted(op.boundary(rowptr, colidx, part, 0).tolist()) == facts["boundary 0"]
    assert op.dependent_partitions(rowptr, colidx, part, 0) == facts["dependent 0"]
    assert sorted(op.required(rowptr, colidx, part, 1, self_loops=True)) == facts["required 1"]
    assert op.dependent_partitions(rowptr, colidx, part, 1) == facts["dependent 1"]
    # a' reads a, b, g (self-loop included); g is read by a, h, i
    assert sorted(set(colidx[rowptr[0]:rowptr[1]].tolist()) | {0}) == facts["inputs_of 0"]
    users = sorted(v for v in range(9) if 6 in colidx[rowptr[v]:rowptr[v + 1]])
    assert users == facts["users_of 6"]
    # order of the boundary list: by partition id, then vertex id
    b0 = op.boundary(rowptr, colidx, part, 0)
    assert b0.tolist() == sorted(b0.tolist(), key=lambda u: (part[u], u))


def test_boundary_order_is_partition_then_vertex():
    n, k = 60, 4
    rowptr, colidx = small_graph(n, 300, seed=4)
    part = np.array([(7 * v + 3) % k for v in range(n)], dtype=np.int32)
    for p in range(k):
        b = op.boundary(rowptr, colidx, part, p)
        keys = [(int(part[u]), int(u)) for u in b]
        assert keys == sorted(keys) and len(set(keys)) == len(keys)
        assert all(part[u] != p for u in b)
        # brute force over all (vertex, partition) pairs
        brute = [u for u in range(n) if part[u] != p and
                 any(u in colidx[rowptr[v]:rowptr[v + 1]] for v in range(n) if part[v] == p)]
        assert sorted(b.tolist()) == brute


def test_alpha_counts_required_over_targets():
    n, k = 80, 5
    rowptr, colidx = small_graph(n, 400, seed=8)
    part = op.assign_random(n, k, 3)
    total = 0
    for p in range(k):
        own = set(op.owned(part, p).tolist())
        b = set(op.boundary(rowptr, colidx, part, p).tolist())
        total += len(own | b)              # with self-loops every owned vertex is required
    assert abs(op.alpha(rowptr, colidx, part, k, self_loops=True) - total / n) < 1e-15
    assert op.alpha(rowptr, colidx, np.zeros(n, np.int32), 1, self_loops=True) == 1.0


def test_preference_example_from_the_paper():
    facts = {}
    for line in open(os.path.join(GOLD, "preference_example.txt")):
        line = line.split("#")[0].strip()
        if line:
            key, _, rest = line.partition(" ")
            facts[key] = [int(t) for t in rest.split()]
    pref = op.preferences(facts["neighbour_partitions"], 3)
    assert pref[0] == facts["first_preference"][0]
    assert pref[1] == facts["second_preference"][0]


def test_random_assignment_is_balanced_and_seeded():
    for n, k in [(10, 3), (101, 7), (64, 64), (5, 1)]:
        part = op.assign_random(n, k, 42)
        sizes = np.bincount(part, minlength=k)
        assert sizes.max() - sizes.min() <= 1
        assert np.array_equal(part, op.assign_random_fast(n, k, 42))
        if n > 20:
            assert not np.array_equal(part, op.assign_random(n, k, 43))


def test_integer_key_orders_partitions_like_the_papers_score():
    # Score = 1 + #N(v,j)/#N(v,.) - |P_j| / (1.1 |V| / k), evaluated exactly with fractions
    n, k = 70, 4
    rowptr, colidx = small_graph(n, 350, seed=10)
    part = op.assign_random(n, k, 1)
    sizes = np.bincount(part, minlength=k)
    tgt = op.lp_targets(rowptr, colidx, part, k)
    for v in range(n):
        nb = [u for u in colidx[rowptr[v]:rowptr[v + 1]] if u != v]
        if not nb:
            assert tgt[v] == part[v]
            continue
        score = []
        for j in range(k):
            c = sum(1 for u in nb if part[u] == j)
            score.append(1 + Fraction(c, len(nb)) - Fraction(int(sizes[j]) * 10 * k, 11 * n))
        best = max(score)
        winners = [j for j in range(k) if score[j] == best]
        assert tgt[v] == (part[v] if part[v] in winners else winners[0])


def test_lp_vectorised_equals_loop_and_respects_capacity():
    n, k = 300, 6
    rowptr, colidx = small_graph(n, 2500, seed=14)
    a = op.assign_lp(rowptr, colidx, k, seed=5, rounds=4, fast=True)
    b = op.assign_lp(rowptr, colidx, k, seed=5, rounds=4, fast=False)
    assert np.array_equal(a, b)
    cap = (11 * n) // (10 * k)
    assert np.bincount(a, minlength=k).max() <= max(cap, -(-n // k))
    # label propagation must not make the cut worse than the random start
    start = op.assign_random(n, k, 5)
    src = colidx
    dst = np.repeat(np.arange(n), np.diff(rowptr))
    assert (a[src] != a[dst]).sum() <= (start[src] != start[dst]).sum()


@pytest.mark.parametrize("model,gkw", [
    ("gcn", dict(symmetric=True, self_loops=True)),
    ("gcn", dict(symmetric=False, self_loops=False)),
    ("sage", dict(symmetric=True, self_loops=False)),
    ("sage", dict(symmetric=False, self_loops=False)),
])
def test_partitionwise_equals_full_graph_for_any_k(model, gkw):
    n, dims = 36, (6, 8, 7, 5)
    rowptr, colidx = small_graph(n, 140, seed=15, **gkw)
    rng = np.random.default_rng(1)
    X = rng.standard_normal((n, dims[0]))
    y = rng.integers(0, dims[-1], n).astype(np.int32)
    m = (rng.random(n) < 0.5).astype(np.uint8)
    w = random_weights(dims, 2, sage=(model == "sage"))
    full = og.epoch(model, rowptr, colidx, dims, X, w, y, m)
    assignments = [(k, op.assign_random(n, k, 9)) for k in (1, 2, 3, 7, n)]
    assignments.append((3, np.zeros(n, dtype=np.int32)))                       # two empty parts
    assignments.append((4, (np.arange(n) % 4).astype(np.int32)))               # round robin
    alone = np.zeros(n, dtype=np.int32)
    alone[n // 2] = 1
    assignments.append((2, alone))                                             # one vertex alone
    for k, part in assignments:
        pw = op.partitionwise_epoch(model, rowptr, colidx, dims, X, w, y, m, part, k)
        assert abs(pw["loss"] - full["loss"]) < 1e-12
        for key in ("act", "gW", "gb", "gact") + (("gWs",) if model == "sage" else ()):
            for a, b in zip(pw[key], full[key]):
                assert np.abs(a - b).max() < 1e-12, (key, k)


# ----------------------------------------------------------------------------------------
# the complete switching-aware partitioner
# ----------------------------------------------------------------------------------------
def _read_group_example():
    path = os.path.join(os.path.dirname(__file__), "golden", "switching_group_example.txt")
    fx = {"rows": {}, "first": {}, "second": {}}
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        key, *vals = line.split()
        vals = [int(x) for x in vals]
        if key == "row":
            fx["rows"][vals[0]] = vals[1:]
        elif key == "first_preference":
            fx["first"][vals[0]] = vals[1]
        elif key == "second_preference":
            fx["second"][vals[0]] = vals[1]
        else:
            fx[key] = vals
    return fx


def test_switching_group_example_from_the_paper():
    fx = _read_group_example()
    n, k = fx["n"][0], fx["k"][0]
    part = np.full(n, -1, dtype=np.int32)
    for j in range(k):
        part[fx["partition%d" % j]] = j
    assert part.min() >= 0
    rowptr = np.zeros(n + 1, dtype=np.int64)
    cols = []
    for v in range(n):
        cols += sorted(fx["rows"].get(v, []))
        rowptr[v + 1] = len(cols)
    colidx = np.array(cols, dtype=np.int32)
    sizes = np.bincount(part, minlength=k)
    for v in fx["candidates_of_partition2"]:
        nb = colidx[rowptr[v]:rowptr[v + 1]]
        first, second = op.switching_preferences(part[nb], int(part[v]), n, k, sizes)
        assert (first, second) == (fx["first"][v], fx["second"][v]), v
    for workers in (1, 2):      # with two ranges vertices 0, 6, 8 are still in the same one
        new = op.switching_iteration(rowptr, colidx, part, k, workers)
        moved = np.flatnonzero(new != part)
        assert list(moved) == fx["relocated_to_partition2"]
        assert np.all(new[moved] == 2)
    assert np.array_equal(op.switching_iteration_fast(rowptr, colidx, part, k, 1), new)


def _random_graph(n, m, seed, symmetric=True):
    rng = np.random.default_rng(seed)
    src = rng.integers(0, n, m)
    dst = (src + 1 + rng.zipf(1.6, m) % (n - 1)) % n
    if symmetric:
        src, dst = np.concatenate([src, dst]), np.concatenate([dst, src])
    key = np.unique(dst.astype(np.int64) * n + src)
    rows, cols = key // n, key % n
    rowptr = np.zeros(n + 1, dtype=np.int64)
    np.add.at(rowptr, rows + 1, 1)
    return np.cumsum(rowptr), cols.astype(np.int32)


@pytest.mark.parametrize("n,m,k,workers", [(300, 1500, 5, 3), (257, 900, 9, 16), (64, 400, 2, 1)])
def test_switching_vectorised_equals_loop_and_keeps_the_capacity(n, m, k, workers):
    rowptr, colidx = _random_graph(n, m, seed=n + k)
    part = op.assign_random(n, k, 3)
    cap = (11 * n) // (10 * k)
    for it in range(6):
        assert op.switching_objective(rowptr, colidx, part, k) == \
            op.switching_objective_fast(rowptr, colidx, part, k)
        new = op.switching_iteration(rowptr, colidx, part, k, workers)
        assert np.array_equal(new, op.switching_iteration_fast(rowptr, colidx, part, k, workers))
        sizes, new_sizes = np.bincount(part, minlength=k), np.bincount(new, minlength=k)
        assert new_sizes.max() <= max(cap, sizes.max())
        # no range sends a partition more vertices than its share of the relocation capacity
        for w in range(workers):
            lo, hi = (w * n) // workers, ((w + 1) * n) // workers
            into = np.bincount(new[lo:hi][new[lo:hi] != part[lo:hi]], minlength=k)
            for j in range(k):
                assert into[j] <= op.worker_capacity(max(0, cap - int(sizes[j])), workers, w)
        part = new


def test_switching_objective_is_the_papers_sum_of_scores():
    n, k = 200, 4
    rowptr, colidx = _random_graph(n, 1200, seed=9)
    part = op.assign_random(n, k, 1)
    part[:30] = 0                                   # unbalanced on purpose: the penalty matters
    sizes = np.bincount(part, minlength=k)
    total = 0.0
    for v in range(n):
        nb = colidx[rowptr[v]:rowptr[v + 1]]
        nb = nb[nb != v]
        frac = np.mean(part[nb] == part[v]) if len(nb) else 0.0
        total += 1.0 + frac - sizes[part[v]] / (1.1 * n / k)
    exact = op.switching_objective(rowptr, colidx, part, k) / (11 * n * op.FRAC_ONE)
    assert abs(exact - total) <= n * 2.0 ** -20 + 1e-9 * abs(total)


def test_switching_halts_on_five_small_improvements_in_a_row_or_after_fifty():
    rowptr, colidx = _random_graph(40, 100, seed=2)
    def run(values):
        seq = iter(values)
        part, hist = op.assign_switching(rowptr, colidx, 2, 0, workers=1,
                                         iteration=lambda rp, ci, p, k, w: p,
                                         objective=lambda rp, ci, p, k: next(seq))
        return len(hist) - 1
    big = [1000 * 2 ** i for i in range(60)]
    assert run(big) == 50                                        # never converges: the cap
    flat = [1000000] * 60
    assert run(flat) == 5                                        # five small steps from the start
    # an improvement of exactly 0.1 % of the previous value still counts as an improvement
    def chain(step):
        v = [1000000]
        for _ in range(60):
            v.append(v[-1] + step(v[-1]))
        return v
    assert run(chain(lambda prev: -(-prev // 1000))) == 50
    assert run(chain(lambda prev: -(-prev // 1000) - 1)) == 5
    # a real improvement resets the count; a loss counts as "no improvement"
    seq = [1000, 2000, 2001, 2001, 1990, 1990, 3000, 3001, 3001, 3001, 3001, 3001, 9999]
    assert run(seq + [9999] * 50) == 11


def test_switching_improves_the_expansion_ratio_of_a_power_law_graph():
    cfg, rowptr, colidx = make_config("tiny")
    n, k = cfg["n"], 4
    rnd = op.assign_random(n, k, 5)
    part, hist = op.assign_switching(rowptr, colidx, k, 5, workers=16,
                                     iteration=op.switching_iteration_fast,
                                     objective=op.switching_objective_fast)
    assert len(hist) - 1 <= 50 and hist[-1] > hist[0]
    assert np.bincount(part, minlength=k).max() <= (11 * n) // (10 * k)
    a0 = op.alpha(rowptr, colidx, rnd, k, self_loops=True)
    a1 = op.alpha(rowptr, colidx, part, k, self_loops=True)
    assert a1 < 0.97 * a0, (a0, a1)
