"""Seeded R-MAT graphs in CSR-by-destination form.

Recipe (stated once here, used by every config):

* draw ``m`` directed pairs with the recursive-matrix (R-MAT) process on a
  ``2**scale x 2**scale`` grid with quadrant probabilities ``(a, b, c, d)``;
* squeeze ids from ``[0, 2**scale)`` to ``[0, n)`` with ``id * n >> scale`` (neighbouring
  R-MAT ids have like degree, so merging them keeps the heavy tail);
* pass ids through a seeded random permutation so that vertex id carries no degree or
  locality information;
* drop self-draws, remove duplicates (of the unordered pair when ``symmetric``),
  optionally mirror every edge, optionally add one self-loop per vertex;
* emit CSR whose row ``v`` lists the in-neighbours ``u`` of ``v`` (edge ``u -> v``),
  columns strictly ascending.

The paper trains on ogbn-products, IGB-medium and ogbn-papers100M and on Kronecker
graphs; none of those files is used here.  The configs below only borrow their node
count, edge count and feature width.
"""
from __future__ import annotations

import numpy as np

RMAT_ABCD = (0.57, 0.19, 0.19, 0.05)


def _rmat_pairs(rng: np.random.Generator, scale: int, m: int, abcd=RMAT_ABCD,
                chunk: int = 1 << 24):
    """``m`` (src, dst) pairs of the R-MAT process, int64 ids in ``[0, 2**scale)``."""
    a, b, c, _ = abcd
    src = np.empty(m, dtype=np.int64)
    dst = np.empty(m, dtype=np.int64)
    for lo in range(0, m, chunk):
        hi = min(m, lo + chunk)
        s = np.zeros(hi - lo, dtype=np.int64)
        t = np.zeros(hi - lo, dtype=np.int64)
        for _ in range(scale):
            r = rng.random(hi - lo, dtype=np.float32)
            # quadrants: [0,a) -> (0,0); [a,a+b) -> (0,1); [a+b,a+b+c) -> (1,0); rest -> (1,1)
            sbit = r >= np.float32(a + b)
            tbit = ((r >= np.float32(a)) & ~sbit) | (r >= np.float32(a + b + c))
            s = (s << 1) | sbit
            t = (t << 1) | tbit
        src[lo:hi] = s
        dst[lo:hi] = t
    return src, dst


def csr_from_edges(n: int, src: np.ndarray, dst: np.ndarray):
    """CSR by destination from distinct (src, dst) pairs; columns ascending in each row."""
    key = dst.astype(np.int64) * np.int64(n) + src.astype(np.int64)
    key.sort()
    d = key // n
    colidx = (key - d * n).astype(np.int32)
    counts = np.bincount(d, minlength=n)
    rowptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(counts, out=rowptr[1:])
    return rowptr, colidx


def rmat_graph(n: int, m_draw: int, seed: int, *, symmetric: bool, self_loops: bool,
               scale: int | None = None, abcd=RMAT_ABCD):
    """Seeded R-MAT graph on ``n`` vertices from ``m_draw`` draws.

    Returns ``(rowptr int64[n+1], colidx int32[nnz])``, CSR by destination.
    """
    if scale is None:
        scale = max(1, int(np.ceil(np.log2(n))))
    rng = np.random.default_rng([seed, 0x6A09E667])
    s, t = _rmat_pairs(rng, scale, m_draw, abcd)
    s = (s * n) >> scale
    t = (t * n) >> scale
    perm = rng.permutation(n).astype(np.int64)
    s = perm[s]
    t = perm[t]
    keep = s != t
    s, t = s[keep], t[keep]
    if symmetric:
        lo = np.minimum(s, t)
        hi = np.maximum(s, t)
        key = np.unique(lo * np.int64(n) + hi)
        lo = key // n
        hi = key - lo * n
        s = np.concatenate([lo, hi])
        t = np.concatenate([hi, lo])
    else:
        key = np.unique(t * np.int64(n) + s)
        t = key // n
        s = key - t * n
    if self_loops:
        v = np.arange(n, dtype=np.int64)
        s = np.concatenate([s, v])
        t = np.concatenate([t, v])
    return csr_from_edges(n, s, t)


_counter_lib = None


def _counter():
    """The compiled counter-based generator (``rmat_counter.cpp``), built on first use."""
    global _counter_lib
    if _counter_lib is None:
        import ctypes as C
        from . import build as _build
        lib = C.CDLL(_build.build(force=False))
        lib.rmat_counter_generate.restype = C.c_void_p
        lib.rmat_counter_generate.argtypes = [C.c_int64, C.c_int64, C.c_uint64, C.c_int, C.c_double,
                                              C.c_double, C.c_double, C.c_int, C.c_int,
                                              C.POINTER(C.c_int64)]
        lib.rmat_counter_fetch.restype = None
        lib.rmat_counter_fetch.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
        lib.normal_counter_fill.restype = None
        lib.normal_counter_fill.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_uint64]
        _counter_lib = lib
    return _counter_lib


def rmat_graph_counter(n: int, m_draw: int, seed: int, *, symmetric: bool, self_loops: bool,
                       scale: int | None = None, abcd=RMAT_ABCD):
    """The same recipe as :func:`rmat_graph` with counter-based draws (SplitMix64 of the edge
    index and level) and a permutation by sorted SplitMix64 keys, generated and sorted on all
    host cores by ``rmat_counter.cpp``: for graphs of 10^8 and more draws.  A different random
    stream, hence a different graph than :func:`rmat_graph` gives for the same seed."""
    import ctypes as C
    if scale is None:
        scale = max(1, int(np.ceil(np.log2(n))))
    lib = _counter()
    nnz = C.c_int64(0)
    h = lib.rmat_counter_generate(n, m_draw, seed, scale, abcd[0], abcd[1], abcd[2],
                                  1 if symmetric else 0, 1 if self_loops else 0, C.byref(nnz))
    if not h:
        raise MemoryError("rmat_counter_generate: out of memory")
    rowptr = np.empty(n + 1, dtype=np.int64)
    colidx = np.empty(nnz.value, dtype=np.int32)
    lib.rmat_counter_fetch(h, rowptr.ctypes.data, colidx.ctypes.data)
    return rowptr, colidx


def normal_counter(n: int, d: int, seed: int) -> np.ndarray:
    """``[n, d]`` float32 standard-normal numbers, element ``i`` a function of ``(seed, i)``
    alone (Box-Muller on SplitMix64 draws), filled on all host cores."""
    out = np.empty((n, d), dtype=np.float32)
    _counter().normal_counter_fill(out.ctypes.data, 0, n * d, seed)
    return out


# Workload shapes.  "m_draw" is tuned so the distinct-edge count lands near the target.
# "gen": which generator draws the graph and the features: "numpy" (default) or "counter" (the
# parallel counter-based one, for the workloads whose inputs would otherwise take minutes).
CONFIGS = {
    # parity fixture: 10,000 nodes, ~100,000 draws symmetrised, self-loops, 2-layer GCN
    "tiny": dict(n=10_000, m_draw=100_000, seed=1, symmetric=True, self_loops=True,
                 model="gcn", dims=(64, 64, 16), dtype="f32", k=4, part="random",
                 train_frac=0.5),
    # products-shaped: 2.4M nodes, ~62M undirected edges, 3-layer SAGE-mean
    "mid": dict(n=2_400_000, m_draw=70_500_000, seed=2, symmetric=True, self_loops=False,
                model="sage", dims=(100, 256, 256, 47), dtype="f32", k=16, part="switching",
                train_frac=0.1),
    # the same graph and widths with graph-attention layers (the paper's second model family)
    "mid_gat": dict(n=2_400_000, m_draw=70_500_000, seed=2, symmetric=True, self_loops=False,
                    model="gat", dims=(100, 256, 256, 47), dtype="f32", k=16, part="switching",
                    train_frac=0.1),
    # half of papers100M's shape: 50M nodes, ~800M directed edges, 3-layer GCN
    "large": dict(n=50_000_000, m_draw=830_000_000, seed=3, symmetric=False, self_loops=True,
                  model="gcn", dims=(128, 128, 128, 172), dtype="f32", k=64, part="switching_device",
                  train_frac=0.1, gen="counter"),
    # the beyond-HBM recipe (papers100M symmetrised: 100M nodes, ~2e9 entries, 3-layer SAGE-mean
    # 128->256->256->64, k = 256) scaled to 6 % of its vertices at the same average degree (20),
    # widths and partition count, so that activations + gradients (15 GB) fit the pinned host
    # memory of a GPU machine; it runs through the streaming schedule with a pool below that
    "beyond": dict(n=6_000_000, m_draw=64_000_000, seed=5, symmetric=True, self_loops=False,
                   model="sage", dims=(128, 256, 256, 64), dtype="f32", k=256, part="switching_device",
                   train_frac=0.1, gen="counter"),
    # wide hidden sizes, bf16 transforms
    "dense": dict(n=4_000_000, m_draw=55_000_000, seed=4, symmetric=True, self_loops=True,
                  model="gcn", dims=(512, 1024, 1024, 64), dtype="bf16", k=16, part="lp",
                  train_frac=0.1),
    # small stand-ins with the same structure, for tests
    "mini_sage": dict(n=3_000, m_draw=40_000, seed=12, symmetric=True, self_loops=False,
                      model="sage", dims=(100, 256, 256, 47), dtype="f32", k=5, part="lp",
                      train_frac=0.1),
    "mini_gcn_directed": dict(n=4_000, m_draw=50_000, seed=13, symmetric=False,
                              self_loops=True, model="gcn", dims=(128, 128, 128, 172),
                              dtype="f32", k=7, part="lp", train_frac=0.1),
}


def make_config(name: str, **override):
    """Graph of a named config (after ``override``).  Returns ``(cfg, rowptr, colidx)``."""
    cfg = dict(CONFIGS[name])
    cfg.update(override)
    gen = rmat_graph_counter if cfg.get("gen") == "counter" else rmat_graph
    rowptr, colidx = gen(cfg["n"], cfg["m_draw"], cfg["seed"],
                         symmetric=cfg["symmetric"], self_loops=cfg["self_loops"])
    return cfg, rowptr, colidx
