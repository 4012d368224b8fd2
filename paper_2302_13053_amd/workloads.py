"""Seeded synthetic inputs shaped like the paper's evaluation graphs.

The paper evaluates on seven public node-classification datasets (dataset
statistics table in the evaluation appendix).  None of them is available here,
so every input is synthetic: a seeded random graph with the node count, edge
count and degree skew of one of those datasets, a seeded feature matrix with
its width and value distribution, and seeded Glorot-style parameters with the
model widths the hyper-parameter paragraph gives (adjusted per workload, see
``WORKLOADS``).

This module only *draws inputs*.  It contains none of the method's arithmetic
(no CSR construction, no normalisation, no transform, no aggregation): the
edge lists it returns are raw undirected pairs, and turning them into a CSR is
the job of the library under test and, separately, of the CPU oracle.  Both
the tests and the benchmark feed the same arrays to either side.

Random numbers come from numpy's counter-based Philox generator keyed by an
integer seed, so every array is a pure function of (workload, seed).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Tuple

import numpy as np

BASE_SEED = 20230213


# ----------------------------------------------------------------------------
# descriptions
# ----------------------------------------------------------------------------
@dataclass(frozen=True)
class Stage:
    """One call on the embed-and-aggregate path.

    kind: "round"      -> transform (if d_in != 0) followed by aggregation
          "transform"  -> bare dense transform (the final classifier layer)
          "head_mean"  -> mean over the ``heads`` column blocks of the last attention round
                          (d_in = heads * d_out columns in, d_out out)
    For kind == "round", ``w`` False means the identity transform (the very
    first message-passing round is taken over the raw features).
    """
    kind: str
    d_in: int
    d_out: int
    w: bool = True
    relu: bool = False
    mode: str = "mean"          # mean | sum | gcn_sym | gat_softmax
    concat: bool = False
    heads: int = 1

    @property
    def out_width(self) -> int:
        if self.kind in ("transform", "head_mean"):
            return self.d_out
        return 2 * self.d_out if self.concat else self.d_out


@dataclass(frozen=True)
class Workload:
    index: int
    name: str
    family: str                 # sage | gcn | gat
    n_nodes: int
    graph: str                  # er | chung_lu | ba | power_law
    graph_args: Dict[str, float]
    self_loops: bool
    feat_dim: int
    feat_kind: str              # bernoulli | tfidf | normal
    stages: Tuple[Stage, ...] = field(default_factory=tuple)
    stands_in_for: str = ""


def _sage(f0: int, hidden: int, rounds: int, classes: int) -> Tuple[Stage, ...]:
    st: List[Stage] = [Stage("round", f0, f0, w=False, mode="mean", concat=True)]
    width = 2 * f0
    for _ in range(rounds - 1):
        st.append(Stage("round", width, hidden, relu=True, mode="mean", concat=True))
        width = 2 * hidden
    st.append(Stage("transform", width, classes))
    return tuple(st)


def _gcn(f0: int, hidden: int, rounds: int, classes: int) -> Tuple[Stage, ...]:
    st: List[Stage] = [Stage("round", f0, f0, w=False, mode="gcn_sym")]
    width = f0
    for _ in range(rounds - 1):
        st.append(Stage("round", width, hidden, relu=True, mode="gcn_sym"))
        width = hidden
    st.append(Stage("transform", width, classes))
    return tuple(st)


def _gat(f0: int, heads: int, dh: int, rounds: int, classes: int) -> Tuple[Stage, ...]:
    st: List[Stage] = []
    width = f0
    for r in range(rounds):
        out = heads * (dh if r < rounds - 1 else classes)
        st.append(Stage("round", width, out, mode="gat_softmax", heads=heads))
        width = out
    # the last round's heads are averaged into the class scores
    st.append(Stage("head_mean", width, classes, w=False, heads=heads))
    return tuple(st)


WORKLOADS: Tuple[Workload, ...] = (
    Workload(0, "sage_tiny_er", "sage", 2708, "er", {"edges": 5429}, False,
             1433, "bernoulli", _sage(1433, 64, 2, 7), "Cora-shaped"),
    Workload(1, "gcn_citation_chunglu", "gcn", 19717, "chung_lu",
             {"edges": 44338, "exponent": 2.5, "max_w": 300.0}, True,
             500, "tfidf", _gcn(500, 256, 3, 3), "PubMed-shaped"),
    Workload(2, "sage_social_ba", "sage", 22470, "ba", {"edges": 171002}, False,
             128, "normal", _sage(128, 256, 3, 4), "Facebook-page-shaped"),
    Workload(3, "sage_large_powerlaw", "sage", 232965, "power_law",
             {"raw_pairs": 58_620_000, "exponent": 2.5, "mean_w": 503.0, "max_w": 23000.0},
             False, 602, "normal", _sage(602, 256, 2, 41), "Reddit-shaped"),
    Workload(4, "gat_products_powerlaw", "gat", 2449029, "power_law",
             {"raw_pairs": 61_920_000, "exponent": 2.8, "mean_w": 50.63, "max_w": 17500.0},
             False, 100, "normal", _gat(100, 4, 64, 3, 47), "ogbn-products-shaped"),
)


def workload(index_or_name) -> Workload:
    for w in WORKLOADS:
        if w.index == index_or_name or w.name == index_or_name:
            return w
    raise KeyError(index_or_name)


def seed_for(index: int) -> int:
    return BASE_SEED * 10 + index + 1


def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[seed, stream]))


# ----------------------------------------------------------------------------
# graphs: every function returns raw undirected pairs (src, dst) as int32
# ----------------------------------------------------------------------------
def _distinct_pairs(draw, n_edges: int) -> Tuple[np.ndarray, np.ndarray]:
    """Keep drawing batches from ``draw(k)`` until ``n_edges`` distinct
    unordered non-loop pairs have been seen; first occurrences are kept."""
    got_lo = np.empty(0, np.int64)
    got_hi = np.empty(0, np.int64)
    seen = np.empty(0, np.int64)
    while got_lo.size < n_edges:
        k = int((n_edges - got_lo.size) * 1.3) + 64
        a, b = draw(k)
        lo = np.minimum(a, b).astype(np.int64)
        hi = np.maximum(a, b).astype(np.int64)
        keep = lo != hi
        lo, hi = lo[keep], hi[keep]
        key = (lo << 32) | hi
        _, first = np.unique(key, return_index=True)
        first.sort()
        lo, hi, key = lo[first], hi[first], key[first]
        fresh = ~np.isin(key, seen)
        lo, hi, key = lo[fresh], hi[fresh], key[fresh]
        got_lo = np.concatenate([got_lo, lo])
        got_hi = np.concatenate([got_hi, hi])
        seen = np.concatenate([seen, key])
    return got_lo[:n_edges].astype(np.int32), got_hi[:n_edges].astype(np.int32)


def graph_er(n: int, n_edges: int, seed: int) -> Tuple[np.ndarray, np.ndarray]:
    """G(n, m): ``n_edges`` distinct undirected edges chosen uniformly."""
    rng = _rng(seed, 0)

    def draw(k):
        return rng.integers(0, n, k), rng.integers(0, n, k)

    return _distinct_pairs(draw, n_edges)


def power_law_weights(n: int, exponent: float, mean_w: float, max_w: float) -> np.ndarray:
    """Expected-degree sequence w_i proportional to rank^(-1/(exponent-1)),
    clipped at ``max_w`` and scaled (by bisection on the scale) so that the
    clipped sequence has mean ``mean_w``.  Returned in rank order."""
    base = np.arange(1, n + 1, dtype=np.float64) ** (-1.0 / (exponent - 1.0))
    lo, hi = 0.0, max_w * n
    for _ in range(200):
        mid = 0.5 * (lo + hi)
        if np.minimum(mid * base, max_w).mean() < mean_w:
            lo = mid
        else:
            hi = mid
    return np.minimum(hi * base, max_w)


def _endpoint_table(w: np.ndarray, log2_slots: int) -> np.ndarray:
    """Lookup table in which node i occupies a share of slots proportional to
    w_i (at least one), so that a uniform slot draw is a draw proportional to
    the weights up to quantisation."""
    slots = 1 << log2_slots
    cnt = np.maximum(1, np.rint(w / w.sum() * slots)).astype(np.int64)
    return np.repeat(np.arange(w.size, dtype=np.int32), cnt)


def _weighted_endpoints(n: int, exponent: float, mean_w: float, max_w: float,
                        seed: int, log2_slots: int):
    w = power_law_weights(n, exponent, mean_w, max_w)
    rng = _rng(seed, 0)
    # node ids carry no degree information: ranks are scattered by a seeded permutation
    ids = rng.permutation(n).astype(np.int32)
    table = ids[_endpoint_table(w, log2_slots)]
    return rng, table


def graph_chung_lu(n: int, n_edges: int, exponent: float, max_w: float,
                   seed: int) -> Tuple[np.ndarray, np.ndarray]:
    """Chung-Lu style graph with exactly ``n_edges`` distinct undirected edges:
    both endpoints drawn independently, proportional to power-law weights."""
    rng, table = _weighted_endpoints(n, exponent, 2.0 * n_edges / n, max_w, seed, 22)

    def draw(k):
        return (table[rng.integers(0, table.size, k)],
                table[rng.integers(0, table.size, k)])

    return _distinct_pairs(draw, n_edges)


def graph_power_law(n: int, raw_pairs: int, exponent: float, mean_w: float,
                    max_w: float, seed: int) -> Tuple[np.ndarray, np.ndarray]:
    """Large power-law graph: ``raw_pairs`` endpoint pairs drawn as in
    ``graph_chung_lu`` and returned RAW, i.e. still containing the repeated
    pairs and self pairs the draw produces (the heavy nodes repeat often).
    Cleaning them is part of CSR construction, not of input generation."""
    rng, table = _weighted_endpoints(n, exponent, mean_w, max_w, seed, 27)
    src = np.empty(raw_pairs, np.int32)
    dst = np.empty(raw_pairs, np.int32)
    step = 1 << 23
    for s in range(0, raw_pairs, step):
        e = min(raw_pairs, s + step)
        src[s:e] = table[rng.integers(0, table.size, e - s)]
        dst[s:e] = table[rng.integers(0, table.size, e - s)]
    return src, dst


def graph_ba(n: int, n_edges: int, seed: int) -> Tuple[np.ndarray, np.ndarray]:
    """Barabasi-Albert preferential attachment.  Each new node attaches to 7 or
    8 distinct earlier nodes (chosen with probability proportional to their
    current degree); the 7/8 mix is spread evenly so that the total comes to
    ``n_edges``."""
    rng = _rng(seed, 0)
    m_hi = -(-n_edges // n)                    # ceil
    m_lo = m_hi - 1
    m0 = m_hi + 1                              # seed clique size
    seed_edges = m0 * (m0 - 1) // 2
    new_nodes = n - m0
    n_hi = (n_edges - seed_edges) - m_lo * new_nodes   # how many nodes take m_hi
    if not (0 <= n_hi <= new_nodes):
        raise ValueError("edge count not reachable with a 2-value attachment mix")
    src: List[np.ndarray] = []
    dst: List[np.ndarray] = []
    iu, ju = np.triu_indices(m0, 1)
    src.append(iu.astype(np.int32))
    dst.append(ju.astype(np.int32))
    ends = np.empty(2 * n_edges, np.int32)     # every edge endpoint so far
    ends[:seed_edges] = iu
    ends[seed_edges:2 * seed_edges] = ju
    fill = 2 * seed_edges
    for t in range(new_nodes):
        v = m0 + t
        m = m_hi if ((t + 1) * n_hi) // new_nodes > (t * n_hi) // new_nodes else m_lo
        chosen = np.unique(ends[rng.integers(0, fill, m)])
        while chosen.size < m:
            extra = ends[rng.integers(0, fill, m - chosen.size)]
            chosen = np.unique(np.concatenate([chosen, extra]))
        src.append(np.full(m, v, np.int32))
        dst.append(chosen.astype(np.int32))
        ends[fill:fill + m] = v
        ends[fill + m:fill + 2 * m] = chosen
        fill += 2 * m
    s = np.concatenate(src)
    d = np.concatenate(dst)
    assert s.size == n_edges
    return s, d


def make_graph(wl: Workload, seed: Optional[int] = None) -> Tuple[np.ndarray, np.ndarray]:
    seed = seed_for(wl.index) if seed is None else seed
    a = wl.graph_args
    if wl.graph == "er":
        return graph_er(wl.n_nodes, int(a["edges"]), seed)
    if wl.graph == "chung_lu":
        return graph_chung_lu(wl.n_nodes, int(a["edges"]), a["exponent"], a["max_w"], seed)
    if wl.graph == "ba":
        return graph_ba(wl.n_nodes, int(a["edges"]), seed)
    if wl.graph == "power_law":
        return graph_power_law(wl.n_nodes, int(a["raw_pairs"]), a["exponent"],
                               a["mean_w"], a["max_w"], seed)
    raise ValueError(wl.graph)


# ----------------------------------------------------------------------------
# features and parameters
# ----------------------------------------------------------------------------
def pad_ld(width: int, multiple: int = 32) -> int:
    """Leading dimension (in floats) rounded up so that every row starts on a
    128-byte boundary when ``multiple`` is 32."""
    return -(-width // multiple) * multiple


def make_features(wl: Workload, ld: Optional[int] = None,
                  seed: Optional[int] = None) -> np.ndarray:
    """[n_nodes, ld] float32 array whose first ``feat_dim`` columns hold the
    features; padding columns (if any) are zero."""
    seed = seed_for(wl.index) if seed is None else seed
    rng = _rng(seed, 1)
    n, f = wl.n_nodes, wl.feat_dim
    ld = f if ld is None else ld
    out = np.zeros((n, ld), np.float32)
    rows = max(1, (1 << 24) // max(f, 1))
    for s in range(0, n, rows):
        e = min(n, s + rows)
        if wl.feat_kind == "bernoulli":
            blk = (rng.random((e - s, f), dtype=np.float32) < 0.013).astype(np.float32)
        elif wl.feat_kind == "tfidf":
            mask = rng.random((e - s, f), dtype=np.float32) < 0.15
            val = rng.standard_exponential((e - s, f), dtype=np.float32)
            blk = np.where(mask, val, np.float32(0))
            nrm = np.sqrt((blk.astype(np.float64) ** 2).sum(axis=1, keepdims=True))
            nrm[nrm == 0] = 1.0
            blk = (blk / nrm).astype(np.float32)
        elif wl.feat_kind == "normal":
            blk = rng.standard_normal((e - s, f), dtype=np.float32)
        else:
            raise ValueError(wl.feat_kind)
        out[s:e, :f] = blk
    return out


@dataclass
class StageParams:
    W: Optional[np.ndarray] = None       # [d_in, d_out] row-major
    b: Optional[np.ndarray] = None       # [d_out]
    a_src: Optional[np.ndarray] = None   # [heads, d_out // heads]
    a_dst: Optional[np.ndarray] = None


def glorot(rng: np.random.Generator, fan_in: int, fan_out: int, shape) -> np.ndarray:
    lim = np.sqrt(6.0 / (fan_in + fan_out))
    return rng.uniform(-lim, lim, shape).astype(np.float32)


def make_params(wl: Workload, seed: Optional[int] = None) -> List[StageParams]:
    """Untrained stand-ins for the per-round parameters: Glorot-uniform weight
    matrices, small uniform biases, Glorot attention vectors."""
    seed = seed_for(wl.index) if seed is None else seed
    out: List[StageParams] = []
    for r, st in enumerate(wl.stages):
        rng = _rng(seed, 2 + r)
        p = StageParams()
        if st.w:
            p.W = glorot(rng, st.d_in, st.d_out, (st.d_in, st.d_out))
            p.b = rng.uniform(-0.1, 0.1, st.d_out).astype(np.float32)
        if st.kind == "round" and st.mode == "gat_softmax":
            dh = st.d_out // st.heads
            p.a_src = glorot(rng, dh, 1, (st.heads, dh))
            p.a_dst = glorot(rng, dh, 1, (st.heads, dh))
        out.append(p)
    return out


# ----------------------------------------------------------------------------
# small free-form inputs for tests
# ----------------------------------------------------------------------------
def random_pairs(n: int, n_pairs: int, seed: int, skew: float = 0.0):
    """Raw pairs with repeats and self pairs left in.  ``skew`` > 0 bends the
    endpoint distribution towards low ids (u**(1+skew)), giving a few heavy
    rows."""
    rng = _rng(seed, 7)
    u = rng.random(n_pairs) ** (1.0 + skew)
    v = rng.random(n_pairs) ** (1.0 + skew)
    return ((u * n).astype(np.int32).clip(0, n - 1),
            (v * n).astype(np.int32).clip(0, n - 1))


def random_matrix(rows: int, cols: int, seed: int, ld: Optional[int] = None,
                  kind: str = "normal") -> np.ndarray:
    rng = _rng(seed, 8)
    ld = cols if ld is None else ld
    out = np.zeros((rows, ld), np.float32)
    if kind == "normal":
        out[:, :cols] = rng.standard_normal((rows, cols), dtype=np.float32)
    elif kind == "absnormal":
        out[:, :cols] = np.abs(rng.standard_normal((rows, cols), dtype=np.float32))
    elif kind == "smallint":
        out[:, :cols] = rng.integers(-3, 4, (rows, cols)).astype(np.float32)
    else:
        raise ValueError(kind)
    return out
