"""Synthetic heterogeneous graphs, layer-wise neighbour sampling and weights.

Everything is drawn from one master seed per configuration
(`240808490 + config index`), split into independent streams
(graph, features, weights, sampler, labels) with `numpy.random.SeedSequence`.

The graphs stand in for the RDF datasets the paper evaluates on (its Table 2):
only their *shape* is imitated (vertex types, relations with reverses, skewed
degrees); none of their records are reproduced.

Mini-batch structure (the reading used throughout this repository):
hop-k "blocks".  Layer l of L (executed l-th) consumes the block sampled at hop
L-l+1.  In every block the destination vertices of a type are the first
`n_dst[t]` of that type's source vertices (targets first, then newly reached
vertices in first-appearance order), so a layer's output rows are the next
layer's input rows.  A block's edges are a single COO list over all relations
(local source index, local destination index), plus per-edge global edge ids
whose relation is looked up in a global edge-type table -- the inputs of the
paper's Algorithm 2.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import numpy as np

MASTER_SEED = 240808490
CONFIG_NAMES = ["tiny_rgcn_f32", "academic_rgcn_f32", "academic_rgcn_bf16",
                "many_types_rgcn_f32", "academic_rgat_bf16",
                "relation_heavy_small_f32", "relation_heavy_large_bf16", "widest_schema_f32"]


# --------------------------------------------------------------------------- #
# containers
# --------------------------------------------------------------------------- #
@dataclass
class Schema:
    num_types: int
    rel_src: List[int]
    rel_dst: List[int]

    @property
    def num_rels(self) -> int:
        return len(self.rel_src)


@dataclass
class HeteroGraph:
    schema: Schema
    num_nodes: List[int]
    feat_dim: List[int]
    # per relation r: in-neighbour CSR over destination vertices of type dst(r)
    in_indptr: List[np.ndarray]          # int64 [num_nodes[dst]+1]
    in_nbr: List[np.ndarray]             # int32 [E_r] source vertex ids
    edge_off: np.ndarray                 # int64 [R+1]; global edge id = edge_off[r] + position in in_nbr[r]
    edge_type: np.ndarray                # int32 [E_total], global per-edge relation id
    stores: List[np.ndarray]             # float32 [num_nodes[t], feat_dim[t]]


@dataclass
class Block:
    n_src: List[int]
    n_dst: List[int]
    edge_index: np.ndarray               # int64 [2, E]: row 0 local src, row 1 local dst
    edge_id: np.ndarray                  # int64 [E] global edge ids
    edge_type: np.ndarray                # int32 [E] (= graph.edge_type[edge_id]; convenience copy)


@dataclass
class MiniBatch:
    ids: List[np.ndarray]                # per type int64 global ids of the first layer's source rows
    blocks: List[Block]                  # execution order: blocks[0] feeds layer 1
    target_type: int
    labels: Optional[np.ndarray] = None  # int64 [batch] for cross-entropy configs
    grad_out: Optional[List[np.ndarray]] = None  # per type float32 upstream gradient for non-xent configs


@dataclass
class LayerWeights:
    in_dim: List[int]
    out_dim: int
    w_rel: List[np.ndarray]              # [R] float32 [F_src(r), H]
    w_root: List[Optional[np.ndarray]]   # [T] float32 [F_t, H] or None
    bias: List[Optional[np.ndarray]]     # [T] float32 [H] or None
    relu: bool
    # attention variant only
    w_type: List[Optional[np.ndarray]] = field(default_factory=list)   # [T] [F_t, H]
    a_src: List[Optional[np.ndarray]] = field(default_factory=list)    # [R] [heads, H/heads]
    a_dst: List[Optional[np.ndarray]] = field(default_factory=list)
    w_sem: Optional[np.ndarray] = None   # [H, 128]
    b_sem: Optional[np.ndarray] = None   # [128]
    q_sem: Optional[np.ndarray] = None   # [128]


@dataclass
class Config:
    index: int
    name: str
    dtype: str                           # "f32" | "bf16"
    kind: str                            # "rgcn" | "rgat"
    layer_out: List[int]                 # output width of each layer, execution order
    relu: List[bool]
    bias: bool
    fanouts: List[int]                   # per hop, hop 1 (nearest the targets) first
    batch: int
    loss: str                            # "sum" | "xent" | "dot" (sum of G*h with seeded G)
    num_classes: int = 0
    heads: int = 1
    scale: float = 1.0                   # shrinks vertex and edge counts (tests); 1.0 = as specified


def bf16_round(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even); returns float32.

    Storage-format conversion only, so that both sides start from bit-identical
    bf16-representable inputs."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty_like(x)
    xf, of = x.reshape(-1), out.reshape(-1)
    step = 1 << 22

    def work(a):
        u = xf[a: a + step].view(np.uint32)
        r = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
        r &= np.uint32(0xFFFF0000)
        o = r.view(np.float32)
        bad = ~np.isfinite(xf[a: a + step])
        if bad.any():
            o[bad] = xf[a: a + step][bad]
        of[a: a + step] = o
    starts = range(0, xf.size, step)
    if xf.size > step:
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(max_workers=8) as ex:
            list(ex.map(work, starts))
    else:
        for a in starts:
            work(a)
    return out


def _streams(index: int):
    ss = np.random.SeedSequence(MASTER_SEED + index).spawn(5)
    return {k: np.random.default_rng(s) for k, s in
            zip(["graph", "features", "weights", "sampler", "labels"], ss)}


# --------------------------------------------------------------------------- #
# configurations
# --------------------------------------------------------------------------- #
def make_config(index: int, scale: float = 1.0, batch: Optional[int] = None) -> Config:
    if index == 0:
        c = Config(0, CONFIG_NAMES[0], "f32", "rgcn", [16], [False], False, [5], 64, "sum")
    elif index == 1:
        c = Config(1, CONFIG_NAMES[1], "f32", "rgcn", [256, 349], [True, False], True,
                   [25, 20], 1024, "xent", num_classes=349)
    elif index == 2:
        c = Config(2, CONFIG_NAMES[2], "bf16", "rgcn", [512, 349], [True, False], True,
                   [25, 20], 4096, "xent", num_classes=349)
    elif index == 3:
        c = Config(3, CONFIG_NAMES[3], "f32", "rgcn", [128, 128], [True, False], True,
                   [10, 10], 512, "dot")
    elif index == 4:
        c = Config(4, CONFIG_NAMES[4], "bf16", "rgat", [256, 256, 256], [True, True, False], True,
                   [15, 10, 5], 2048, "dot", heads=8)
    elif index == 5:
        # the regime of the smallest graph of the paper's Table 2: a few thousand vertices, ~100 relations
        c = Config(5, CONFIG_NAMES[5], "f32", "rgcn", [64, 32], [True, False], True,
                   [10, 10], 128, "dot")
    elif index == 6:
        # the regime of its largest graph: ~1.9 M vertices, ~5.7 M edges, 7 vertex types, 108 relations
        c = Config(6, CONFIG_NAMES[6], "bf16", "rgcn", [128, 64], [True, False], True,
                   [10, 10], 1024, "dot")
    elif index == 7:
        # the widest schema the library takes: 32 vertex types, 128 relations, ragged widths, small graph
        c = Config(7, CONFIG_NAMES[7], "f32", "rgcn", [24, 16], [True, False], True, [4, 3], 48, "dot")
    else:
        raise ValueError("config index must be 0..7")
    c.scale = scale
    if batch is not None:
        c.batch = batch
    return c


# --------------------------------------------------------------------------- #
# graphs
# --------------------------------------------------------------------------- #
def _dedup_pairs(src, dst, n_dst):
    key = np.unique(src.astype(np.int64) * np.int64(n_dst) + dst.astype(np.int64))
    return (key // n_dst).astype(np.int64), (key % n_dst).astype(np.int64)


def _in_csr(src, dst, n_src, n_dst):
    """Group (src, dst) pairs by destination; neighbours in ascending source id."""
    key = dst.astype(np.int64) * np.int64(n_src) + src.astype(np.int64)
    key.sort()
    nbr = (key % n_src).astype(np.int32)
    indptr = np.zeros(n_dst + 1, dtype=np.int64)
    np.cumsum(np.bincount(dst, minlength=n_dst), out=indptr[1:])
    return indptr, nbr


def _iid_categorical(rng, weights, n):
    """n i.i.d. draws from Categorical(weights), returned in random order.
    (Counts per category from one multinomial draw, then a random permutation.)"""
    counts = rng.multinomial(n, weights / weights.sum())
    return rng.permutation(np.repeat(np.arange(len(weights), dtype=np.int64), counts))


def _normal_store(rng, n, d, scale=1.0, chunk=65536):
    """float32 N(0, scale^2) matrix, filled chunk-by-chunk from child streams so the
    values do not depend on how many threads do the filling."""
    from concurrent.futures import ThreadPoolExecutor
    out = np.empty((n, d), dtype=np.float32)
    starts = list(range(0, n, chunk))
    kids = rng.bit_generator.seed_seq.spawn(len(starts)) if hasattr(rng.bit_generator, "seed_seq") \
        else np.random.SeedSequence(int(rng.integers(1 << 62))).spawn(len(starts))

    def fill(i):
        a = starts[i]; b = min(n, a + chunk)
        np.random.default_rng(kids[i]).standard_normal((b - a, d), dtype=np.float32, out=out[a:b])
        if scale != 1.0:
            out[a:b] *= np.float32(scale)
    with ThreadPoolExecutor(max_workers=8) as ex:
        list(ex.map(fill, range(len(starts))))
    return out


def _zipf_pairs(rng, n_src, n_dst, n_edges, exponent=2.1, cap=1e4):
    ws = np.minimum(rng.zipf(exponent, n_src).astype(np.float64), cap)
    wd = np.minimum(rng.zipf(exponent, n_dst).astype(np.float64), cap)
    src = _iid_categorical(rng, ws, n_edges)
    dst = _iid_categorical(rng, wd, n_edges)
    return _dedup_pairs(src, dst, n_dst)


def _finish_graph(schema, num_nodes, feat_dim, pairs_per_rel, stores):
    in_indptr, in_nbr, counts = [], [], []
    for r in range(schema.num_rels):
        src, dst = pairs_per_rel[r]
        ip, nb = _in_csr(src, dst, num_nodes[schema.rel_src[r]], num_nodes[schema.rel_dst[r]])
        in_indptr.append(ip); in_nbr.append(nb); counts.append(len(nb))
    edge_off = np.zeros(schema.num_rels + 1, dtype=np.int64)
    np.cumsum(counts, out=edge_off[1:])
    edge_type = np.repeat(np.arange(schema.num_rels, dtype=np.int32), counts)
    return HeteroGraph(schema, list(num_nodes), list(feat_dim), in_indptr, in_nbr,
                       edge_off, edge_type, stores)


def build_graph(cfg: Config) -> HeteroGraph:
    rs = _streams(cfg.index)
    g, f = rs["graph"], rs["features"]
    sc = cfg.scale
    if cfg.index == 0:
        schema = Schema(2, [0, 1, 1], [1, 0, 1])          # A->B, B->A, B->B
        num_nodes, feat_dim = [200, 300], [16, 32]
        pairs = []
        for r in range(3):
            ns, nd = num_nodes[schema.rel_src[r]], num_nodes[schema.rel_dst[r]]
            pairs.append(_dedup_pairs(g.integers(0, ns, 1500), g.integers(0, nd, 1500), nd))
        stores = [_normal_store(f, n, d) for n, d in zip(num_nodes, feat_dim)]
        return _finish_graph(schema, num_nodes, feat_dim, pairs, stores)

    if cfg.index in (1, 2, 4):
        num_nodes = [max(8, int(round(n * sc))) for n in (736_000, 1_130_000, 8_700, 60_000)]
        feat_dim = [128] * 4
        # forward relations r0 T1->T0, r2 T0->T0, r4 T0->T3, r6 T1->T2; odd ids are their reverses
        fwd = [(1, 0, 7_100_000), (0, 0, 5_400_000), (0, 3, 7_500_000), (1, 2, 1_000_000)]
        rel_src, rel_dst, pairs = [], [], []
        for (s, d, e) in fwd:
            src, dst = _zipf_pairs(g, num_nodes[s], num_nodes[d], max(16, int(round(e * sc))))
            rel_src += [s, d]; rel_dst += [d, s]
            pairs += [(src, dst), (dst, src)]
        schema = Schema(4, rel_src, rel_dst)
        stores = [_normal_store(f, num_nodes[0], 128)]
        for t in (1, 2, 3):
            stores.append(_normal_store(f, num_nodes[t], 128, scale=0.1))
        return _finish_graph(schema, num_nodes, feat_dim, pairs, stores)

    if cfg.index == 3:
        T, R = 10, 30
        sizes = np.exp(g.uniform(np.log(5e3), np.log(5e5), T))
        num_nodes = [max(8, int(round(s * sc))) for s in sizes]
        feat_dim = [int(x) for x in g.choice([32, 64, 128, 256, 384], T)]
        rel_src = [int(x) for x in g.integers(0, T, R)]
        rel_dst = [int(x) for x in g.integers(0, T, R)]
        schema = Schema(T, rel_src, rel_dst)
        pairs = [_zipf_pairs(g, num_nodes[s], num_nodes[d], max(16, int(round(2_000_000 * sc))))
                 for s, d in zip(rel_src, rel_dst)]
        stores = [_normal_store(f, n, d) for n, d in zip(num_nodes, feat_dim)]
        return _finish_graph(schema, num_nodes, feat_dim, pairs, stores)
    if cfg.index == 7:
        T, n_fwd = 32, 64
        num_nodes = [max(8, int(round(x * sc))) for x in g.integers(60, 400, T)]
        feat_dim = [int(x) for x in g.choice([8, 16, 32, 40], T)]
        rel_src, rel_dst, pairs = [], [], []
        for i in range(n_fwd):
            sT, dT = int(g.integers(0, T)), int(g.integers(0, T))
            src, dst = _zipf_pairs(g, num_nodes[sT], num_nodes[dT], max(4, int(round(g.integers(20, 900) * sc))))
            rel_src += [sT, dT]; rel_dst += [dT, sT]
            pairs += [(src, dst), (dst, src)]
        schema = Schema(T, rel_src, rel_dst)
        stores = [_normal_store(f, n, d) for n, d in zip(num_nodes, feat_dim)]
        return _finish_graph(schema, num_nodes, feat_dim, pairs, stores)
    if cfg.index in (5, 6):
        # Shapes only: 7 vertex types of very unequal size, 52 / 54 forward relations between random type pairs
        # plus their reverses, edge counts spread over three orders of magnitude (many relations are tiny).
        T = 7
        n_fwd, total_nodes, total_edges, width = ((52, 7_300, 24_000, 64) if cfg.index == 5
                                                  else (54, 1_900_000, 2_850_000, 128))
        share = g.dirichlet(np.full(T, 0.6))
        num_nodes = [max(8, int(round(total_nodes * sc * x))) for x in share]
        feat_dim = [width] * T
        e_share = np.exp(g.normal(0.0, 1.8, n_fwd))
        e_share /= e_share.sum()
        rel_src, rel_dst, pairs = [], [], []
        for i in range(n_fwd):
            sT, dT = int(g.integers(0, T)), int(g.integers(0, T))
            src, dst = _zipf_pairs(g, num_nodes[sT], num_nodes[dT], max(4, int(round(total_edges * sc * e_share[i]))))
            rel_src += [sT, dT]; rel_dst += [dT, sT]
            pairs += [(src, dst), (dst, src)]
        schema = Schema(T, rel_src, rel_dst)
        stores = [_normal_store(f, n, d, scale=0.1) for n, d in zip(num_nodes, feat_dim)]
        return _finish_graph(schema, num_nodes, feat_dim, pairs, stores)
    raise ValueError(cfg.index)


def default_target_type(cfg: Config, graph: HeteroGraph) -> int:
    if cfg.index == 0:
        return 1
    if cfg.index in (3, 5, 6, 7):
        inc = np.bincount(graph.schema.rel_dst, minlength=graph.schema.num_types)
        if cfg.index != 3:                             # a type too small to draw the batch from is no target
            inc = np.where(np.asarray(graph.num_nodes) >= cfg.batch, inc, -1)
        return int(np.argmax(inc))                     # ties -> lowest id
    return 0


# --------------------------------------------------------------------------- #
# sampler
# --------------------------------------------------------------------------- #
def _sample_rows(rng, indptr, rows, fanout):
    """For each destination vertex in `rows` pick min(deg, fanout) distinct positions
    of its in-neighbour list, uniformly (Floyd's subset sampling for long lists).
    Returns (flat positions into the neighbour array, flat index into `rows`)."""
    start = indptr[rows]
    deg = indptr[rows + 1] - start
    small = deg <= fanout
    # rows that keep every neighbour
    ks = np.where(small, deg, 0)
    rep = np.repeat(np.arange(len(rows)), ks)
    offs = np.arange(ks.sum()) - np.repeat(np.cumsum(ks) - ks, ks)
    pos_small, row_small = start[rep] + offs, rep
    big = np.nonzero(~small)[0]
    if len(big) == 0:
        return pos_small, row_small
    D = deg[big]
    S = np.full((len(big), fanout), -1, dtype=np.int64)
    for i in range(fanout):
        j = D - fanout + i
        t = np.minimum((rng.random(len(big)) * (j + 1)).astype(np.int64), j)
        dup = (S[:, :i] == t[:, None]).any(axis=1) if i else np.zeros(len(big), bool)
        S[:, i] = np.where(dup, j, t)
    pos_big = (start[big][:, None] + S).ravel()
    row_big = np.repeat(big, fanout)
    pos = np.concatenate([pos_small, pos_big])
    row = np.concatenate([row_small, row_big])
    order = np.argsort(row, kind="stable")
    return pos[order], row[order]


def sample_minibatch(cfg: Config, graph: HeteroGraph, rng=None, target_type: Optional[int] = None,
                     targets: Optional[np.ndarray] = None, shuffle_edges: bool = True) -> MiniBatch:
    sch = graph.schema
    T, R = sch.num_types, sch.num_rels
    if rng is None:
        rng = _streams(cfg.index)["sampler"]
    tt = default_target_type(cfg, graph) if target_type is None else target_type
    if targets is None:
        targets = rng.choice(graph.num_nodes[tt], size=min(cfg.batch, graph.num_nodes[tt]), replace=False)
    dst_ids = [np.zeros(0, dtype=np.int64) for _ in range(T)]
    dst_ids[tt] = np.asarray(targets, dtype=np.int64)
    luts = [np.full(n, -1, dtype=np.int64) for n in graph.num_nodes]
    blocks = []
    for fanout in cfg.fanouts:
        src_ids = [d.copy() for d in dst_ids]
        extra = [[] for _ in range(T)]
        n_cur = [len(d) for d in dst_ids]
        for t in range(T):
            luts[t][dst_ids[t]] = np.arange(len(dst_ids[t]))
        es, ed, et, eid = [], [], [], []
        for r in range(R):
            s, d = sch.rel_src[r], sch.rel_dst[r]
            rows = dst_ids[d]
            if len(rows) == 0:
                continue
            pos, row = _sample_rows(rng, graph.in_indptr[r], rows, fanout)
            if len(pos) == 0:
                continue
            u = graph.in_nbr[r][pos].astype(np.int64)
            loc = luts[s][u]
            new = loc < 0
            if new.any():
                cand = u[new]
                uniq, first = np.unique(cand, return_index=True)
                uniq = uniq[np.argsort(first, kind="stable")]       # first-appearance order
                luts[s][uniq] = n_cur[s] + np.arange(len(uniq))
                n_cur[s] += len(uniq)
                extra[s].append(uniq)
                loc = luts[s][u]
            es.append(loc); ed.append(row.astype(np.int64))
            et.append(np.full(len(pos), r, dtype=np.int32))
            eid.append(graph.edge_off[r] + pos)
        for t in range(T):
            if extra[t]:
                src_ids[t] = np.concatenate([src_ids[t]] + extra[t])
        if es:
            src_l, dst_l = np.concatenate(es), np.concatenate(ed)
            ety, eids = np.concatenate(et), np.concatenate(eid)
        else:
            src_l = dst_l = eids = np.zeros(0, dtype=np.int64)
            ety = np.zeros(0, dtype=np.int32)
        if shuffle_edges and len(src_l):
            p = rng.permutation(len(src_l))
            src_l, dst_l, ety, eids = src_l[p], dst_l[p], ety[p], eids[p]
        blocks.append(Block([len(x) for x in src_ids], [len(x) for x in dst_ids],
                            np.stack([src_l, dst_l]).astype(np.int64), eids.astype(np.int64),
                            ety.astype(np.int32)))
        for t in range(T):                                           # reset lookup tables
            luts[t][src_ids[t]] = -1
        dst_ids = src_ids
    blocks.reverse()
    mb = MiniBatch(ids=dst_ids, blocks=blocks, target_type=tt)
    lab = _streams(cfg.index)["labels"]
    nb = len(targets)
    if cfg.loss == "xent":
        mb.labels = lab.integers(0, cfg.num_classes, nb).astype(np.int64)
    else:
        last = blocks[-1]
        mb.grad_out = []
        for t in range(T):
            shp = (last.n_dst[t], cfg.layer_out[-1])
            mb.grad_out.append(np.ones(shp, np.float32) if cfg.loss == "sum"
                               else lab.standard_normal(shp, dtype=np.float32))
    return mb


# --------------------------------------------------------------------------- #
# weights
# --------------------------------------------------------------------------- #
def _glorot(rng, fan_in, fan_out, shape):
    a = np.sqrt(6.0 / (fan_in + fan_out))
    return rng.uniform(-a, a, size=shape).astype(np.float32)


def init_weights(cfg: Config, graph: HeteroGraph) -> List[LayerWeights]:
    rng = _streams(cfg.index)["weights"]
    sch = graph.schema
    T, R = sch.num_types, sch.num_rels
    layers = []
    in_dim = list(graph.feat_dim)
    for li, H in enumerate(cfg.layer_out):
        lw = LayerWeights(in_dim=list(in_dim), out_dim=H, w_rel=[], w_root=[], bias=[], relu=cfg.relu[li])
        if cfg.kind == "rgcn":
            lw.w_rel = [_glorot(rng, in_dim[sch.rel_src[r]], H, (in_dim[sch.rel_src[r]], H)) for r in range(R)]
            lw.w_root = [_glorot(rng, in_dim[t], H, (in_dim[t], H)) for t in range(T)]
        else:
            D = H // cfg.heads
            lw.w_type = [_glorot(rng, in_dim[t], H, (in_dim[t], H)) for t in range(T)]
            lw.a_src = [_glorot(rng, D, 1, (cfg.heads, D)) for _ in range(R)]
            lw.a_dst = [_glorot(rng, D, 1, (cfg.heads, D)) for _ in range(R)]
            lw.w_sem = _glorot(rng, H, 128, (H, 128))
            lw.b_sem = rng.uniform(-0.1, 0.1, 128).astype(np.float32)
            lw.q_sem = _glorot(rng, 128, 1, (128,))
        lw.bias = [rng.uniform(-0.1, 0.1, H).astype(np.float32) if cfg.bias else None for _ in range(T)]
        layers.append(lw)
        in_dim = [H] * T
    return layers


# --------------------------------------------------------------------------- #
# inputs of the optimiser tests (plain normal draws; no update arithmetic here)
# --------------------------------------------------------------------------- #
def optimizer_case(seed: int, shapes: Sequence[Sequence[int]], steps: int):
    """Parameters ~ N(0, 0.1) and, per step, gradients ~ N(0, 1) * 10^U(-4, 0) per tensor."""
    rng = np.random.default_rng([MASTER_SEED, 31337, seed])
    theta = [rng.normal(0.0, 0.1, size=s).astype(np.float32) for s in shapes]
    grads = [[(rng.normal(0.0, 1.0, size=s) * 10.0 ** rng.uniform(-4, 0)).astype(np.float32) for s in shapes]
             for _ in range(steps)]
    return theta, grads
