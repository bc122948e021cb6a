"""Pins for the oracle's integer outputs (type-first offsets, Algorithm 2 selection,
merged CSR and its transpose) and for the synthetic sampler's invariants."""
import numpy as np
import pytest

from oracle import hgnn_oracle as O
from workloads import make_config, build_graph, sample_minibatch, bf16_round


def _lexsort_csr(block, rel_src, rel_dst):
    """Independent construction with numpy.lexsort (stable on ties by position)."""
    R = len(rel_src)
    et = block.edge_type.astype(np.int64)
    src, dst = block.edge_index[0], block.edge_index[1]
    row_off = np.concatenate([[0], np.cumsum(block.n_src)])
    rel_row_off = np.concatenate([[0], np.cumsum([block.n_dst[rel_dst[r]] for r in range(R)])])
    E = len(et)
    order = np.lexsort((np.arange(E), dst, et))
    rho = rel_row_off[et] + dst
    rowptr = np.concatenate([[0], np.cumsum(np.bincount(rho, minlength=rel_row_off[-1]))])
    colidx = (row_off[np.array(rel_src)[et]] + src)[order]
    corder = np.lexsort((np.arange(E), colidx))
    cptr = np.concatenate([[0], np.cumsum(np.bincount(colidx, minlength=row_off[-1]))])
    crow = rho[order][corder]
    return dict(row_off=row_off, rel_row_off=rel_row_off, rowptr=rowptr, colidx=colidx, perm=order,
                cptr=cptr, crow=crow, cperm=corder)


@pytest.mark.parametrize("index,scale", [(0, 1.0), (2, 0.01), (3, 0.002)])
def test_semantic_csr_matches_lexsort(index, scale):
    cfg = make_config(index, scale=scale, batch=64)
    g = build_graph(cfg)
    mb = sample_minibatch(cfg, g)
    sch = g.schema
    for b in mb.blocks:
        sel = O.edge_index_select(b.edge_index, sch.num_rels, edge_id=b.edge_id, global_edge_type=g.edge_type)
        sel2 = O.edge_index_select(b.edge_index, sch.num_rels, edge_type=b.edge_type)
        for a, c in zip(sel, sel2):
            assert all(np.array_equal(u, v) for u, v in zip(a, c))
        csr = O.semantic_csr(sel, sch.rel_src, sch.rel_dst, b.n_src, b.n_dst)
        ref = _lexsort_csr(b, sch.rel_src, sch.rel_dst)
        for k, v in ref.items():
            assert np.array_equal(csr[k], v.astype(np.int32)), k
        counts = [len(s[0]) for s in sel]
        assert np.array_equal(csr["rel_edge_off"], np.concatenate([[0], np.cumsum(counts)]))


def test_selection_keeps_input_order():
    ei = np.array([[5, 1, 7, 1, 3], [0, 2, 0, 2, 1]])
    et = np.array([1, 0, 1, 0, 1], dtype=np.int32)
    sel = O.edge_index_select(ei, 3, edge_type=et)
    assert sel[0][0].tolist() == [1, 1] and sel[0][2].tolist() == [1, 3]
    assert sel[1][0].tolist() == [5, 7, 3] and sel[1][1].tolist() == [0, 0, 1] and sel[1][2].tolist() == [0, 2, 4]
    assert len(sel[2][0]) == 0


def test_semantic_csr_rejects_out_of_range():
    sel = [(np.array([3]), np.array([0]), np.array([0]))]
    with pytest.raises(ValueError):
        O.semantic_csr(sel, [0], [0], [3], [1])


def test_merge_features_offsets_and_rows():
    rng = np.random.default_rng(0)
    stores = [rng.standard_normal((10, 3)), rng.standard_normal((7, 5)), rng.standard_normal((4, 2))]
    ids = [np.array([9, 0, 3]), np.array([], dtype=np.int64), np.array([2, 2])]
    blocks, row_off, elem_off, flat = O.merge_features(stores, ids)
    assert row_off.tolist() == [0, 3, 3, 5] and elem_off.tolist() == [0, 9, 9, 13]
    assert np.array_equal(flat[:9].reshape(3, 3), stores[0][[9, 0, 3]])
    assert np.array_equal(flat[9:].reshape(2, 2), stores[2][[2, 2]])
    assert row_off.dtype == np.int32 and elem_off.dtype == np.int64


@pytest.mark.parametrize("index,scale", [(0, 1.0), (1, 0.01), (3, 0.002), (4, 0.01)])
def test_sampler_invariants(index, scale):
    cfg = make_config(index, scale=scale, batch=32)
    g = build_graph(cfg)
    mb = sample_minibatch(cfg, g)
    sch = g.schema
    assert len(mb.blocks) == len(cfg.fanouts)
    n_prev = None
    # blocks are in execution order: the outermost hop first
    for li, b in enumerate(mb.blocks):
        fan = cfg.fanouts[len(cfg.fanouts) - 1 - li]
        if n_prev is not None:
            assert b.n_src == n_prev                  # this layer reads the previous layer's output rows
        n_prev = b.n_dst
        assert all(d <= s for d, s in zip(b.n_dst, b.n_src))
        assert np.array_equal(g.edge_type[b.edge_id], b.edge_type)
        for r in range(sch.num_rels):
            m = b.edge_type == r
            s, d = b.edge_index[0][m], b.edge_index[1][m]
            if len(s) == 0:
                continue
            assert s.min() >= 0 and s.max() < b.n_src[sch.rel_src[r]]
            assert d.min() >= 0 and d.max() < b.n_dst[sch.rel_dst[r]]
            assert len(np.unique(s * (d.max() + 1) + d)) == len(s)      # no duplicate (r, v, u)
            cnt = np.bincount(d, minlength=b.n_dst[sch.rel_dst[r]])
            assert cnt.max() <= fan
    # first block's ids: row lengths equal min(degree, fanout) for the outermost hop
    b = mb.blocks[0]
    fan = cfg.fanouts[-1]
    ids = mb.ids
    for r in range(sch.num_rels):
        d = sch.rel_dst[r]
        if b.n_dst[d] == 0:
            continue
        gids = ids[d][: b.n_dst[d]]
        deg = g.in_indptr[r][gids + 1] - g.in_indptr[r][gids]
        cnt = np.bincount(b.edge_index[1][b.edge_type == r], minlength=b.n_dst[d])
        assert np.array_equal(cnt, np.minimum(deg, fan))
    assert mb.blocks[-1].n_dst[mb.target_type] == min(32, g.num_nodes[mb.target_type])
    # sampled edges are edges of the graph
    b = mb.blocks[0]
    for k in range(0, b.edge_index.shape[1], max(1, b.edge_index.shape[1] // 50)):
        r = b.edge_type[k]
        u = ids[sch.rel_src[r]][b.edge_index[0][k]]
        v = ids[sch.rel_dst[r]][b.edge_index[1][k]]
        lo, hi = g.in_indptr[r][v], g.in_indptr[r][v + 1]
        assert u in g.in_nbr[r][lo:hi]


def test_sampler_is_deterministic():
    cfg = make_config(0)
    a = sample_minibatch(cfg, build_graph(cfg))
    b = sample_minibatch(cfg, build_graph(cfg))
    assert np.array_equal(a.blocks[0].edge_index, b.blocks[0].edge_index)
    assert all(np.array_equal(x, y) for x, y in zip(a.ids, b.ids))


def test_bf16_round_ties_to_even():
    x = np.array([1.0, 1.00390625, 1.01171875, 1.0 + 2 ** -9, -3.1415927, 0.0, 65504.0], dtype=np.float32)
    r = bf16_round(x)
    assert r[0] == 1.0
    assert r[1] == 1.0                      # halfway between 1.0 and 1.0078125 -> even mantissa
    assert r[2] == np.float32(1.015625)     # halfway, odd below -> rounds up to even
    assert r[3] == 1.0
    assert np.all((r.view(np.uint32) & 0xFFFF) == 0)
    assert np.all(np.abs(r - x) <= np.abs(x) * 2 ** -8)
