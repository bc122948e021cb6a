"""CPU-only checks of the C-ABI library: it loads, exports every symbol the header declares,
validates arguments, and its multi-threaded host semantic-graph build (which needs no GPU when
the context is created with device < 0) is bit-exact against the oracle."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from oracle import hgnn_oracle as O
from workloads import make_config, build_graph, sample_minibatch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def B():
    lib = os.path.join(ROOT, "paper_2408_08490_amd", "libhgnn.so")
    if not os.path.exists(lib):                      # build only when nothing has been built
        from paper_2408_08490_amd.build import build_library
        build_library(verbose=False)
    from paper_2408_08490_amd import binding
    return binding


def test_exports_match_header(B):
    hdr = open(os.path.join(ROOT, "include", "hgnn.h")).read()
    declared = set(re.findall(r"^(?:hgnn_status|void|const char \*)\s*(hgnn_[a-z_0-9]+)\s*\(", hdr, flags=re.M))
    assert declared, "no declarations found"
    for name in declared:
        assert hasattr(B.lib, name), f"{name} declared in include/hgnn.h but not exported"
    assert set(B.EXPORTS) == declared


def _host_ctx(B, sch, dtype="f32", threads=4, concurrent_builds=0):
    return B.Context(sch.rel_src, sch.rel_dst, sch.num_types, dtype, device=-1, host_threads=threads,
                     concurrent_builds=concurrent_builds)


@pytest.mark.parametrize("index,scale,threads", [(0, 1.0, 1), (0, 1.0, 4), (2, 0.02, 8), (3, 0.003, 3), (5, 1.0, 2),
                                                 (6, 0.1, 4), (7, 1.0, 3)])
@pytest.mark.parametrize("use_edge_id", [False, True, "registered", "registered_interleaved", "no_permutation"])
def test_host_build_bit_exact(B, index, scale, threads, use_edge_id):
    cfg = make_config(index, scale=scale, batch=96)
    g = build_graph(cfg)
    mb = sample_minibatch(cfg, g)
    ctx = _host_ctx(B, g.schema, threads=threads)
    with_perm = use_edge_id != "no_permutation"
    if not with_perm:                               # the build that leaves perm / cperm out: all else unchanged
        ctx.hgnn_set_build_permutation(False)
        use_edge_id = True
    if use_edge_id == "registered":                 # edge ids alone, types from the table the context keeps
        ctx.hgnn_set_edge_types(g.edge_type)        # (ids grouped by relation: few runs of equal type)
        gr = ctx.hgnn_build_semantic_csr(mb.blocks, None, use_edge_id=True)
    elif use_edge_id == "registered_interleaved":   # the same through renumbered ids: types alternate all along
        import copy
        p = np.random.default_rng(3).permutation(g.edge_type.size)
        table = np.empty_like(g.edge_type)
        table[p] = g.edge_type
        ctx.hgnn_set_edge_types(table)
        blocks = []
        for b in mb.blocks:
            b2 = copy.copy(b)
            b2.edge_id = p[b.edge_id]
            blocks.append(b2)
        gr = ctx.hgnn_build_semantic_csr(blocks, None, use_edge_id=True)
    else:
        gr = ctx.hgnn_build_semantic_csr(mb.blocks, g.edge_type, use_edge_id=use_edge_id)
    gr.wait()
    for l, b in enumerate(mb.blocks):
        sel = O.edge_index_select(b.edge_index, g.schema.num_rels, edge_type=b.edge_type)
        ref = O.semantic_csr(sel, g.schema.rel_src, g.schema.rel_dst, b.n_src, b.n_dst)
        v = gr.host_view(l)
        assert v["rows"] == ref["rowptr"].size - 1 and v["edges"] == ref["colidx"].size
        for k in ("rel_row_off", "rel_edge_off", "rowptr", "colidx", "perm", "cptr", "crow", "cperm"):
            if k in ("perm", "cperm") and not with_perm:
                assert v[k] is None
                continue
            assert np.array_equal(v[k], ref[k]), (l, k)
    gr.release()
    ctx.close()


def test_registered_edge_types_errors(B):
    cfg = make_config(0)
    g = build_graph(cfg)
    mb = sample_minibatch(cfg, g)
    ctx = _host_ctx(B, g.schema)
    with pytest.raises(B.HgnnError, match="none registered"):       # edge ids alone need a table
        ctx.hgnn_build_semantic_csr(mb.blocks, None, use_edge_id=True)
    bad = g.edge_type.copy()
    bad[3] = g.schema.num_rels
    with pytest.raises(B.HgnnError, match="outside"):
        ctx.hgnn_set_edge_types(bad)
    short = g.edge_type[: int(mb.blocks[0].edge_id.max())]         # at least one sampled id is past its end
    ctx.hgnn_set_edge_types(short)
    gr = ctx.hgnn_build_semantic_csr(mb.blocks, None, use_edge_id=True)
    with pytest.raises(B.HgnnError, match="registered edge-type table"):
        gr.wait()
    gr.release()
    ctx.hgnn_set_edge_types(g.edge_type)                            # a later registration replaces the table
    gr = ctx.hgnn_build_semantic_csr(mb.blocks, None, use_edge_id=True)
    gr.wait()
    gr.release()
    ctx.close()


def test_host_build_int32_indices_and_repeat(B):
    cfg = make_config(0)
    g = build_graph(cfg)
    mb = sample_minibatch(cfg, g)
    ctx = _host_ctx(B, g.schema)
    b = mb.blocks[0]

    class Blk:
        pass
    b32 = Blk()
    b32.n_src, b32.n_dst, b32.edge_type = b.n_src, b.n_dst, b.edge_type
    b32.edge_index = b.edge_index.astype(np.int32)
    views = []
    for _ in range(3):                              # pooled buffers are reused: results must not change
        gr = ctx.hgnn_build_semantic_csr([b32])
        views.append(gr.host_view(0))
        gr.release()
    gr = ctx.hgnn_build_semantic_csr([b])
    v64 = gr.host_view(0)
    gr.release()
    for v in views:
        for k in ("rowptr", "colidx", "perm", "cptr", "crow", "cperm"):
            assert np.array_equal(v[k], v64[k])
    ctx.close()


def test_empty_layer_and_empty_relation(B):
    from workloads import Schema

    class Blk:
        pass
    sch = Schema(2, [0, 1], [1, 1])
    ctx = _host_ctx(B, sch)
    b = Blk()
    b.n_src, b.n_dst = [3, 2], [0, 2]
    b.edge_index = np.zeros((2, 0), dtype=np.int64)
    b.edge_type = np.zeros(0, dtype=np.int32)
    gr = ctx.hgnn_build_semantic_csr([b])
    v = gr.host_view(0)
    assert v["rows"] == 4 and v["edges"] == 0
    assert v["rowptr"].tolist() == [0] * 5 and v["cptr"].tolist() == [0] * 6
    assert v["rel_row_off"].tolist() == [0, 2, 4]
    gr.release()
    ctx.close()


def _bad_block(mb, **kw):
    class Blk:
        pass
    b = Blk()
    src = mb.blocks[0]
    b.n_src, b.n_dst = list(src.n_src), list(src.n_dst)
    b.edge_index, b.edge_type = src.edge_index.copy(), src.edge_type.copy()
    for k, v in kw.items():
        setattr(b, k, v)
    return b


def test_validation_errors(B):
    cfg = make_config(0)
    g = build_graph(cfg)
    mb = sample_minibatch(cfg, g)
    ctx = _host_ctx(B, g.schema)
    # edge type out of range
    et = mb.blocks[0].edge_type.copy(); et[5] = 7
    gr = ctx.hgnn_build_semantic_csr([_bad_block(mb, edge_type=et)])
    with pytest.raises(B.HgnnError) as e:
        gr.wait()
    assert e.value.status == -1 and "type" in str(e.value)
    gr.release()
    # source index out of range
    ei = mb.blocks[0].edge_index.copy(); ei[0, 3] = 10 ** 6
    gr = ctx.hgnn_build_semantic_csr([_bad_block(mb, edge_index=ei)])
    with pytest.raises(B.HgnnError):
        gr.host_view(0)
    gr.release()
    # negative destination
    ei = mb.blocks[0].edge_index.copy(); ei[1, 0] = -1
    gr = ctx.hgnn_build_semantic_csr([_bad_block(mb, edge_index=ei)])
    with pytest.raises(B.HgnnError):
        gr.wait()
    gr.release()
    # n_dst > n_src is an argument error reported at once
    nd = list(mb.blocks[0].n_dst); nd[0] = mb.blocks[0].n_src[0] + 1
    with pytest.raises(B.HgnnError) as e:
        ctx.hgnn_build_semantic_csr([_bad_block(mb, n_dst=nd)])
    assert e.value.status == -1
    # a good build still works afterwards
    gr = ctx.hgnn_build_semantic_csr(mb.blocks)
    gr.wait(); gr.release()
    ctx.close()


def test_create_rejects_bad_schema(B):
    with pytest.raises(B.HgnnError):
        B.Context([0, 5], [0, 0], 2, "f32", device=-1)
    with pytest.raises(B.HgnnError):
        B.Context(list(range(200)), list(range(200)), 200, "f32", device=-1)


def test_device_entry_points_refuse_host_only_context(B):
    cfg = make_config(0)
    g = build_graph(cfg)
    ctx = _host_ctx(B, g.schema)
    loss = C.c_float()
    st = B.lib.hgnn_softmax_xent(ctx.handle, None, None, None, 0, 4, C.byref(loss), None)
    assert st == -6
    assert b"host-only" in B.lib.hgnn_last_error()
    ctx.close()


@pytest.mark.parametrize("threads,builders", [(4, 0), (4, 4), (6, 4), (8, 2)])
def test_overlapping_builds_from_one_context(B, threads, builders):
    """Several builders (single- or multi-threaded) work on queued graphs at once."""
    cfg = make_config(2, scale=0.02, batch=64)
    g = build_graph(cfg)
    mbs = [sample_minibatch(cfg, g, rng=np.random.default_rng(i)) for i in range(6)]
    ctx = _host_ctx(B, g.schema, threads=threads, concurrent_builds=builders)
    graphs = [ctx.hgnn_build_semantic_csr(mb.blocks) for mb in mbs]       # all queued before any wait
    for mb, gr in zip(mbs, graphs):
        for l, b in enumerate(mb.blocks):
            sel = O.edge_index_select(b.edge_index, g.schema.num_rels, edge_type=b.edge_type)
            ref = O.semantic_csr(sel, g.schema.rel_src, g.schema.rel_dst, b.n_src, b.n_dst)
            v = gr.host_view(l)
            for k in ("rowptr", "colidx", "cptr", "crow"):
                assert np.array_equal(v[k], ref[k])
        gr.release()
    ctx.close()


def test_transpose_restricted_to_wanted_types(B):
    cfg = make_config(2, scale=0.02, batch=96)
    g = build_graph(cfg)
    mb = sample_minibatch(cfg, g)
    ctx = _host_ctx(B, g.schema, threads=4)
    want = [0, 1, 1, 1]
    gr = ctx.hgnn_build_semantic_csr(mb.blocks, g.edge_type, use_edge_id=True,
                                     transpose_types=[want] + [None] * (len(mb.blocks) - 1))
    for l, b in enumerate(mb.blocks):
        sel = O.edge_index_select(b.edge_index, g.schema.num_rels, edge_type=b.edge_type)
        ref = O.semantic_csr(sel, g.schema.rel_src, g.schema.rel_dst, b.n_src, b.n_dst,
                             transpose_types=want if l == 0 else None)
        v = gr.host_view(l)
        for k in ("rowptr", "colidx", "perm", "cptr", "crow", "cperm"):
            assert np.array_equal(v[k], ref[k]), (l, k)
        if l == 0:
            assert v["transpose_edges"] < v["edges"] and v["cptr"][b.n_src[0]] == 0
    gr.release()
    ctx.close()


def test_attention_plan_validation_without_gpu(B):
    """hgnn_layer_workspace_bytes needs no GPU: the attention variant's shape rules are checked on a host-only
    context (head width a power of two times 16 bytes, H a multiple of the head count, all transpose entries)."""
    import torch
    cfg = make_config(4, scale=0.01, batch=8)
    g = build_graph(cfg)
    mb = sample_minibatch(cfg, g)
    sch = g.schema
    T, R = sch.num_types, sch.num_rels
    ctx = B.Context(sch.rel_src, sch.rel_dst, T, "f32", device=-1, host_threads=2, heads=8, attention=True)
    gr = ctx.hgnn_build_semantic_csr(mb.blocks, g.edge_type, use_edge_id=True)
    gr.wait()

    def layer(H):
        D = max(H // 8, 1)
        attn = dict(w_type=[torch.zeros(f, H) for f in g.feat_dim], a_src=[torch.zeros(8, D) for _ in range(R)],
                    a_dst=[torch.zeros(8, D) for _ in range(R)], w_sem=torch.zeros(H, 128), b_sem=torch.zeros(128),
                    q_sem=torch.zeros(128))
        return B.Layer(ctx, g.feat_dim, H, True, None, None, None, attn=attn)

    saved, scratch = ctx.hgnn_layer_workspace_bytes(gr, 0, layer(256))
    b0 = mb.blocks[0]
    rows = sum(b0.n_dst[d] for d in sch.rel_dst)
    assert saved >= (sum(b0.n_src) + rows) * 256 * 4 and scratch > 0
    for bad_h in (250, 8 * 12, 8 * 2):          # not a multiple of 8 heads / head width 12 or 2 floats
        with pytest.raises(B.HgnnError) as e:
            ctx.hgnn_layer_workspace_bytes(gr, 0, layer(bad_h))
        assert e.value.status in (-1, -6)
    gr.release()
    # a graph whose transpose skips a type cannot serve the attention backward
    gr2 = ctx.hgnn_build_semantic_csr(mb.blocks, g.edge_type, use_edge_id=True,
                                      transpose_types=[[0, 1, 1, 1]] + [None] * (len(mb.blocks) - 1))
    gr2.wait()
    with pytest.raises(B.HgnnError):
        ctx.hgnn_layer_workspace_bytes(gr2, 0, layer(256))
    gr2.release()
    ctx.close()


@pytest.mark.parametrize("dtype,width,vec", [("f32", 6, 4), ("f32", 130, 4), ("bf16", 12, 8), ("bf16", 4, 8)])
def test_feature_widths_off_the_16_byte_grid_are_refused(B, dtype, width, vec):
    """Rows move as 16-byte vectors, so every entry point that takes a feature width refuses one that is not a
    multiple of 16 bytes / sizeof(dtype) before it touches the device: the layer plan (workspace query), the
    feature merge and the row-wise Adam update, each with a message that names the width and the multiple."""
    import torch
    cfg = make_config(0)
    g = build_graph(cfg)
    mb = sample_minibatch(cfg, g)
    sch = g.schema
    T, R = sch.num_types, sch.num_rels
    ctx = B.Context(sch.rel_src, sch.rel_dst, T, dtype, device=-1, host_threads=2)
    gr = ctx.hgnn_build_semantic_csr(mb.blocks)
    gr.wait()
    good = [64] * T
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16

    def layer(dims):                                     # host tensors: the query reads no weight, only pointers
        return B.Layer(ctx, dims, 64, True, [torch.zeros(max(dims[s], 1), 64, dtype=tdt) for s in sch.rel_src],
                       [torch.zeros(max(d, 1), 64, dtype=tdt) for d in dims], [torch.zeros(64) for _ in dims])

    saved, scratch = ctx.hgnn_layer_workspace_bytes(gr, 0, layer(good))
    assert saved > 0 and scratch > 0
    for t in range(T):
        dims = list(good); dims[t] = width
        with pytest.raises(B.HgnnError) as e:
            ctx.hgnn_layer_workspace_bytes(gr, 0, layer(dims))
        assert e.value.status == -6 and "in_dim[%d]=%d is not a positive multiple of %d" % (t, width, vec) in str(e.value)
    with pytest.raises(B.HgnnError):
        ctx.hgnn_layer_workspace_bytes(gr, 0, layer([0] + good[1:]))
    gr.release()
    # the merge: arguments are validated before the host-only context is refused
    vp = C.c_void_p
    store = (vp * T)(*[None] * T)
    ids = (vp * T)(*[None] * T)
    nr = (C.c_int64 * T)(*[0] * T)
    fd = (C.c_int32 * T)(*([64] * (T - 1) + [width]))
    ro, eo = (C.c_int32 * (T + 1))(), (C.c_int64 * (T + 1))()
    st = B.lib.hgnn_merge_features(ctx.handle, None, store, fd, ids, nr, None, ro, eo)
    assert st == -1 and ("feat_dim[%d]=%d is not a positive multiple of %d" % (T - 1, width, vec)).encode() in B.lib.hgnn_last_error()
    hp = B.AdamParams(1e-3, 0.9, 0.999, 1e-8, 1)
    st = B.lib.hgnn_adam_update_rows(ctx.handle, None, None, None, None, None, width, None, 0, None, C.byref(hp))
    assert st == -1 and ("feat_dim=%d is not a positive multiple of %d" % (width, vec)).encode() in B.lib.hgnn_last_error()
    ctx.close()


def test_ablation_entry_points_validate_before_touching_the_device(B):
    """The baselines' entry points on a host-only context: argument errors come first, then the refusal to run device
    work (never a crash): the device-side index build, the index-first feature stage, the gather-from-stores layer."""
    cfg = make_config(0)
    g = build_graph(cfg)
    mb = sample_minibatch(cfg, g)
    sch = g.schema
    T = sch.num_types
    ctx = _host_ctx(B, sch)
    with pytest.raises(B.HgnnError) as e:
        B._check(B.lib.hgnn_build_semantic_csr_device(ctx.handle, None, 1, (B.CooLayer * 1)(), C.byref(C.c_void_p()), None))
    assert e.value.status == -6 and "host-only" in str(e.value)
    vp = C.c_void_p
    none = (vp * T)(*[None] * T)
    nr = (C.c_int64 * T)(*[0] * T)
    ro, eo = (C.c_int32 * (T + 1))(), (C.c_int64 * (T + 1))()
    ragged = (C.c_int32 * T)(*([64] * (T - 1) + [32]))
    st = B.lib.hgnn_merge_features_index_first(ctx.handle, None, none, ragged, none, nr, none, None)
    assert st == -6 and b"one width" in B.lib.hgnn_last_error()
    st = B.lib.hgnn_select_type_first(ctx.handle, None, None, ragged, none, nr, None, ro, eo)
    assert st == -6 and b"one width" in B.lib.hgnn_last_error()
    same = (C.c_int32 * T)(*[64] * T)
    st = B.lib.hgnn_merge_features_index_first(ctx.handle, None, none, same, none, nr, None, None)
    assert st == -1                                   # NULL position table
    st = B.lib.hgnn_select_type_first(ctx.handle, None, None, same, none, nr, None, ro, eo)
    assert st == -6 and b"host-only" in B.lib.hgnn_last_error()
    st = B.lib.hgnn_layer_fwd_gather(ctx.handle, None, None, 0, None, None, None, None, None, None, 0, None, 0)
    assert st == -1
    ctx.close()


# ---- sampling in the loop: the library's sampler against the sampler oracle, bit for bit ----
def _sampler(B, ctx, g):
    return ctx.hgnn_sampler_create(g.num_nodes, g.in_indptr, g.in_nbr, g.edge_off)


@pytest.mark.parametrize("index,scale,fanouts,nt,threads,conc", [(0, 1.0, [5], 64, 1, 0), (0, 1.0, [3, 2, 2], 40, 4, 2),
                                                                 (2, 0.02, [6, 4], 300, 4, 4), (5, 1.0, [4, 4], 60, 2, 0),
                                                                 (3, 0.003, [5, 5], 50, 3, 0)])
def test_sampler_matches_oracle_and_feeds_the_build(B, index, scale, fanouts, nt, threads, conc):
    from oracle import sampler_oracle as SO
    from workloads.synth import default_target_type
    cfg = make_config(index, scale=scale, batch=nt)
    g = build_graph(cfg)
    sch = g.schema
    tt = default_target_type(cfg, g)
    ctx = _host_ctx(B, sch, threads=threads, concurrent_builds=conc)
    sm = _sampler(B, ctx, g)
    rng = np.random.default_rng(11)
    graphs, wants = [], []
    for k in range(3):                                              # several in flight on the same builders
        targets = rng.choice(g.num_nodes[tt], nt, replace=False)
        graphs.append(ctx.hgnn_sample_and_build(sm, tt, targets, fanouts, seed=1000 + k))
        wants.append(SO.sample_minibatch(g.num_nodes, sch.rel_src, sch.rel_dst, g.in_indptr, g.in_nbr, g.edge_off, tt,
                                         targets, fanouts, 1000 + k))
    for gr, want in zip(graphs, wants):
        n_rows, ids = gr.ids()
        assert n_rows == [len(x) for x in want["ids"]]
        for t in range(sch.num_types):
            assert np.array_equal(ids[t], want["ids"][t]), t
        for l, wb in enumerate(want["blocks"]):
            v = gr.minibatch_view(l)
            assert v["n_src"] == wb["n_src"] and v["n_dst"] == wb["n_dst"]
            assert np.array_equal(v["edge_index"], wb["edge_index"]) and np.array_equal(v["edge_id"], wb["edge_id"])
            sel = O.edge_index_select(wb["edge_index"], sch.num_rels, edge_id=wb["edge_id"], global_edge_type=g.edge_type)
            ref = O.semantic_csr(sel, sch.rel_src, sch.rel_dst, wb["n_src"], wb["n_dst"])
            hv = gr.host_view(l)
            for key in ("rel_row_off", "rel_edge_off", "rowptr", "colidx", "perm", "cptr", "crow", "cperm"):
                assert np.array_equal(hv[key], ref[key]), (l, key)
        gr.release()
    sm.close()
    ctx.close()


def test_attention_context_keeps_the_permutations(B):
    """hgnn_set_build_permutation(0) is ignored by a context of the attention variant (its backward walks cperm);
    a NULL context is an error."""
    import ctypes as C
    cfg = make_config(0)
    g = build_graph(cfg)
    mb = sample_minibatch(cfg, g)
    sch = g.schema
    ctx = B.Context(sch.rel_src, sch.rel_dst, sch.num_types, "f32", device=-1, host_threads=2, heads=2, attention=True)
    ctx.hgnn_set_build_permutation(False)
    gr = ctx.hgnn_build_semantic_csr(mb.blocks, g.edge_type, use_edge_id=True)
    gr.wait()
    for l, b in enumerate(mb.blocks):
        sel = O.edge_index_select(b.edge_index, sch.num_rels, edge_type=b.edge_type)
        ref = O.semantic_csr(sel, sch.rel_src, sch.rel_dst, b.n_src, b.n_dst)
        v = gr.host_view(l)
        assert np.array_equal(v["perm"], ref["perm"]) and np.array_equal(v["cperm"], ref["cperm"])
    gr.release()
    ctx.close()
    assert B.STATUS_NAMES[B.lib.hgnn_set_build_permutation(None, 0)] == "HGNN_EINVAL"


def test_sampler_errors(B):
    cfg = make_config(0)
    g = build_graph(cfg)
    ctx = _host_ctx(B, g.schema)
    sm = _sampler(B, ctx, g)
    with pytest.raises(B.HgnnError, match="not a vertex"):
        ctx.hgnn_sample_and_build(sm, 1, [0, g.num_nodes[1]], [5], 1)
    with pytest.raises(B.HgnnError, match="fanouts"):
        ctx.hgnn_sample_and_build(sm, 1, [0, 1], [0], 1)
    with pytest.raises(B.HgnnError, match="target_type"):
        ctx.hgnn_sample_and_build(sm, 7, [0, 1], [5], 1)
    gr = ctx.hgnn_sample_and_build(sm, 1, [3, 4, 3], [5], 1)       # a repeated target is found by the sampling task
    with pytest.raises(B.HgnnError, match="listed twice"):
        gr.ids()
    with pytest.raises(B.HgnnError, match="listed twice"):
        gr.wait()
    gr.release()
    gr = ctx.hgnn_sample_and_build(sm, 1, [3, 4, 5], [5], 1)       # the tables were put back: the next one works
    assert gr.ids()[0][1] >= 3
    gr.release()
    plain = ctx.hgnn_build_semantic_csr(sample_minibatch(cfg, g).blocks, g.edge_type, use_edge_id=True)
    with pytest.raises(B.HgnnError, match="not made by"):
        plain.ids()
    plain.release()
    bad = [p.copy() for p in g.in_indptr]
    bad[0][-1] += 1
    with pytest.raises(B.HgnnError, match="does not span"):
        ctx.hgnn_sampler_create(g.num_nodes, bad, g.in_nbr, g.edge_off)
    sm.close()
    ctx.close()


def test_host_build_three_int_records():
    """The sort's level-1 records take two ints where the payload fits 20 bits and three otherwise; no test graph is
    large enough for the latter, so a child process asks for it and repeats a bit-exact comparison."""
    import subprocess
    import sys
    code = (
        "import numpy as np\n"
        "from oracle import hgnn_oracle as O\n"
        "from paper_2408_08490_amd import binding as B\n"
        "from workloads import make_config, build_graph, sample_minibatch\n"
        "cfg = make_config(2, scale=0.02, batch=96); g = build_graph(cfg); mb = sample_minibatch(cfg, g)\n"
        "ctx = B.Context(g.schema.rel_src, g.schema.rel_dst, g.schema.num_types, 'f32', device=-1, host_threads=3)\n"
        "gr = ctx.hgnn_build_semantic_csr(mb.blocks, g.edge_type, use_edge_id=True, transpose_types=[[0, 1, 1, 1], None])\n"
        "for l, b in enumerate(mb.blocks):\n"
        "    sel = O.edge_index_select(b.edge_index, g.schema.num_rels, edge_type=b.edge_type)\n"
        "    ref = O.semantic_csr(sel, g.schema.rel_src, g.schema.rel_dst, b.n_src, b.n_dst,\n"
        "                         transpose_types=[0, 1, 1, 1] if l == 0 else None)\n"
        "    v = gr.host_view(l)\n"
        "    for k in ('rowptr', 'colidx', 'perm', 'cptr', 'crow', 'cperm'):\n"
        "        assert np.array_equal(v[k], ref[k]), (l, k)\n"
        "gr.release()\n"
        "ctx.hgnn_set_build_permutation(False)\n"      # the same records with the permutations left out
        "gr = ctx.hgnn_build_semantic_csr(mb.blocks, g.edge_type, use_edge_id=True, transpose_types=[[0, 1, 1, 1], None])\n"
        "for l, b in enumerate(mb.blocks):\n"
        "    sel = O.edge_index_select(b.edge_index, g.schema.num_rels, edge_type=b.edge_type)\n"
        "    ref = O.semantic_csr(sel, g.schema.rel_src, g.schema.rel_dst, b.n_src, b.n_dst,\n"
        "                         transpose_types=[0, 1, 1, 1] if l == 0 else None)\n"
        "    v = gr.host_view(l)\n"
        "    assert v['perm'] is None and v['cperm'] is None\n"
        "    for k in ('rowptr', 'colidx', 'cptr', 'crow'):\n"
        "        assert np.array_equal(v[k], ref[k]), (l, k)\n"
        "print('ok')\n")
    env = dict(os.environ, HGNN_WIDE_RECORDS="1")
    r = subprocess.run([sys.executable, "-c", code], env=env, capture_output=True, text=True, cwd=ROOT, timeout=300)
    assert r.returncode == 0 and r.stdout.strip().endswith("ok"), r.stderr[-2000:]


def test_header_compiles_as_c99(tmp_path):
    """The boundary is a C ABI: include/hgnn.h alone must go through a C99 compiler without warnings."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler")
    src = tmp_path / "use_hgnn.c"
    src.write_text('#include "hgnn.h"\nint main(void) { return (int)sizeof(hgnn_layer_params) == 0; }\n')
    r = subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", os.path.join(ROOT, "include"),
                        "-fsyntax-only", str(src)], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
