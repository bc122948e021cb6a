"""GPU parity: the C-ABI path against the CPU oracle, element by element, on seeded inputs."""
import numpy as np
import pytest

from tests.parity import run_case

pytestmark = pytest.mark.gpu


def _assert_ok(rep):
    bad = {k: v for k, v in rep.items() if v == "MISMATCH"}
    assert rep["ok"], {"bad": bad, "report": {k: v for k, v in rep.items() if isinstance(v, tuple)}}


def test_config0_tiny_rgcn_fp32():
    _assert_ok(run_case(0, verbose=True, check_naive=True))


def test_builds_with_the_permutations():
    """The runner's default leaves perm / cperm out of the index build (the mean layers never read them); here
    they are asked for and compared bit for bit like the other index arrays."""
    rep = run_case(0, verbose=True, build_permutation=True)
    _assert_ok(rep)
    assert rep["L0.perm"] == "exact" and rep["L0.cperm"] == "exact"
    rep = run_case(2, scale=0.05, batch=512, verbose=True, build_permutation=True, sampled=dict(seed=11))
    _assert_ok(rep)
    assert rep["L0.perm"] == "exact" and rep["L1.cperm"] == "exact"


def test_config0_per_edge_type_input():
    _assert_ok(run_case(0, verbose=True, use_edge_id=False))


def test_config1_fp32_scaled():
    _assert_ok(run_case(1, scale=0.05, batch=256, verbose=True, check_naive=True))


def test_config2_bf16_scaled():
    _assert_ok(run_case(2, scale=0.05, batch=512, verbose=True, check_naive=True))


def test_config2_bf16_scaled_without_input_grads_of_fixed_features():
    # T0 carries fixed features, T1-T3 learnable embeddings: only those need input gradients in layer 1
    _assert_ok(run_case(2, scale=0.05, batch=512, verbose=True, input_grad=[0, 1, 1, 1]))


def test_first_layer_without_input_gradient_buffer():
    """Without an input-gradient buffer the first layer's backward runs the weight-gradient GEMM alone and adds
    the partial bias sums up in a launch of their own (fp32; bf16 with an output width that is no multiple of eight)."""
    _assert_ok(run_case(1, scale=0.05, batch=256, verbose=True, need_input_grad=False))
    _assert_ok(run_case(2, scale=0.05, batch=256, verbose=True, need_input_grad=False))


def test_first_layer_gathers_from_the_feature_stores():
    """hgnn_layer_fwd_gather / hgnn_layer_bwd_gather: the aggregation reads source rows through per-edge addresses into
    the per-type stores and only the destination rows are merged; same checks against the oracle, same bits as the
    fully merged path.  fp32 (config 1), bf16 with remainder planes (config 2), sampled in the loop (device ids)."""
    _assert_ok(run_case(1, scale=0.05, batch=256, verbose=True, check_gather=True, check_naive=True))
    _assert_ok(run_case(2, scale=0.05, batch=512, verbose=True, check_gather=True))
    _assert_ok(run_case(2, scale=0.05, batch=512, verbose=True, check_gather=True, sampled=dict(seed=5)))


def test_two_step_aggregation_of_algorithm_1():
    """The materialising form of Algorithm 1 (gather into FeatureCat, then reduce by destination) gives the
    oracle's outputs and the fused kernel's bits: fp32 (config 1), bf16 (config 2), many relations (config 5)."""
    _assert_ok(run_case(1, scale=0.05, batch=256, verbose=True, backward=False, check_two_step=True))
    _assert_ok(run_case(2, scale=0.05, batch=512, verbose=True, backward=False, check_two_step=True))
    _assert_ok(run_case(5, verbose=True, backward=False, check_two_step=True))


def test_two_step_aggregation_rejects_ragged_widths():
    from paper_2408_08490_amd.binding import HgnnError
    with pytest.raises(HgnnError, match="one input width"):
        run_case(0, backward=False, check_two_step=True)


def test_config3_many_types_fp32_scaled():
    _assert_ok(run_case(3, scale=0.02, batch=128, verbose=True, check_naive=True))


def test_config5_relation_heavy_small_fp32():
    """104 relations over 7 vertex types on a graph of a few thousand vertices: more relations than the forward
    GEMM examines in one pass, most of them with a handful of edges or none."""
    _assert_ok(run_case(5, verbose=True, check_naive=True))


def test_config6_relation_heavy_large_bf16():
    """108 relations, ~1.9 M vertices, ~5.5 M edges, bf16."""
    _assert_ok(run_case(6, verbose=True))


def test_config2_sampled_in_the_loop():
    """The mini-batch is drawn by the library's own sampler (sample, select edge indices, upload: one host task)
    and by the sampler oracle; ids, index arrays, outputs and gradients are compared as everywhere else."""
    _assert_ok(run_case(2, scale=0.05, batch=256, verbose=True, input_grad=[0, 1, 1, 1], sampled=dict(seed=4242)))


def test_config5_sampled_in_the_loop_many_relations():
    _assert_ok(run_case(5, verbose=True, sampled=dict(seed=7, fanouts=[4, 3])))


def test_config2_full_size_headline_workload():
    """The workload bench.py times (full graph, 4096 targets, bf16, hidden 512, input gradients only for the
    learnable embeddings), compared element by element with the oracle."""
    rep = run_case(2, scale=1.0, verbose=True, input_grad=[0, 1, 1, 1])
    _assert_ok(rep)
    assert rep["sizes"][0][2] > 900_000 and rep["sizes"][1][1] == 4096


def test_config1_full_size_fp32():
    """Config 1 as stated: the full academic-graph-shaped graph, 1024 targets, fanout [25, 20], fp32, hidden 256."""
    rep = run_case(1, scale=1.0, verbose=True, check_naive=True)
    _assert_ok(rep)
    assert rep["sizes"][1][1] == 1024 and rep["sizes"][0][2] > 200_000


def test_config3_full_size_many_types_fp32():
    """Config 3 as stated: 10 vertex types of ragged widths, 30 relations of ~2M edges, 512 targets, fanout [10, 10]."""
    rep = run_case(3, scale=1.0, verbose=True)
    _assert_ok(rep)
    assert rep["sizes"][1][1] == 512 and rep["sizes"][0][2] > 300_000


def test_forward_gemm_on_the_lds_dma_core(monkeypatch):
    """The alternative bf16 forward GEMM (operand tiles loaded straight into LDS, persistent blocks), which a context
    uses when HGNN_DMA_GEMM is set: 128-row tiles (scaled config 2, ragged widths with partial K-steps, 108
    relations) and 256-row tiles (the headline size)."""
    monkeypatch.setenv("HGNN_DMA_GEMM", "1")
    _assert_ok(run_case(2, scale=0.05, batch=512, verbose=True))
    _assert_ok(run_case(3, scale=0.02, batch=128, verbose=True, cfg_edit=_as_bf16))
    _assert_ok(run_case(6, verbose=True))
    _assert_ok(run_case(2, scale=1.0, verbose=True, input_grad=[0, 1, 1, 1], backward=False))


def _as_f32(cfg, g, mb, ws):
    cfg.dtype = "f32"


def _as_bf16(cfg, g, mb, ws):
    """Hook for run_case: the same inputs in bf16 storage (every value rounded first, so both sides start equal)."""
    from workloads import bf16_round
    cfg.dtype = "bf16"
    g.stores = [bf16_round(s) for s in g.stores]
    for lw in ws:
        lw.w_rel = [bf16_round(w) for w in lw.w_rel]
        lw.w_root = [None if w is None else bf16_round(w) for w in lw.w_root]
        lw.bias = [None if b is None else bf16_round(b) for b in lw.bias]
    if mb.grad_out is not None:
        mb.grad_out = [bf16_round(x) for x in mb.grad_out]


def test_ragged_widths_in_bf16():
    """Configs 3 and 7 (10 / 32 vertex types with different feature widths, 30 / 128 relations) in bf16 storage: the
    ragged-width gather kernels and the GEMM tables with 16-bit elements."""
    _assert_ok(run_case(3, scale=0.02, batch=128, verbose=True, cfg_edit=_as_bf16))
    _assert_ok(run_case(7, verbose=True, cfg_edit=_as_bf16))


def test_config4_attention_fp32_scaled():
    """Attention variant (3 layers, 8 heads, semantic-attention fusion) at config 4's shape on a reduced graph, in
    fp32 storage: every output and every gradient (per-type projections, attention vectors, semantic-attention
    MLP, biases, features) within 1e-4 of the oracle."""
    r = run_case(4, scale=0.02, batch=64, verbose=True, cfg_edit=_as_f32)
    assert r["ok"], r


def test_config4_attention_bf16_scaled():
    """The same in bf16 storage: features, parameters, layer outputs and the gradients handed from layer to layer
    are bf16, the layer's own arithmetic is fp32.  Every layer is run on the inputs the oracle's layer gets (the
    oracle's previous output and next input gradient, rounded to bf16 as the boundary stores them), so each is held
    to 2e-2 in every output and gradient, the attention vectors' included, on its own."""
    r = run_case(4, scale=0.02, batch=64, verbose=True, layerwise=True)
    assert r["ok"], r


def test_config4_attention_fp32_layer_by_layer():
    """fp32 storage through the layer-by-layer comparison as well (shared inputs at every layer boundary)."""
    r = run_case(4, scale=0.02, batch=64, verbose=True, cfg_edit=_as_f32, layerwise=True)
    assert r["ok"], r


def test_config4_attention_full_size_bf16():
    """configs[4] at its full size (3 layers, 8 heads, all 2048 targets: ~607k source rows and ~1.8M edges in the first
    layer), bf16 storage, layer by layer on shared inputs; the oracle takes about two minutes."""
    r = run_case(4, verbose=True, layerwise=True)
    assert r["ok"], r
    assert r["sizes"][-1][1] == 2048 and r["sizes"][0][2] > 1_500_000, r["sizes"]


def _drop_edges(keep):
    """Hook for run_case: keeps only the edges of the first block for which keep(edge_type) is true."""
    def edit(cfg, g, mb, ws):
        b = mb.blocks[0]
        m = np.array([bool(keep(int(t))) for t in b.edge_type], dtype=bool)
        b.edge_index = np.ascontiguousarray(b.edge_index[:, m])
        b.edge_id, b.edge_type = b.edge_id[m], b.edge_type[m]
    return edit


def test_relation_without_edges_and_block_without_edges():
    """Degenerate inputs: a relation that loses all its edges (its aggregate rows are zero, its weight gradient
    exactly zero), and a block with no edge at all (only the root term and the bias remain)."""
    r = run_case(0, verbose=True, cfg_edit=_drop_edges(lambda t: t != 0))
    assert r["ok"], r
    r = run_case(0, verbose=True, cfg_edit=_drop_edges(lambda t: False))
    assert r["ok"], r
    r = run_case(4, scale=0.02, batch=16, verbose=True, cfg_edit=lambda c, g, mb, ws: (_as_f32(c, g, mb, ws),
                                                                                       _drop_edges(lambda t: t != 1)(c, g, mb, ws)))
    assert r["ok"], r


def test_config7_widest_schema():
    """32 vertex types and 128 relations (the library's limits), ragged widths, two passes of the forward GEMM's
    relation window, most relations with a handful of edges."""
    _assert_ok(run_case(7, verbose=True, check_naive=True))
    _assert_ok(run_case(7, verbose=True, sampled=dict(seed=5)))


def test_empty_minibatch():
    """No target at all: every launch is skipped or empty, the outputs are empty, and the weight gradients -- sums
    over nothing -- are exactly zero."""
    import torch
    from paper_2408_08490_amd.runner import Model
    from workloads import build_graph, init_weights, make_config
    from workloads.synth import Block, MiniBatch
    cfg = make_config(0)
    g = build_graph(cfg)
    ws = init_weights(cfg, g)
    T = g.schema.num_types
    blk = Block([0] * T, [0] * T, np.zeros((2, 0), np.int64), np.zeros(0, np.int64), np.zeros(0, np.int32))
    mb = MiniBatch(ids=[np.zeros(0, np.int64) for _ in range(T)], blocks=[blk], target_type=1,
                   grad_out=[np.zeros((0, cfg.layer_out[-1]), np.float32) for _ in range(T)])
    model = Model(g.schema, g.feat_dim, g.stores, ws, dtype="f32", loss="dot", target_type=1)
    for w in model.weights:                              # the backward overwrites them: make that visible
        for t in w["dw_rel"] + [x for x in w["dw_root"] if x is not None]:
            t.fill_(7.0)
    bt = model.prepare(mb, g.edge_type, use_edge_id=True)
    view = bt.graph.host_view(0)
    assert view["rows"] == 0 and view["edges"] == 0 and np.array_equal(view["rowptr"], [0])
    out = model.run(bt)
    torch.cuda.synchronize()
    assert out["h"][0].numel() == 0 and out["dx"][0].numel() == 0
    for w in model.weights:
        for t in w["dw_rel"] + [x for x in w["dw_root"] if x is not None]:
            assert float(t.abs().max()) == 0.0
    model.close()


def test_single_target_minibatch():
    """One target vertex: every tile and lane group is ragged."""
    r = run_case(1, scale=0.05, batch=1, verbose=True)
    assert r["ok"], r
    r = run_case(2, scale=0.05, batch=1, verbose=True)
    assert r["ok"], r


def test_index_first_baseline_round_trip():
    """The index-first baseline of the feature stage (hgnn_merge_features_index_first + hgnn_select_type_first): rows of
    all types interleaved in one buffer, then selected back per type, give hgnn_merge_features' x_merged and offsets
    bit for bit; the interleaved buffer holds every row at its stated position."""
    import torch
    import paper_2408_08490_amd.binding as B
    from paper_2408_08490_amd.runner import to_device
    from workloads import make_config, build_graph, sample_minibatch, bf16_round
    for dtype in ("f32", "bf16"):
        cfg = make_config(2, scale=0.02, batch=256)
        g = build_graph(cfg)
        mb = sample_minibatch(cfg, g)
        sch = g.schema
        T = sch.num_types
        dev = torch.device("cuda", 0)
        ctx = B.Context(sch.rel_src, sch.rel_dst, T, dtype, device=0, host_threads=1)
        stores_np = [bf16_round(s) if dtype == "bf16" else np.asarray(s, np.float32) for s in g.stores]
        stores = [to_device(s, dtype, dev) for s in stores_np]
        ids = [torch.from_numpy(np.ascontiguousarray(i, dtype=np.int64)).to(dev) for i in mb.ids]
        n = [len(i) for i in mb.ids]
        total, F = sum(n), g.feat_dim[0]
        # proportional interleaving of the types (a permutation of 0 .. total - 1)
        key = np.concatenate([(np.arange(k) + 0.5) / max(k, 1) for k in n])
        order = np.argsort(key, kind="stable")
        rank = np.empty(total, np.int64); rank[order] = np.arange(total)
        off = np.concatenate([[0], np.cumsum(n)])
        pos_np = [rank[off[t]: off[t + 1]].astype(np.int32) for t in range(T)]
        pos = [torch.from_numpy(p).to(dev) for p in pos_np]
        tdt = torch.float32 if dtype == "f32" else torch.bfloat16
        x_int = torch.empty(total * F, device=dev, dtype=tdt)
        x_sel = torch.empty(total * F, device=dev, dtype=tdt)
        x_ref = torch.empty(total * F, device=dev, dtype=tdt)
        ctx.hgnn_merge_features_index_first(stores, ids, pos, x_int, g.feat_dim)
        ro, eo = ctx.hgnn_select_type_first(x_int, pos, x_sel, g.feat_dim)
        ro2, eo2 = ctx.hgnn_merge_features(stores, ids, x_ref, g.feat_dim)
        torch.cuda.synchronize()
        assert np.array_equal(ro, ro2) and np.array_equal(eo, eo2)
        assert torch.equal(x_sel.view(torch.uint8), x_ref.view(torch.uint8))
        want = np.empty((total, F), np.float32)
        for t in range(T):
            want[pos_np[t]] = stores_np[t][mb.ids[t]]
        assert np.array_equal(x_int.float().cpu().numpy().reshape(total, F), want)
        # ragged widths are refused
        with pytest.raises(B.HgnnError):
            ctx.hgnn_merge_features_index_first(stores, ids, pos, x_int, [F] * (T - 1) + [F * 2])
        ctx.close()
