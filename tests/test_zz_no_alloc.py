"""hgnn_layer_fwd_static (the forward entry point that allocates nothing: its work area is a fixed device array of
the library) against hgnn_layer_fwd on the same inputs: every output bit for bit, on two calls in a row, the second
on a smaller mini-batch (the fixed array still holds the first call's contents), and a third on a layer without
an activation.  A layer that needs more than the array holds is refused."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _forward_both(model, bt, torch):
    """Layer by layer: hgnn_layer_fwd into one set of buffers, hgnn_layer_fwd_static into another; returns the
    pairs (h, saved) of both."""
    ctx = model.ctx
    n0 = sum(n * f for n, f in zip(bt.n_rows, model.feat_dim))
    tdt = torch.bfloat16 if model.dtype == "bf16" else torch.float32
    x = torch.empty(n0, device=model.dev, dtype=tdt)
    ctx.hgnn_merge_features(model.stores, bt.ids_dev, x, model.feat_dim)
    res = []
    xin = x
    for l, lp in enumerate(model.layers):
        blk = bt.blocks[l]
        sb, cb = ctx.hgnn_layer_workspace_bytes(bt.graph, l, lp)
        nh = sum(blk.n_dst) * lp.out_dim
        outs = []
        for static in (False, True):
            h = torch.full((max(nh, 1),), 7.0, device=model.dev, dtype=tdt)[:nh]
            sv = torch.full((max(sb, 256),), 0x5A, device=model.dev, dtype=torch.uint8)
            if static:
                ctx.hgnn_layer_fwd_static(bt.graph, l, lp, xin, h, sv)
            else:
                sc = torch.full((max(cb, 256),), 0xA5, device=model.dev, dtype=torch.uint8)
                ctx.hgnn_layer_fwd(bt.graph, l, lp, xin, h, sv, sc)
            outs.append((h, sv[:sb]))
        torch.cuda.synchronize()
        res.append(outs)
        xin = outs[0][0]
    return res


def _same_bits(a, b, torch):
    return torch.equal(a.contiguous().view(torch.uint8), b.contiguous().view(torch.uint8))


def test_static_area_forward_matches_the_allocating_entry_point_on_two_calls_in_a_row():
    import torch
    from paper_2408_08490_amd.runner import Model
    from tests.parity import prepare_inputs
    cfg, g, mb, ws = prepare_inputs(2, scale=0.05, batch=512)          # bf16, ReLU layer: both planes in the area
    model = Model(g.schema, g.feat_dim, g.stores, ws, dtype=cfg.dtype, loss="xent", target_type=mb.target_type)
    bt = model.prepare(mb, g.edge_type, use_edge_id=True)
    first = _forward_both(model, bt, torch)
    for l, ((h_a, sv_a), (h_b, sv_b)) in enumerate(first):
        assert h_a.numel() > 0 and _same_bits(h_a, h_b, torch) and _same_bits(sv_a, sv_b, torch), l
    bt.graph.release()
    # second call, smaller input, same process: the area still holds what the first call left
    cfg2, _, mb2, _ = prepare_inputs(2, scale=0.05, batch=48, graph=g)
    bt2 = model.prepare(mb2, g.edge_type, use_edge_id=True)
    second = _forward_both(model, bt2, torch)
    for l, ((h_a, sv_a), (h_b, sv_b)) in enumerate(second):
        assert 0 < h_a.numel() < first[l][0][0].numel()
        assert _same_bits(h_a, h_b, torch) and _same_bits(sv_a, sv_b, torch), l
    bt2.graph.release()
    model.close()


def test_static_area_forward_in_fp32_with_ragged_widths():
    import torch
    from paper_2408_08490_amd.runner import Model
    from tests.parity import prepare_inputs
    cfg, g, mb, ws = prepare_inputs(0)
    model = Model(g.schema, g.feat_dim, g.stores, ws, dtype=cfg.dtype, loss="dot", target_type=mb.target_type)
    bt = model.prepare(mb, g.edge_type, use_edge_id=True)
    for l, ((h_a, sv_a), (h_b, sv_b)) in enumerate(_forward_both(model, bt, torch)):
        assert _same_bits(h_a, h_b, torch) and _same_bits(sv_a, sv_b, torch), l
    bt.graph.release()
    model.close()


def test_static_area_forward_refuses_a_layer_beyond_the_fixed_size():
    import torch
    from paper_2408_08490_amd import binding as B
    from paper_2408_08490_amd.runner import Model
    from tests.parity import prepare_inputs
    cfg, g, mb, ws = prepare_inputs(2, scale=1.0)                       # headline size: 38 MB fit ...
    model = Model(g.schema, g.feat_dim, g.stores, ws, dtype=cfg.dtype, loss="xent", target_type=mb.target_type)
    bt = model.prepare(mb, g.edge_type, use_edge_id=True)
    for l, ((h_a, sv_a), (h_b, sv_b)) in enumerate(_forward_both(model, bt, torch)):
        assert _same_bits(h_a, h_b, torch) and _same_bits(sv_a, sv_b, torch), l
    bt.graph.release()
    model.close()
    cfg, g, mb, ws = prepare_inputs(2, scale=1.0, batch=3 * 4096, graph=g)   # ... three times the targets do not
    model = Model(g.schema, g.feat_dim, g.stores, ws, dtype=cfg.dtype, loss="xent", target_type=mb.target_type)
    bt = model.prepare(mb, g.edge_type, use_edge_id=True)
    x = torch.empty(sum(n * f for n, f in zip(bt.n_rows, model.feat_dim)), device=model.dev, dtype=torch.bfloat16)
    model.ctx.hgnn_merge_features(model.stores, bt.ids_dev, x, model.feat_dim)
    lp, blk = model.layers[0], bt.blocks[0]
    sb, _ = model.ctx.hgnn_layer_workspace_bytes(bt.graph, 0, lp)
    h = torch.full((sum(blk.n_dst) * lp.out_dim,), 7.0, device=model.dev, dtype=torch.bfloat16)
    sv = torch.empty(sb, device=model.dev, dtype=torch.uint8)
    with pytest.raises(B.HgnnError, match="static one holds"):
        model.ctx.hgnn_layer_fwd_static(bt.graph, 0, lp, x, h, sv)
    torch.cuda.synchronize()
    assert float(h.float().min()) == 7.0 and float(h.float().max()) == 7.0      # nothing was enqueued
    bt.graph.release()
    model.close()
