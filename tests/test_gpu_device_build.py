"""The semantic-graph build done by device kernels (hgnn_build_semantic_csr_device): its index arrays against the
index oracle bit for bit, and whole models on its graphs."""
import numpy as np
import pytest

from tests.parity import run_case
from tests.test_gpu_parity import _assert_ok

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("index,scale,batch,use_edge_id", [(0, 1.0, None, True), (0, 1.0, None, False), (1, 0.05, 256, True),
                                                          (2, 0.05, 512, True), (5, 1.0, None, True), (3, 0.02, 128, False)])
def test_device_build_gives_the_host_builds_arrays_and_results(index, scale, batch, use_edge_id):
    """Every index array (merged CSR, transpose, both permutations) equals the oracle's; layers run on the graph."""
    rep = run_case(index, scale=scale, batch=batch, verbose=True, use_edge_id=use_edge_id, device_build=True,
                   build_permutation=True)
    _assert_ok(rep)
    assert rep["L0.perm"] == "exact" and rep["L0.cperm"] == "exact" and rep["L0.crow"] == "exact"


def test_device_build_with_restricted_transpose_and_long_rows():
    """Transpose entries only for the types that need input gradients (the others' rows stay empty), and a graph whose
    transpose has rows long enough for the chunk lists (config 2 at a size where hubs collect hundreds of edges)."""
    _assert_ok(run_case(2, scale=0.05, batch=512, verbose=True, input_grad=[0, 1, 1, 1], device_build=True))
    _assert_ok(run_case(2, scale=0.2, batch=2048, verbose=True, device_build=True))


def test_device_build_attention_variant_keeps_cperm_on_the_device():
    r = run_case(4, scale=0.02, batch=64, verbose=True, device_build=True, layerwise=True)
    assert r["ok"], r


def test_device_build_reports_bad_edges():
    import paper_2408_08490_amd.binding as B
    from workloads import make_config, build_graph, sample_minibatch
    cfg = make_config(0)
    g = build_graph(cfg)
    mb = sample_minibatch(cfg, g)
    sch = g.schema
    ctx = B.Context(sch.rel_src, sch.rel_dst, sch.num_types, "f32", device=0, host_threads=2)

    class Blk:
        pass

    def bad(**kw):
        b, src = Blk(), mb.blocks[0]
        b.n_src, b.n_dst = list(src.n_src), list(src.n_dst)
        b.edge_index, b.edge_type = src.edge_index.copy(), src.edge_type.copy()
        for k, v in kw.items():
            setattr(b, k, v)
        return b

    et = mb.blocks[0].edge_type.copy(); et[5] = 7
    with pytest.raises(B.HgnnError) as e:
        ctx.hgnn_build_semantic_csr_device([bad(edge_type=et)])
    assert e.value.status == -1 and "type" in str(e.value)
    ei = mb.blocks[0].edge_index.copy(); ei[0, 3] = 10 ** 6
    with pytest.raises(B.HgnnError) as e:
        ctx.hgnn_build_semantic_csr_device([bad(edge_index=ei)])
    assert "source" in str(e.value)
    ei = mb.blocks[0].edge_index.copy(); ei[1, 0] = -1
    with pytest.raises(B.HgnnError) as e:
        ctx.hgnn_build_semantic_csr_device([bad(edge_index=ei)])
    assert "destination" in str(e.value)
    gr = ctx.hgnn_build_semantic_csr_device(mb.blocks)      # a good build still works afterwards
    assert gr.build_gpu_ms > 0
    v = gr.host_view(0)
    assert v["rowptr"][-1] == mb.blocks[0].edge_index.shape[1]
    gr.release()
    ctx.close()


def test_device_build_degenerate_and_int32_inputs():
    """A block without any edge, a relation that lost its edges, a single target, int32 COO indices with per-edge types."""
    from tests.test_gpu_parity import _drop_edges

    def as_i32(cfg, g, mb, ws):
        for b in mb.blocks:
            b.edge_index = b.edge_index.astype(np.int32)
    _assert_ok(run_case(0, verbose=True, device_build=True, cfg_edit=_drop_edges(lambda t: False)))
    _assert_ok(run_case(0, verbose=True, device_build=True, cfg_edit=_drop_edges(lambda t: t != 1), check_naive=True))
    _assert_ok(run_case(2, scale=0.02, batch=1, verbose=True, device_build=True, check_gather=True))
    _assert_ok(run_case(2, scale=0.05, batch=512, verbose=True, device_build=True, cfg_edit=as_i32, use_edge_id=False))
