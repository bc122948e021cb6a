"""CPU checks of the parity harness itself (tests/parity.py): the rounding band inside which the GPU tests accept
either ReLU decision is computed from oracle quantities only, and is what its comment says it is."""
import types

import numpy as np

from oracle import hgnn_oracle as O
from tests import parity as PH


def _case(rng):
    x = [rng.standard_normal((6, 3)), rng.standard_normal((7, 4))]
    rel_src, rel_dst, n_dst = [0, 1, 1], [1, 1, 0], [3, 4]
    ei = np.array([[0, 1, 5, 2, 2, 6, 3, 0], [0, 0, 1, 3, 0, 2, 2, 1]])
    et = np.array([0, 0, 0, 1, 1, 1, 2, 2], dtype=np.int32)
    w_rel = [rng.standard_normal((3, 5)), rng.standard_normal((4, 5)), rng.standard_normal((4, 5))]
    w_root = [rng.standard_normal((3, 5)), rng.standard_normal((4, 5))]
    bias = [rng.standard_normal(5), None]
    sel = O.edge_index_select(ei, 3, edge_type=et)
    h, cache = O.rgcn_layer_forward(x, sel, rel_src, rel_dst, n_dst, w_rel, w_root, bias, True)
    return x, ei, et, rel_src, rel_dst, n_dst, w_rel, w_root, bias, sel, cache


def test_band_is_eps_times_the_sum_of_term_magnitudes():
    rng = np.random.default_rng(0)
    x, ei, et, rel_src, rel_dst, n_dst, w_rel, w_root, bias, sel, cache = _case(rng)
    # S by hand, dense: |b| + |x_v| |W0| + sum_r mean_u |x_u| . |W_r|
    S = [np.zeros((n_dst[t], 5)) for t in range(2)]
    for t in range(2):
        S[t] += np.abs(x[t][: n_dst[t]]) @ np.abs(w_root[t])
        if bias[t] is not None:
            S[t] += np.abs(bias[t])[None, :]
    for r in range(3):
        for v in range(n_dst[rel_dst[r]]):
            nb = [int(a) for a, b, ty in zip(ei[0], ei[1], et) if ty == r and b == v]
            if nb:
                S[rel_dst[r]][v] += np.abs(x[rel_src[r]][nb]).mean(axis=0) @ np.abs(w_rel[r])
    for dtype in ("f32", "bf16"):
        cfg = types.SimpleNamespace(dtype=dtype)
        for layer, eps in ((0, PH.EPS[dtype]), (1, PH.EPS_ACT[dtype])):
            band = PH.decision_band(cfg, cache, sel, layer)
            for t in range(2):
                assert np.array_equal(band[t], np.abs(cache["pre"][t]) <= eps * S[t])
                assert np.all(S[t] >= np.abs(cache["pre"][t]) - 1e-12)       # the triangle inequality it rests on


def test_band_is_empty_for_generic_inputs_and_holds_exact_zeros():
    rng = np.random.default_rng(1)
    *_, sel, cache = _case(rng)
    cfg = types.SimpleNamespace(dtype="bf16")
    band = PH.decision_band(cfg, cache, sel, 0)
    assert sum(int(b.sum()) for b in band) == 0          # |pre| ~ 1 against eps * S ~ 1e-4
    cache["pre"][1][2, 3] = 0.0
    band = PH.decision_band(cfg, cache, sel, 0)
    assert band[1][2, 3] and sum(int(b.sum()) for b in band) == 1
