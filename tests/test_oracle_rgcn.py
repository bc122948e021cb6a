"""Pins for the CPU oracle's R-GCN layer: each test fixes it to something other
than itself (hand arithmetic, dense linear algebra, scipy.sparse, invariants,
finite differences)."""
import json
import os

import numpy as np
import pytest
import scipy.sparse as sp

from oracle import hgnn_oracle as O

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _random_case(rng, n_nodes=(6, 8), feat=(3, 5), H=4, rels=((0, 1), (1, 0), (1, 1), (0, 1)),
                 n_dst=(4, 5), n_edges=14, bias=True, dup=False):
    T, R = len(n_nodes), len(rels)
    x = [rng.standard_normal((n_nodes[t], feat[t])) for t in range(T)]
    rel_src = [s for s, _ in rels]
    rel_dst = [d for _, d in rels]
    src, dst, et = [], [], []
    for r, (s, d) in enumerate(rels):
        ne = n_edges
        pairs = set()
        while len(pairs) < ne and len(pairs) < n_nodes[s] * n_dst[d]:
            pairs.add((int(rng.integers(n_nodes[s])), int(rng.integers(n_dst[d]))))
        for (a, b) in sorted(pairs):
            src.append(a); dst.append(b); et.append(r)
        if dup and pairs:
            a, b = sorted(pairs)[0]
            src.append(a); dst.append(b); et.append(r)
    p = rng.permutation(len(src))
    ei = np.array([src, dst])[:, p]
    et = np.array(et, dtype=np.int32)[p]
    w_rel = [rng.standard_normal((feat[rel_src[r]], H)) for r in range(R)]
    w_root = [rng.standard_normal((feat[t], H)) for t in range(T)]
    b = [rng.standard_normal(H) if bias else None for t in range(T)]
    return dict(x=x, ei=ei, et=et, rel_src=rel_src, rel_dst=rel_dst, n_dst=list(n_dst),
                n_src=list(n_nodes), w_rel=w_rel, w_root=w_root, bias=b, H=H, feat=list(feat))


def _fwd(c, relu=False, x=None, w_rel=None, w_root=None, bias=None):
    sel = O.edge_index_select(c["ei"], len(c["rel_src"]), edge_type=c["et"])
    return O.rgcn_layer_forward(c["x"] if x is None else x, sel, c["rel_src"], c["rel_dst"], c["n_dst"],
                                c["w_rel"] if w_rel is None else w_rel,
                                c["w_root"] if w_root is None else w_root,
                                c["bias"] if bias is None else bias, relu)


def test_hand_worked_example():
    g = json.load(open(os.path.join(GOLD, "hand_example.json")))
    x = [np.array(g["x_A"])[:, None], np.array(g["x_B"])[:, None]]
    ei = np.array([g["edges_src"], g["edges_dst"]])
    sel = O.edge_index_select(ei, 2, edge_type=np.array(g["edges_type"]))
    rel_src, rel_dst, n_dst = [0, 1], [1, 1], [0, 2]
    w_rel = [np.array([[g["W_r0"]]]), np.array([[g["W_r1"]]])]
    w_root = [np.array([[g["W_0"]]]), np.array([[g["W_0"]]])]
    h, cache = O.rgcn_layer_forward(x, sel, rel_src, rel_dst, n_dst, w_rel, w_root, [None, None], False)
    assert h[0].shape == (0, 1)
    np.testing.assert_allclose(h[1][:, 0], g["h_B"], rtol=0, atol=1e-15)
    dx, dw_rel, dw_root, db = O.rgcn_layer_backward(cache, [np.zeros((0, 1)), np.ones((2, 1))])
    assert dw_root[1][0, 0] == g["dW_0"] and dw_root[0][0, 0] == 0.0
    assert dw_rel[0][0, 0] == g["dW_r0"] and dw_rel[1][0, 0] == g["dW_r1"]
    np.testing.assert_allclose(dx[0][:, 0], g["dx_A"], atol=1e-15)
    np.testing.assert_allclose(dx[1][:, 0], g["dx_B"], atol=1e-15)
    csr = O.semantic_csr(sel, rel_src, rel_dst, [2, 2], n_dst)
    for k in ("row_off", "rel_row_off", "rowptr", "colidx", "cptr", "crow"):
        assert csr[k].tolist() == g[k], k


@pytest.mark.parametrize("seed", [0, 1, 2])
@pytest.mark.parametrize("relu", [False, True])
def test_dense_adjacency_brute_force(seed, relu):
    """h = act(X_d W_0 + b + sum_r D_r^-1 A_r X_s W_r) with dense 0/1 (count) matrices."""
    rng = np.random.default_rng(seed)
    c = _random_case(rng, dup=(seed == 2))
    h, _ = _fwd(c, relu)
    T, R = 2, len(c["rel_src"])
    ref = [c["x"][t][: c["n_dst"][t]] @ c["w_root"][t] + c["bias"][t] for t in range(T)]
    for r in range(R):
        s, d = c["rel_src"][r], c["rel_dst"][r]
        A = np.zeros((c["n_dst"][d], c["n_src"][s]))
        m = c["et"] == r
        for a, b in zip(c["ei"][0][m], c["ei"][1][m]):
            A[b, a] += 1.0
        deg = A.sum(1)
        Dinv = np.diag(np.where(deg > 0, 1.0 / np.maximum(deg, 1), 0.0))
        ref[d] = ref[d] + Dinv @ A @ c["x"][s] @ c["w_rel"][r]
    for t in range(T):
        np.testing.assert_allclose(h[t], np.maximum(ref[t], 0) if relu else ref[t], rtol=1e-12, atol=1e-12)


def test_single_relation_equals_scipy_row_normalised_spmm():
    rng = np.random.default_rng(5)
    n_src, n_dst, F, H, E = 40, 17, 6, 5, 90
    src = rng.integers(0, n_src, E); dst = rng.integers(0, n_dst, E)
    x = [rng.standard_normal((n_src, F))]
    w = rng.standard_normal((F, H))
    sel = O.edge_index_select(np.array([src, dst]), 1, edge_type=np.zeros(E, np.int32))
    h, _ = O.rgcn_layer_forward(x, sel, [0], [0], [n_dst], [w], [None], [None], False)
    A = sp.coo_matrix((np.ones(E), (dst, src)), shape=(n_dst, n_src)).tocsr()   # duplicates add up
    deg = np.asarray(A.sum(1)).ravel()
    Dinv = sp.diags(np.where(deg > 0, 1.0 / np.maximum(deg, 1), 0.0))
    ref = (Dinv @ A) @ x[0] @ w
    np.testing.assert_allclose(h[0], ref, rtol=1e-12, atol=1e-12)


def test_merged_equals_unmerged():
    rng = np.random.default_rng(7)
    c = _random_case(rng, n_nodes=(9, 11), n_dst=(5, 7), n_edges=25)
    sel = O.edge_index_select(c["ei"], len(c["rel_src"]), edge_type=c["et"])
    csr = O.semantic_csr(sel, c["rel_src"], c["rel_dst"], c["n_src"], c["n_dst"])
    flat = np.concatenate([a.ravel() for a in c["x"]])
    h, _ = _fwd(c, True)
    hm = O.rgcn_layer_forward_merged(flat, c["feat"], csr, c["rel_src"], c["rel_dst"], c["n_dst"],
                                     c["w_rel"], c["w_root"], c["bias"], True)
    for a, b in zip(h, hm):
        np.testing.assert_allclose(a, b, rtol=1e-14, atol=1e-14)


def test_mean_of_constant_features_is_the_constant():
    rng = np.random.default_rng(3)
    F = 4
    c = _random_case(rng, feat=(F, F), H=F, rels=((0, 1), (1, 1)), n_edges=4, bias=False)
    cval = 2.5
    x = [np.full_like(a, cval) for a in c["x"]]
    eye = [np.eye(F), np.zeros((F, F))]            # only relation 0 contributes
    h, cache = _fwd(c, False, x=x, w_rel=eye, w_root=[None, None], bias=[None, None])
    deg = np.bincount(c["ei"][1][c["et"] == 0], minlength=c["n_dst"][1])
    assert (deg == 0).any() and (deg > 0).any()
    assert np.all(h[1][deg > 0] == cval)
    assert np.all(h[1][deg == 0] == 0.0)
    assert h[0].shape == (c["n_dst"][0], F) and np.all(h[0] == 0.0)


def test_vertex_permutation_and_edge_order_invariance():
    rng = np.random.default_rng(11)
    c = _random_case(rng, n_nodes=(7, 9), n_dst=(4, 6), n_edges=20)
    h, cache = _fwd(c, True)
    g = [rng.standard_normal(a.shape) for a in h]
    dx, dwr, dw0, db = O.rgcn_layer_backward(cache, g)
    # permute vertices inside each type keeping destinations a prefix; shuffle edges
    perms, inv = [], []
    for t in range(2):
        pd = rng.permutation(c["n_dst"][t])
        pr = c["n_dst"][t] + rng.permutation(c["n_src"][t] - c["n_dst"][t])
        p = np.concatenate([pd, pr])                 # new row i holds old row p[i]
        perms.append(p); q = np.empty_like(p); q[p] = np.arange(len(p)); inv.append(q)
    x2 = [c["x"][t][perms[t]] for t in range(2)]
    ei2 = c["ei"].copy()
    for k in range(ei2.shape[1]):
        r = c["et"][k]
        ei2[0, k] = inv[c["rel_src"][r]][c["ei"][0, k]]
        ei2[1, k] = inv[c["rel_dst"][r]][c["ei"][1, k]]
    sh = rng.permutation(ei2.shape[1])
    c2 = dict(c, x=x2, ei=ei2[:, sh], et=c["et"][sh])
    h2, cache2 = _fwd(c2, True)
    g2 = [g[t][perms[t][: c["n_dst"][t]]] for t in range(2)]
    dx2, dwr2, dw02, db2 = O.rgcn_layer_backward(cache2, g2)
    for t in range(2):
        np.testing.assert_allclose(h2[t], h[t][perms[t][: c["n_dst"][t]]], rtol=1e-12, atol=1e-12)
        np.testing.assert_allclose(dx2[t], dx[t][perms[t]], rtol=1e-12, atol=1e-12)
        np.testing.assert_allclose(dw02[t], dw0[t], rtol=1e-11, atol=1e-12)
        np.testing.assert_allclose(db2[t], db[t], rtol=1e-11, atol=1e-12)
    for r in range(len(dwr)):
        np.testing.assert_allclose(dwr2[r], dwr[r], rtol=1e-11, atol=1e-12)


def test_projection_and_aggregation_commute():
    """mean_u(x_u W) == (mean_u x_u) W: aggregate-then-project gives the same layer."""
    rng = np.random.default_rng(13)
    c = _random_case(rng)
    h, _ = _fwd(c, False)
    T = 2
    ref = [c["x"][t][: c["n_dst"][t]] @ c["w_root"][t] + c["bias"][t] for t in range(T)]
    for r in range(len(c["rel_src"])):
        s, d = c["rel_src"][r], c["rel_dst"][r]
        m = c["et"] == r
        z = np.zeros((c["n_dst"][d], c["feat"][s])); cnt = np.zeros(c["n_dst"][d])
        for a, b in zip(c["ei"][0][m], c["ei"][1][m]):
            z[b] += c["x"][s][a]; cnt[b] += 1
        z[cnt > 0] /= cnt[cnt > 0][:, None]
        ref[d] += z @ c["w_rel"][r]
    for t in range(T):
        np.testing.assert_allclose(h[t], ref[t], rtol=1e-12, atol=1e-12)


def _loss(c, G, relu, **kw):
    h, _ = _fwd(c, relu, **kw)
    return sum(float((G[t] * h[t]).sum()) for t in range(len(h)))


@pytest.mark.parametrize("relu", [False, True])
def test_finite_difference_gradients(relu):
    rng = np.random.default_rng(17)
    c = _random_case(rng, dup=True)
    h, cache = _fwd(c, relu)
    G = [rng.standard_normal(a.shape) for a in h]
    dx, dwr, dw0, db = O.rgcn_layer_backward(cache, G)
    eps = 1e-6

    def fd(arr_list, idx, key):
        out = np.zeros_like(arr_list[idx])
        it = np.nditer(arr_list[idx], flags=["multi_index"])
        for _ in it:
            i = it.multi_index
            saved = arr_list[idx][i]
            arr_list[idx][i] = saved + eps; lp = _loss(c, G, relu, **{key: arr_list})
            arr_list[idx][i] = saved - eps; lm = _loss(c, G, relu, **{key: arr_list})
            arr_list[idx][i] = saved
            out[i] = (lp - lm) / (2 * eps)
        return out

    for r in range(len(dwr)):
        np.testing.assert_allclose(dwr[r], fd([w.copy() for w in c["w_rel"]], r, "w_rel"), rtol=1e-6, atol=1e-7)
    for t in range(2):
        np.testing.assert_allclose(dw0[t], fd([w.copy() for w in c["w_root"]], t, "w_root"), rtol=1e-6, atol=1e-7)
        np.testing.assert_allclose(db[t], fd([w.copy() for w in c["bias"]], t, "bias"), rtol=1e-6, atol=1e-7)
        np.testing.assert_allclose(dx[t], fd([w.copy() for w in c["x"]], t, "x"), rtol=1e-6, atol=1e-7)


def test_unused_relation_gets_zero_gradient():
    rng = np.random.default_rng(19)
    c = _random_case(rng, n_dst=(0, 5))        # relation (1,0) has no destination rows
    keep = c["et"] != 1
    c["ei"], c["et"] = c["ei"][:, keep], c["et"][keep]
    h, cache = _fwd(c, False)
    dx, dwr, dw0, db = O.rgcn_layer_backward(cache, [np.ones_like(a) for a in h])
    assert np.all(dwr[1] == 0.0) and dwr[1].shape == c["w_rel"][1].shape
    assert np.all(dw0[0] == 0.0)


def test_softmax_xent_closed_forms_and_fd():
    n, C = 5, 7
    loss, g = O.softmax_xent(np.zeros((n, C)), np.arange(n) % C)
    assert abs(loss - np.log(C)) < 1e-15
    np.testing.assert_allclose(g.sum(1), 0, atol=1e-16)
    assert abs(g[0, 0] - (1.0 / C - 1.0) / n) < 1e-16
    rng = np.random.default_rng(0)
    z = rng.standard_normal((n, C)) * 3; lab = rng.integers(0, C, n)
    loss, g = O.softmax_xent(z, lab)
    ref = np.mean([-np.log(np.exp(z[i, lab[i]]) / np.exp(z[i]).sum()) for i in range(n)])
    assert abs(loss - ref) < 1e-12
    eps = 1e-6
    for i, j in [(0, 0), (2, 3), (4, 6)]:
        zp = z.copy(); zp[i, j] += eps; zm = z.copy(); zm[i, j] -= eps
        fd = (O.softmax_xent(zp, lab)[0] - O.softmax_xent(zm, lab)[0]) / (2 * eps)
        assert abs(fd - g[i, j]) < 1e-8
    # large logits do not overflow
    loss, g = O.softmax_xent(np.array([[1000.0, 0.0]]), np.array([0]))
    assert np.isfinite(loss) and abs(loss) < 1e-12


def test_two_layer_model_gradients_by_finite_differences():
    rng = np.random.default_rng(23)
    T, rel_src, rel_dst = 2, [0, 1, 1], [1, 0, 1]
    n = [[10, 12], [5, 6], [0, 3]]                 # rows per type: layer-1 src, layer-1 dst, layer-2 dst
    feat, H1, C = [3, 4], 5, 4

    def edges(ns, nd, k):
        src, dst, et = [], [], []
        for r in range(3):
            s, d = rel_src[r], rel_dst[r]
            if nd[d] == 0 or ns[s] == 0:
                continue
            for _ in range(k):
                src.append(int(rng.integers(ns[s]))); dst.append(int(rng.integers(nd[d]))); et.append(r)
        return np.array([src, dst]), np.array(et, np.int32)
    e1, t1 = edges(n[0], n[1], 12)
    e2, t2 = edges(n[1], n[2], 6)
    sel = [O.edge_index_select(e1, 3, edge_type=t1), O.edge_index_select(e2, 3, edge_type=t2)]
    x0 = [rng.standard_normal((n[0][t], feat[t])) for t in range(T)]
    L1 = dict(w_rel=[rng.standard_normal((feat[rel_src[r]], H1)) for r in range(3)],
              w_root=[rng.standard_normal((feat[t], H1)) for t in range(T)],
              bias=[rng.standard_normal(H1) for t in range(T)], relu=True)
    L2 = dict(w_rel=[rng.standard_normal((H1, C)) for r in range(3)],
              w_root=[rng.standard_normal((H1, C)) for t in range(T)],
              bias=[rng.standard_normal(C) for t in range(T)], relu=False)
    labels = rng.integers(0, C, n[2][1])

    def run():
        return O.rgcn_model_forward_backward(x0, sel, rel_src, rel_dst, [n[1], n[2]], [L1, L2], "xent",
                                             labels=labels, target_type=1)
    out = run()
    eps = 1e-6
    for (arr, grad) in [(L1["w_rel"][0], out["grads"][0]["dw_rel"][0]), (L1["w_root"][1], out["grads"][0]["dw_root"][1]),
                        (L2["w_rel"][2], out["grads"][1]["dw_rel"][2]), (L1["bias"][0], out["grads"][0]["dbias"][0]),
                        (x0[0], out["dx0"][0]), (x0[1], out["dx0"][1])]:
        for _ in range(6):
            i = tuple(int(rng.integers(s)) for s in arr.shape)
            sv = arr[i]
            arr[i] = sv + eps; lp = run()["loss"]
            arr[i] = sv - eps; lm = run()["loss"]
            arr[i] = sv
            assert abs((lp - lm) / (2 * eps) - grad[i]) < 1e-7 * max(1.0, abs(grad[i]))


# --------------------------------------------------------------------------- #
# The `relu_mask` branch of the backward (parity tests hand it the decisions of units whose
# pre-activation is zero to within rounding)
# --------------------------------------------------------------------------- #
def test_relu_mask_equal_to_own_decisions_reproduces_the_plain_backward_bit_for_bit():
    rng = np.random.default_rng(11)
    c = _random_case(rng)
    h, cache = _fwd(c, relu=True)
    G = [rng.standard_normal(a.shape) for a in h]
    plain = O.rgcn_layer_backward(cache, G)
    masked = O.rgcn_layer_backward(cache, G, relu_mask=[p > 0 for p in cache["pre"]])
    for a, b in zip(plain, masked):
        for u, v in zip(a, b):
            assert (u is None and v is None) or np.array_equal(u, v)


@pytest.mark.parametrize("seed", [0, 1])
def test_flipping_one_relu_decision_moves_exactly_that_unit_s_terms(seed):
    """Switching unit (t, v, c) off removes g[v, c] from the bias gradient's element c, x_v g[v, c] from column c of
    the root weight gradient, mean_u(x_u) g[v, c] from column c of every relation ending in t, g[v, c] W[:, c] from
    the feature gradients of v and (divided by the neighbourhood size) of its neighbours -- and nothing else.  The
    expected changes are written out here from the layer's definition, not taken from the oracle."""
    rng = np.random.default_rng(100 + seed)
    c = _random_case(rng)
    h, cache = _fwd(c, relu=True)
    G = [rng.standard_normal(a.shape) for a in h]
    t = 1
    act = np.argwhere(cache["pre"][t] > 0)
    v, col = (int(a) for a in act[rng.integers(len(act))])
    mask = [p > 0 for p in cache["pre"]]
    mask[t] = mask[t].copy()
    mask[t][v, col] = False
    dx0, dwr0, dw00, db0 = O.rgcn_layer_backward(cache, G)
    dx1, dwr1, dw01, db1 = O.rgcn_layer_backward(cache, G, relu_mask=mask)
    g = G[t][v, col]
    # bias and root weight
    e = np.zeros_like(db0[t]); e[col] = g
    np.testing.assert_allclose(db0[t] - db1[t], e, atol=1e-12)
    e = np.zeros_like(dw00[t]); e[:, col] = c["x"][t][v] * g
    np.testing.assert_allclose(dw00[t] - dw01[t], e, atol=1e-12)
    for u in range(len(c["x"])):
        if u != t:
            assert np.array_equal(dw00[u], dw01[u]) and np.array_equal(db0[u], db1[u])
    # relation weights and feature gradients
    want_dx = [np.zeros_like(a) for a in c["x"]]
    want_dx[t][v] += g * c["w_root"][t][:, col]
    for r in range(len(c["rel_src"])):
        s, d = c["rel_src"][r], c["rel_dst"][r]
        e = np.zeros_like(dwr0[r])
        if d == t:
            nb = [int(a) for a, b, ty in zip(c["ei"][0], c["ei"][1], c["et"]) if ty == r and b == v]
            if nb:
                e[:, col] = c["x"][s][nb].mean(axis=0) * g
                for a in nb:
                    want_dx[s][a] += g * c["w_rel"][r][:, col] / len(nb)
        np.testing.assert_allclose(dwr0[r] - dwr1[r], e, atol=1e-12)
        keep = np.ones(e.shape[1], bool); keep[col] = d != t
        assert np.array_equal(dwr0[r][:, keep], dwr1[r][:, keep])      # other columns: not a bit moves
    for u in range(len(c["x"])):
        np.testing.assert_allclose(dx0[u] - dx1[u], want_dx[u], atol=1e-12)
