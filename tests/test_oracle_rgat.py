"""Pins of the attention-variant oracle (`rgat_layer_forward/backward`).

The paper cites R-GAT and semantic attention without equations, so nothing here compares against a value the
paper prints; the functions are pinned by (a) a dense masked-softmax evaluation written independently,
(b) special cases that reduce to the mean layer (itself pinned in test_oracle_rgcn.py), (c) softmax
invariants and (d) central finite differences for every parameter and the features."""
import numpy as np
import pytest

from oracle import hgnn_oracle as O


def tiny_case(seed=0, heads=2, D=3, relu=True, with_empty=True):
    rng = np.random.default_rng(seed)
    H = heads * D
    n_src = [5, 6]
    n_dst = [3, 4]
    feat = [4, 5]
    rel_src, rel_dst = [0, 1, 1], [1, 1, 0]          # A->B, B->B, B->A
    x = [rng.normal(size=(n_src[t], feat[t])) for t in range(2)]
    rel_edges = []
    for r in range(3):
        s, d = rel_src[r], rel_dst[r]
        pairs = set()
        for v in range(n_dst[d]):
            if with_empty and v == 0 and r == 1:
                continue                               # an empty neighbourhood
            for u in rng.choice(n_src[s], size=rng.integers(1, 4), replace=False):
                pairs.add((int(u), v))
        pairs = sorted(pairs)
        rng.shuffle(pairs)
        rel_edges.append((np.array([p[0] for p in pairs]), np.array([p[1] for p in pairs])))
    P = dict(
        w_type=[rng.normal(size=(feat[t], H)) * 0.5 for t in range(2)],
        a_src=[rng.normal(size=(heads, D)) for _ in range(3)],
        a_dst=[rng.normal(size=(heads, D)) for _ in range(3)],
        w_sem=rng.normal(size=(H, O.SEM_DIM)) * 0.3, b_sem=rng.normal(size=O.SEM_DIM) * 0.1,
        q_sem=rng.normal(size=O.SEM_DIM) * 0.3,
        bias=[rng.normal(size=H) * 0.1, rng.normal(size=H) * 0.1])
    return dict(x=x, rel_edges=rel_edges, rel_src=rel_src, rel_dst=rel_dst, n_dst=n_dst, n_src=n_src, heads=heads,
                D=D, H=H, relu=relu, P=P)


def fwd(c, P=None, x=None):
    P = c["P"] if P is None else P
    return O.rgat_layer_forward(c["x"] if x is None else x, c["rel_edges"], c["rel_src"], c["rel_dst"], c["n_dst"],
                                P["w_type"], P["a_src"], P["a_dst"], P["w_sem"], P["b_sem"], P["q_sem"], P["bias"],
                                c["relu"], c["heads"])


def dense_attention(c, r):
    """m^r by a dense masked softmax: logits for every (v, u) pair, -inf where there is no edge."""
    P, K, D = c["P"], c["heads"], c["D"]
    s, d = c["rel_src"][r], c["rel_dst"][r]
    z_s = c["x"][s] @ P["w_type"][s]
    z_d = c["x"][d] @ P["w_type"][d]
    M, N = c["n_dst"][d], c["n_src"][s]
    adj = np.zeros((M, N), dtype=bool)
    adj[c["rel_edges"][r][1], c["rel_edges"][r][0]] = True
    out = np.zeros((M, K * D))
    for k in range(K):
        zs, zd = z_s[:, k * D:(k + 1) * D], z_d[:M, k * D:(k + 1) * D]
        logit = (zd @ P["a_dst"][r][k])[:, None] + (zs @ P["a_src"][r][k])[None, :]
        logit = np.where(logit > 0, logit, 0.2 * logit)
        logit = np.where(adj, logit, -np.inf)
        for v in range(M):
            if adj[v].any():
                w = np.exp(logit[v] - logit[v][adj[v]].max())
                w /= w.sum()
                out[v, k * D:(k + 1) * D] = w @ zs
    return out


def test_aggregation_matches_dense_masked_softmax():
    c = tiny_case(seed=1)
    _, cache = fwd(c)
    for r in range(3):
        assert np.allclose(cache["m"][r], dense_attention(c, r), rtol=1e-12, atol=1e-13)
    assert np.all(cache["m"][1][0] == 0)               # the empty neighbourhood gives zero


def test_attention_rows_sum_to_one_and_are_positive():
    c = tiny_case(seed=2)
    _, cache = fwd(c)
    for r in range(3):
        for a in cache["alphas"][r]:
            if a is not None:
                assert np.allclose(a.sum(axis=0), 1.0, atol=1e-14) and (a > 0).all()


def test_zero_attention_vectors_give_the_mean_of_projected_neighbours():
    c = tiny_case(seed=3)
    P = dict(c["P"])
    P["a_src"] = [np.zeros_like(a) for a in P["a_src"]]
    P["a_dst"] = [np.zeros_like(a) for a in P["a_dst"]]
    _, cache = fwd(c, P)
    for r in range(3):
        s, d = c["rel_src"][r], c["rel_dst"][r]
        z = c["x"][s] @ P["w_type"][s]
        A = np.zeros((c["n_dst"][d], c["n_src"][s]))
        np.add.at(A, (c["rel_edges"][r][1], c["rel_edges"][r][0]), 1.0)
        deg = A.sum(axis=1, keepdims=True)
        ref = np.divide(A, deg, out=np.zeros_like(A), where=deg > 0) @ z
        assert np.allclose(cache["m"][r], ref, atol=1e-13)


def test_zero_semantic_query_gives_the_average_over_relations():
    c = tiny_case(seed=4, relu=False)
    P = dict(c["P"])
    P["q_sem"] = np.zeros_like(P["q_sem"])
    h, cache = fwd(c, P)
    # type B (1) receives relations 0 and 1, type A (0) only relation 2
    assert np.allclose(h[1], 0.5 * (cache["m"][0] + cache["m"][1]) + P["bias"][1][None], atol=1e-13)
    assert np.allclose(h[0], cache["m"][2] + P["bias"][0][None], atol=1e-13)
    assert cache["beta"][2] == 1.0 and abs(cache["beta"][0] - 0.5) < 1e-15


def test_semantic_weights_follow_their_definition():
    c = tiny_case(seed=5)
    P = c["P"]
    _, cache = fwd(c)
    w = []
    for r in (0, 1):
        t = np.tanh(cache["m"][r] @ P["w_sem"] + P["b_sem"])
        w.append(np.mean(t @ P["q_sem"]))
    b0 = 1.0 / (1.0 + np.exp(w[1] - w[0]))
    assert abs(cache["beta"][0] - b0) < 1e-14 and abs(cache["beta"][0] + cache["beta"][1] - 1.0) < 1e-14


def test_reduces_to_the_mean_layer_when_attention_is_switched_off():
    """a = 0 and q = 0: h = act( (1/|R_d|) sum_r mean_u x_u W_{src(r)} + b ), which the mean-aggregation
    oracle evaluates with relation weights W_{src(r)} / |R_d| and no root term."""
    c = tiny_case(seed=6)
    P = dict(c["P"])
    P["a_src"] = [np.zeros_like(a) for a in P["a_src"]]
    P["a_dst"] = [np.zeros_like(a) for a in P["a_dst"]]
    P["q_sem"] = np.zeros_like(P["q_sem"])
    h, _ = fwd(c, P)
    cnt = [sum(1 for r in range(3) if c["rel_dst"][r] == d) for d in range(2)]
    w_rel = [P["w_type"][c["rel_src"][r]] / cnt[c["rel_dst"][r]] for r in range(3)]
    h2, _ = O.rgcn_layer_forward(c["x"], c["rel_edges"], c["rel_src"], c["rel_dst"], c["n_dst"], w_rel, [None, None],
                                 P["bias"], c["relu"])
    for t in range(2):
        assert np.allclose(h[t], h2[t], atol=1e-13)


def test_permuting_neighbour_order_changes_nothing():
    c = tiny_case(seed=7)
    h, _ = fwd(c)
    rng = np.random.default_rng(0)
    c2 = dict(c)
    c2["rel_edges"] = []
    for s, d in c["rel_edges"]:
        p = rng.permutation(len(s))
        c2["rel_edges"].append((s[p], d[p]))
    h2, _ = fwd(c2)
    for t in range(2):
        assert np.allclose(h[t], h2[t], atol=1e-13)


@pytest.mark.parametrize("relu", [False, True])
def test_backward_matches_central_differences(relu):
    c = tiny_case(seed=8, relu=relu)
    rng = np.random.default_rng(11)
    coef = [rng.normal(size=(c["n_dst"][t], c["H"])) for t in range(2)]

    def loss(P=None, x=None):
        h, _ = fwd(c, P, x)
        return sum(float((coef[t] * h[t]).sum()) for t in range(2))

    h, cache = fwd(c)
    g = O.rgat_layer_backward(cache, coef)
    eps = 1e-6

    def fd(get, setv, shape, idxs):
        out = []
        for idx in idxs:
            old = get()[idx]
            setv(idx, old + eps); lp = loss(*cur())
            setv(idx, old - eps); lm = loss(*cur())
            setv(idx, old)
            out.append((lp - lm) / (2 * eps))
        return np.array(out)

    P = {k: ([a.copy() for a in v] if isinstance(v, list) else v.copy()) for k, v in c["P"].items()}
    X = [a.copy() for a in c["x"]]
    cur = lambda: (P, X)

    def check(arr, grad, name, n=12):
        flat_idx = rng.choice(arr.size, size=min(n, arr.size), replace=False)
        idxs = [np.unravel_index(i, arr.shape) for i in flat_idx]
        num = fd(lambda: arr, lambda i, v: arr.__setitem__(i, v), arr.shape, idxs)
        ana = np.array([grad[i] for i in idxs])
        scale = max(np.abs(ana).max(), np.abs(num).max(), 1e-8)
        assert np.abs(num - ana).max() / scale < 1e-6, (name, num, ana)

    for t in range(2):
        check(P["w_type"][t], g["dw_type"][t], f"w_type{t}")
        check(P["bias"][t], g["dbias"][t], f"bias{t}")
        check(X[t], g["dx"][t], f"x{t}")
    for r in range(3):
        check(P["a_src"][r], g["da_src"][r], f"a_src{r}")
        check(P["a_dst"][r], g["da_dst"][r], f"a_dst{r}")
    check(P["w_sem"], g["dw_sem"], "w_sem", n=20)
    check(P["b_sem"], g["db_sem"], "b_sem")
    check(P["q_sem"], g["dq_sem"], "q_sem")


def test_relation_without_edges_still_takes_part_in_the_fusion():
    c = tiny_case(seed=9, relu=False)
    c["rel_edges"][0] = (np.zeros(0, dtype=np.int64), np.zeros(0, dtype=np.int64))
    h, cache = fwd(c)
    P = c["P"]
    assert np.all(cache["m"][0] == 0)
    w0 = float(np.tanh(P["b_sem"]) @ P["q_sem"])                      # every row has m = 0
    t1 = np.tanh(cache["m"][1] @ P["w_sem"] + P["b_sem"])
    w1 = float(np.mean(t1 @ P["q_sem"]))
    assert abs(cache["beta"][0] - 1.0 / (1.0 + np.exp(w1 - w0))) < 1e-14
    g = O.rgat_layer_backward(cache, [np.ones_like(a) for a in h])
    assert np.all(g["da_src"][0] == 0) and np.all(g["da_dst"][0] == 0)


def test_relu_mask_equal_to_own_decisions_reproduces_the_plain_backward_bit_for_bit():
    c = tiny_case(seed=5)
    h, cache = fwd(c)
    rng = np.random.default_rng(6)
    G = [rng.normal(size=a.shape) for a in h]
    plain = O.rgat_layer_backward(cache, G)
    masked = O.rgat_layer_backward(cache, G, relu_mask=[p > 0 for p in cache["pre"]])
    for k in plain:
        a, b = plain[k], masked[k]
        if isinstance(a, list):
            for u, v in zip(a, b):
                assert (u is None and v is None) or np.array_equal(u, v)
        else:
            assert np.array_equal(a, b)


def test_flipping_one_relu_decision_equals_zeroing_that_unit_s_output_gradient():
    """The ReLU is the last step of the layer, so switching unit (t, v, c) off must give exactly the gradients of the
    plain backward fed with an output gradient whose element (v, c) is zero -- and the bias gradient's element c must
    drop by that element (the bias is added right before the activation)."""
    c = tiny_case(seed=7)
    h, cache = fwd(c)
    rng = np.random.default_rng(8)
    G = [rng.normal(size=a.shape) for a in h]
    t = 1
    act = np.argwhere(cache["pre"][t] > 0)
    v, col = (int(a) for a in act[len(act) // 2])
    mask = [p > 0 for p in cache["pre"]]
    mask[t] = mask[t].copy()
    mask[t][v, col] = False
    G0 = [g.copy() for g in G]
    G0[t][v, col] = 0.0
    masked = O.rgat_layer_backward(cache, G, relu_mask=mask)
    zeroed = O.rgat_layer_backward(cache, G0)
    plain = O.rgat_layer_backward(cache, G)
    for k in masked:
        a, b = masked[k], zeroed[k]
        for u, w in (zip(a, b) if isinstance(a, list) else [(a, b)]):
            assert (u is None and w is None) or np.array_equal(u, w)
    e = np.zeros_like(plain["dbias"][t]); e[col] = G[t][v, col]
    np.testing.assert_allclose(plain["dbias"][t] - masked["dbias"][t], e, atol=1e-12)
    assert not np.array_equal(plain["dw_type"][0], masked["dw_type"][0])
