"""Pins of the sampler oracle to things other than itself: the published SplitMix64 test vectors, brute-force
neighbourhoods, the structural rules a layer-wise neighbour sample must obey, and the uniformity of the
subset choice."""
import numpy as np
import pytest

from oracle import sampler_oracle as S
from workloads import build_graph, make_config


def test_mix64_is_splitmix64():
    # outputs of SplitMix64 for seed 0 (widely published, e.g. as the seeding sequence of the xoshiro family's
    # reference code) and for seed 1234567 (the Rosetta Code task "Pseudo-random numbers/Splitmix64")
    g = 0x9E3779B97F4A7C15
    m = (1 << 64) - 1
    assert [S.mix64((i * g) & m) for i in range(4)] == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F,
                                                          0xF88BB8A8724C81EC]
    assert [S.mix64((1234567 + i * g) & m) for i in range(5)] == [6457827717110365317, 3203168211198807973,
                                                                   9817491932198370423, 4593380528125082431,
                                                                   16408922859458223821]


def test_subset_choice_is_a_uniform_subset():
    deg, fanout, n = 10, 3, 30000
    counts = np.zeros(deg)
    pair = np.zeros((deg, deg))
    for k in range(n):
        pos = S.choose_positions(deg, fanout, S.mix64(k))
        assert len(pos) == fanout and len(set(pos)) == fanout and all(0 <= p < deg for p in pos)
        counts[pos] += 1
        for a in pos:
            for b in pos:
                pair[a, b] += a != b
    # every position is taken with probability fanout/deg: binomial sd = sqrt(n p (1-p)) ~ 79
    assert np.abs(counts - n * fanout / deg).max() < 5 * np.sqrt(n * 0.3 * 0.7)
    # every unordered pair with probability C(8,1)/C(10,3) = 1/15
    off = pair[~np.eye(deg, dtype=bool)]
    assert np.abs(off - n / 15).max() < 5 * np.sqrt(n / 15 * 14 / 15)
    assert S.choose_positions(4, 4, 99) == [0, 1, 2, 3] and S.choose_positions(0, 5, 1) == []


def _graph(index, scale=1.0):
    cfg = make_config(index, scale=scale)
    return cfg, build_graph(cfg)


def _sample(g, tt, targets, fanouts, seed):
    sch = g.schema
    return S.sample_minibatch(g.num_nodes, sch.rel_src, sch.rel_dst, g.in_indptr, g.in_nbr, g.edge_off, tt, targets,
                              fanouts, seed)


def _global_lists(mb, L):
    """Per layer (execution order) the global ids of its source rows per type: the last hop's are `ids`, every
    earlier layer's are prefixes (destinations first)."""
    out = []
    for l in range(L):
        out.append([mb["ids"][t][: mb["blocks"][l]["n_src"][t]] for t in range(len(mb["ids"]))])
    return out


@pytest.mark.parametrize("index,scale,fanouts,nt", [(0, 1.0, [5], 64), (0, 1.0, [3, 2], 40), (2, 0.01, [6, 4], 50),
                                                    (5, 1.0, [4, 4], 30)])
def test_structure_against_brute_force(index, scale, fanouts, nt):
    cfg, g = _graph(index, scale)
    sch = g.schema
    T, R, L = sch.num_types, sch.num_rels, len(fanouts)
    tt = 1 if index == 0 else int(np.argmax(np.bincount(sch.rel_dst, minlength=T) * (np.array(g.num_nodes) >= nt)))
    targets = np.random.default_rng(5).choice(g.num_nodes[tt], nt, replace=False)
    mb = _sample(g, tt, targets, fanouts, seed=77)
    assert len(mb["blocks"]) == L
    assert np.array_equal(mb["ids"][tt][:nt], targets)                      # targets first
    for t in range(T):
        assert len(np.unique(mb["ids"][t])) == len(mb["ids"][t])           # a vertex has one row
    src_lists = _global_lists(mb, L)
    # brute-force adjacency: set of (src, dst) pairs per relation, and the relation of every global edge id
    for l, b in enumerate(mb["blocks"]):
        fanout = fanouts[L - 1 - l]
        if l + 1 < L:
            assert b["n_dst"] == mb["blocks"][l + 1]["n_src"]               # a layer's outputs feed the next
        else:
            assert b["n_dst"] == [nt if t == tt else 0 for t in range(T)]
        assert all(b["n_dst"][t] <= b["n_src"][t] for t in range(T))
        es, ed = b["edge_index"]
        seen_src = [np.zeros(n, bool) for n in b["n_src"]]
        for r in range(R):
            s, d = sch.rel_src[r], sch.rel_dst[r]
            m = b["edge_type"] == r
            assert np.array_equal(g.edge_type[b["edge_id"][m]], np.full(m.sum(), r))
            pos = b["edge_id"][m] - g.edge_off[r]
            gs, gd = src_lists[l][s][es[m]], src_lists[l][d][ed[m]]
            assert np.array_equal(g.in_nbr[r][pos], gs)                     # the edge exists: right source ...
            assert np.all((g.in_indptr[r][gd] <= pos) & (pos < g.in_indptr[r][gd + 1]))   # ... right destination
            seen_src[s][es[m]] = True
            deg = (g.in_indptr[r][1:] - g.in_indptr[r][:-1])[src_lists[l][d][: b["n_dst"][d]]]
            cnt = np.bincount(ed[m], minlength=b["n_dst"][d])
            assert np.array_equal(cnt, np.minimum(deg, fanout))             # min(deg, fanout) per destination
            assert len(np.unique(b["edge_id"][m])) == m.sum()               # without replacement
        for t in range(T):                                                   # no row beyond the destinations is idle
            assert seen_src[t][b["n_dst"][t]:].all()


def test_large_fanout_returns_whole_neighbourhoods():
    cfg, g = _graph(0)
    sch = g.schema
    targets = np.arange(20)
    mb = _sample(g, 1, targets, [10 ** 6], seed=3)
    b = mb["blocks"][0]
    for r in range(sch.num_rels):
        if sch.rel_dst[r] != 1:
            continue
        m = b["edge_type"] == r
        want = np.concatenate([np.arange(g.in_indptr[r][v], g.in_indptr[r][v + 1]) for v in targets]) + g.edge_off[r]
        assert np.array_equal(b["edge_id"][m], want)                        # every edge, stored order


def test_seed_and_hop_change_the_draws():
    cfg, g = _graph(2, 0.01)
    targets = np.arange(40)
    a = _sample(g, 0, targets, [3, 3], seed=1)
    b = _sample(g, 0, targets, [3, 3], seed=2)
    c = _sample(g, 0, targets, [3, 3], seed=1)
    assert not np.array_equal(a["blocks"][1]["edge_id"], b["blocks"][1]["edge_id"])
    assert all(np.array_equal(x["edge_id"], y["edge_id"]) for x, y in zip(a["blocks"], c["blocks"]))
