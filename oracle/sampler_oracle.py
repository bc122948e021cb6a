"""CPU oracle of the in-the-loop neighbour sampler (test infrastructure only).

The paper's workflow (Section 2.3, step 1 "Sampling"; Fig. 6, the CPU thread that samples and then selects
edge indices) takes layer-wise neighbour sampling as given; it fixes neither the random numbers nor the
order of the output.  This file writes out, in plain Python loops, the rule this repository uses so that a
compiled sampler can be compared with it bit for bit.  It shares no code with the library; only tests,
the smoke check and the benchmark's CPU baseline may import it.

Rule.  Hops are numbered from the targets outward (hop 1 uses fanouts[0]).  In hop h the destination
vertices of every type are the source vertices of hop h-1 (hop 1: the targets, all of one type).  A hop's
source list of a type starts with its destination list (so destinations are a prefix) and grows by every
vertex reached for the first time, in the order it is reached.  Relations are visited in ascending id,
inside a relation the destination vertices in list order; destination v of relation r with in-neighbour
list nb (deg entries, the graph's stored order) contributes

    all positions 0..deg-1 in order                         if deg <= fanout
    a subset of `fanout` positions chosen with Floyd's      otherwise:
      for c = 0..fanout-1:  j = deg - fanout + c;  t = floor(draw(c) * (j + 1) / 2^64);
                            position = j if t was chosen before else t

with draw(c) = mix64(key + c), key = mix64(mix64(mix64(mix64(seed) ^ h) ^ r) ^ v) (v the global id), and
mix64 the SplitMix64 output function (Steele, Lea, Flood 2014): z += 0x9E3779B97F4A7C15; z = (z ^ z>>30) *
0xBF58476D1CE4E5B9; z = (z ^ z>>27) * 0x94D049BB133111EB; z ^ z>>31, all modulo 2^64.  Every chosen
position p gives one edge (local source, local destination) with global edge id edge_off[r] + first + p,
appended in that order.  The block of hop h feeds layer L - h + 1; blocks are returned in execution
order, and `ids` are the source lists of the last hop.
"""
import numpy as np

_M = (1 << 64) - 1


def mix64(z: int) -> int:
    z = (z + 0x9E3779B97F4A7C15) & _M
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _M
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _M
    return z ^ (z >> 31)


def choose_positions(deg: int, fanout: int, key: int):
    if deg <= fanout:
        return list(range(deg))
    chosen = []
    for c in range(fanout):
        j = deg - fanout + c
        t = (mix64((key + c) & _M) * (j + 1)) >> 64
        chosen.append(j if t in chosen else t)
    return chosen


def sample_minibatch(num_nodes, rel_src, rel_dst, in_indptr, in_nbr, edge_off, target_type, targets, fanouts, seed):
    """Returns dict(ids=[T arrays int64], blocks=[per layer, execution order: dict(n_src, n_dst, edge_index
    int64 [2,E], edge_id int64 [E], edge_type int32 [E])])."""
    T, R = len(num_nodes), len(rel_src)
    dst_ids = [[] for _ in range(T)]
    dst_ids[target_type] = [int(v) for v in targets]
    assert len(set(dst_ids[target_type])) == len(dst_ids[target_type]), "targets must be distinct"
    k0 = mix64(int(seed) & _M)
    blocks = []
    for h, fanout in enumerate(fanouts, start=1):
        kh = mix64(k0 ^ h)
        src_ids = [list(d) for d in dst_ids]
        local = [{v: i for i, v in enumerate(d)} for d in dst_ids]
        es, ed, eid, ety = [], [], [], []
        for r in range(R):
            s, d = rel_src[r], rel_dst[r]
            kr = mix64(kh ^ r)
            ptr, nb = in_indptr[r], in_nbr[r]
            for i, v in enumerate(dst_ids[d]):
                first, deg = int(ptr[v]), int(ptr[v + 1] - ptr[v])
                for p in choose_positions(deg, fanout, mix64(kr ^ v)):
                    u = int(nb[first + p])
                    if u not in local[s]:
                        local[s][u] = len(src_ids[s])
                        src_ids[s].append(u)
                    es.append(local[s][u]); ed.append(i); eid.append(int(edge_off[r]) + first + p); ety.append(r)
        blocks.append(dict(n_src=[len(x) for x in src_ids], n_dst=[len(x) for x in dst_ids],
                           edge_index=np.array([es, ed], dtype=np.int64).reshape(2, -1),
                           edge_id=np.array(eid, dtype=np.int64), edge_type=np.array(ety, dtype=np.int32)))
        dst_ids = src_ids
    blocks.reverse()
    return dict(ids=[np.array(x, dtype=np.int64) for x in dst_ids], blocks=blocks)
