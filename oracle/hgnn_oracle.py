"""CPU oracle for the mini-batch HGNN layer hot path (TEST INFRASTRUCTURE ONLY).

Plain, slow numpy in float64.  It evaluates the layer exactly as it is defined,
*unmerged*: one vertex type and one relation (semantic graph) at a time, the
four stages of an HGNN layer in the order the paper lists them (Section 2.2:
semantic graph build, feature projection, neighbour aggregation, semantic
fusion), and the backward pass as the step-by-step reverse of that forward.

Only tests, the smoke check and the benchmark's `cpu_baseline` leg may import
this module.  It shares no code with the HIP path and imports nothing from it.

What the paper fixes and what it leaves open
--------------------------------------------
The paper names the stages and gives two algorithms (Algorithm 1: aggregation
over type-first, merged features; Algorithm 2: edge-index selection).  Both are
exact re-organisations: they change launch structure and data layout, never the
result (Section 4.2).  It prints no layer equations; the R-GCN layer evaluated
here is
    h_v = act( x_v W_0^{type(v)} + b_{type(v)}
               + sum_{r : dst(r)=type(v)}  mean_{u in N_r(v)} x_u W_r )
with an empty neighbourhood contributing zero, the mean taken over the sampled
edges of relation r that end in v.

Pins (see tests/test_oracle_*.py): a hand-worked 4-vertex example, dense
adjacency-matrix brute force, a scipy.sparse reduction for one relation,
merged-vs-unmerged equality, constant-feature means, permutation equivariance,
project/aggregate commutation, finite-difference gradients, numpy.lexsort for
the index outputs, closed forms for the cross-entropy; for the optional
`relu_mask` of the backward functions: the layer's own decisions reproduce the
plain backward bit for bit, and flipping one unit moves exactly that unit's
terms (closed form).

Parity unpinned by the paper: the attention variant's definition (functions
`rgat_*`): the paper cites R-GAT without equations, so those functions follow
the form written out in their docstrings and are pinned by special cases that
reduce to the mean layer, by a dense masked-softmax brute force, by softmax
invariants and by finite differences - not by anything the paper prints.
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


# --------------------------------------------------------------------------- #
# Stage 0: type-first feature layout (Section 4.2, "Reorganizing Features")
# --------------------------------------------------------------------------- #
def merge_features(stores, ids):
    """Rows of the mini-batch, grouped by vertex type first and by position in the
    type's id list second.  Returns (blocks, row_off, elem_off, flat) where block t
    is `stores[t][ids[t]]`, `row_off[t]` counts rows before type t, `elem_off[t]`
    counts scalars before type t and `flat` is the blocks laid end to end."""
    T = len(stores)
    blocks, row_off, elem_off = [], [0], [0]
    for t in range(T):
        blk = np.zeros((len(ids[t]), stores[t].shape[1]), dtype=stores[t].dtype)
        for i, gid in enumerate(ids[t]):
            blk[i, :] = stores[t][int(gid), :]
        blocks.append(blk)
        row_off.append(row_off[-1] + blk.shape[0])
        elem_off.append(elem_off[-1] + blk.shape[0] * blk.shape[1])
    flat = np.concatenate([b.ravel() for b in blocks]) if T else np.zeros(0)
    return blocks, np.array(row_off, dtype=np.int32), np.array(elem_off, dtype=np.int64), flat


# --------------------------------------------------------------------------- #
# Stage 1: semantic graph build (Algorithm 2, then grouping by destination)
# --------------------------------------------------------------------------- #
def edge_index_select(edge_index, num_rels, edge_type=None, edge_id=None, global_edge_type=None):
    """Algorithm 2 for one layer.  The layer's edge types are looked up through the
    edge ids (or given directly); then, for each relation j in turn, the edges whose
    type equals j are selected, keeping their input order.  Returns, per relation,
    (src, dst, pos) with `pos` the selected edges' positions in the input list."""
    if edge_type is None:
        edge_type_layer = np.asarray(global_edge_type)[np.asarray(edge_id)]
    else:
        edge_type_layer = np.asarray(edge_type)
    out = []
    for j in range(num_rels):
        mask = (edge_type_layer == j)
        pos = np.nonzero(mask)[0]
        out.append((np.asarray(edge_index[0])[mask].astype(np.int64),
                    np.asarray(edge_index[1])[mask].astype(np.int64), pos.astype(np.int64)))
    return out


def semantic_csr(selected, rel_src, rel_dst, n_src, n_dst, transpose_types=None):
    """One CSR over all relations.  Relation r owns rows
    rel_row_off[r] .. rel_row_off[r+1]-1, one per destination vertex of type dst(r)
    (also when r has no edge).  A row lists its edges in input order; `colidx` is the
    source's row in the type-first feature matrix; `perm` the edge's input position.
    The transpose groups the same edges by `colidx`, ascending CSR position inside a
    group: `crow` is the edge's CSR row, `cperm` its CSR position.  With
    `transpose_types` (0/1 per vertex type) the transpose lists only the edges whose
    source vertex is of a type flagged 1 (rows of the other types stay empty)."""
    R, T = len(rel_src), len(n_src)
    row_off = [0]
    for t in range(T):
        row_off.append(row_off[-1] + int(n_src[t]))
    rel_row_off = [0]
    for r in range(R):
        rel_row_off.append(rel_row_off[-1] + int(n_dst[rel_dst[r]]))
    rows = [[] for _ in range(rel_row_off[-1])]
    rel_edge_off = [0]
    for r in range(R):
        src, dst, pos = selected[r]
        for k in range(len(src)):
            s, d = int(src[k]), int(dst[k])
            if not (0 <= s < n_src[rel_src[r]] and 0 <= d < n_dst[rel_dst[r]]):
                raise ValueError("edge endpoint out of range")
            rows[rel_row_off[r] + d].append((row_off[rel_src[r]] + s, int(pos[k])))
        rel_edge_off.append(rel_edge_off[-1] + len(src))
    rowptr, colidx, perm = [0], [], []
    for lst in rows:
        for (c, p) in lst:
            colidx.append(c); perm.append(p)
        rowptr.append(len(colidx))
    cols = [[] for _ in range(row_off[-1])]
    type_of_row = []
    for t in range(T):
        type_of_row += [t] * int(n_src[t])
    for rho in range(len(rows)):
        for k in range(rowptr[rho], rowptr[rho + 1]):
            if transpose_types is None or transpose_types[type_of_row[colidx[k]]]:
                cols[colidx[k]].append((rho, k))
    cptr, crow, cperm = [0], [], []
    for lst in cols:
        for (rho, k) in lst:
            crow.append(rho); cperm.append(k)
        cptr.append(len(crow))
    i32 = lambda a: np.array(a, dtype=np.int32)
    return dict(row_off=i32(row_off), rel_row_off=i32(rel_row_off), rel_edge_off=i32(rel_edge_off),
                rowptr=i32(rowptr), colidx=i32(colidx), perm=i32(perm),
                cptr=i32(cptr), crow=i32(crow), cperm=i32(cperm))


def _neighbour_lists(src, dst, num_dst):
    nb = [[] for _ in range(num_dst)]
    for k in range(len(src)):
        nb[int(dst[k])].append(int(src[k]))
    return nb


# --------------------------------------------------------------------------- #
# Stages 2-4: R-GCN layer, forward and backward, unmerged
# --------------------------------------------------------------------------- #
def rgcn_layer_forward(x, rel_edges, rel_src, rel_dst, n_dst, w_rel, w_root, bias, relu):
    """x: per type [N_t, F_t]; rel_edges: per relation (src_local, dst_local, ...);
    w_rel[r]: [F_src(r), H]; w_root[t]: [F_t, H] or None; bias[t]: [H] or None.
    Returns (h per type [n_dst[t], H], cache)."""
    T, R = len(x), len(rel_src)
    x = [np.asarray(a, dtype=F64) for a in x]
    H = int(np.asarray(w_rel[0]).shape[1]) if R else int(np.asarray(w_root[0]).shape[1])
    pre = []
    for t in range(T):                                   # root term and bias
        p = np.zeros((int(n_dst[t]), H), dtype=F64)
        if n_dst[t] > 0:
            if w_root[t] is not None:
                p += x[t][: n_dst[t]] @ np.asarray(w_root[t], dtype=F64)
            if bias[t] is not None:
                p += np.asarray(bias[t], dtype=F64)[None, :]
        pre.append(p)
    nbrs = []
    for r in range(R):
        s, d = rel_src[r], rel_dst[r]
        nb = _neighbour_lists(rel_edges[r][0], rel_edges[r][1], int(n_dst[d]))
        nbrs.append(nb)
        if n_dst[d] == 0 or len(rel_edges[r][0]) == 0:
            continue
        y = x[s] @ np.asarray(w_rel[r], dtype=F64)       # feature projection
        for v in range(int(n_dst[d])):                   # neighbour aggregation (mean)
            if nb[v]:
                pre[d][v] += y[nb[v]].sum(axis=0) / len(nb[v])   # ... and fusion (sum over r)
    h = [np.maximum(p, 0.0) if relu else p.copy() for p in pre]
    cache = dict(x=x, nbrs=nbrs, pre=pre, rel_src=rel_src, rel_dst=rel_dst, n_dst=list(n_dst),
                 w_rel=w_rel, w_root=w_root, bias=bias, relu=relu)
    return h, cache


def rgcn_layer_backward(cache, grad_h, relu_mask=None):
    """Reverse of `rgcn_layer_forward`, one step at a time.  grad_h: per type
    [n_dst[t], H].  Returns (dx per type, dw_rel, dw_root, dbias); parameters that
    received no contribution get zeros (None where the parameter is None).
    relu_mask (per type boolean [n_dst[t], H], optional) replaces the decision
    `pre > 0` of the ReLU's backward; parity tests use it to settle units whose
    pre-activation is zero to within rounding, where either decision is valid."""
    x, nbrs, pre = cache["x"], cache["nbrs"], cache["pre"]
    rel_src, rel_dst, n_dst = cache["rel_src"], cache["rel_dst"], cache["n_dst"]
    w_rel, w_root, bias = cache["w_rel"], cache["w_root"], cache["bias"]
    T, R = len(x), len(rel_src)
    gp = []
    for t in range(T):
        g = np.asarray(grad_h[t], dtype=F64).reshape(pre[t].shape)
        if not cache["relu"]:
            gp.append(g.copy())
        elif relu_mask is not None:
            gp.append(g * np.asarray(relu_mask[t], dtype=bool).reshape(pre[t].shape))
        else:
            gp.append(g * (pre[t] > 0))
    dx = [np.zeros_like(a) for a in x]
    dw_root, dbias = [], []
    for t in range(T):
        if w_root[t] is None:
            dw_root.append(None)
        else:
            w0 = np.asarray(w_root[t], dtype=F64)
            dw_root.append(x[t][: n_dst[t]].T @ gp[t])
            dx[t][: n_dst[t]] += gp[t] @ w0.T
        dbias.append(None if bias[t] is None else gp[t].sum(axis=0))
    dw_rel = []
    for r in range(R):
        s, d = rel_src[r], rel_dst[r]
        w = np.asarray(w_rel[r], dtype=F64)
        dy = np.zeros((x[s].shape[0], w.shape[1]), dtype=F64)
        for v in range(int(n_dst[d])):
            nb = nbrs[r][v]
            if nb:
                np.add.at(dy, nb, gp[d][v] / len(nb))
        dw_rel.append(x[s].T @ dy)
        dx[s] += dy @ w.T
    return dx, dw_rel, dw_root, dbias


def rgcn_layer_forward_merged(flat, feat_dim, csr, rel_src, rel_dst, n_dst, w_rel, w_root, bias, relu):
    """Same layer, but reading the type-first flat feature buffer through the merged
    CSR (the data path of Algorithm 1): each merged row gathers its sources through
    `colidx`, in row order.  Used to check that merging changes no value."""
    T, R = len(feat_dim), len(rel_src)
    row_off, rel_row_off = csr["row_off"], csr["rel_row_off"]
    rowptr, colidx = csr["rowptr"], csr["colidx"]
    blocks, e = [], 0
    for t in range(T):
        n = int(row_off[t + 1] - row_off[t])
        blocks.append(np.asarray(flat[e: e + n * feat_dim[t]], dtype=F64).reshape(n, feat_dim[t]))
        e += n * feat_dim[t]
    H = int(np.asarray(w_rel[0]).shape[1])
    pre = []
    for t in range(T):
        p = np.zeros((int(n_dst[t]), H), dtype=F64)
        if n_dst[t] > 0:
            if w_root[t] is not None:
                p += blocks[t][: n_dst[t]] @ np.asarray(w_root[t], dtype=F64)
            if bias[t] is not None:
                p += np.asarray(bias[t], dtype=F64)[None, :]
        pre.append(p)
    for r in range(R):
        s, d = rel_src[r], rel_dst[r]
        if rel_row_off[r + 1] == rel_row_off[r]:
            continue
        y = blocks[s] @ np.asarray(w_rel[r], dtype=F64)
        for v in range(int(n_dst[d])):
            rho = int(rel_row_off[r]) + v
            a, b = int(rowptr[rho]), int(rowptr[rho + 1])
            if b > a:
                pre[d][v] += y[colidx[a:b] - row_off[s]].sum(axis=0) / (b - a)
    return [np.maximum(p, 0.0) if relu else p for p in pre]


# --------------------------------------------------------------------------- #
# Loss used by the two academic-graph configurations
# --------------------------------------------------------------------------- #
# --------------------------------------------------------------------------- #
# Attention variant: per-relation edge attention + semantic attention fusion
# (the paper evaluates R-GAT, Section 5.1, without printing its equations)
# --------------------------------------------------------------------------- #
LEAKY_SLOPE = 0.2
SEM_DIM = 128


def rgat_layer_forward(x, rel_edges, rel_src, rel_dst, n_dst, w_type, a_src, a_dst, w_sem, b_sem, q_sem,
                       bias, relu, heads):
    """Attention layer, the four stages in order.
      projection   z_t = x_t W_t                       per vertex type, H = heads * D columns
      aggregation  for relation r (s -> d), destination v, head k, neighbours u in N_r(v):
                     e_u = LeakyReLU_0.2( a_src[r][k] . z_s[u]^k  +  a_dst[r][k] . z_d[v]^k )
                     alpha = softmax_u(e)             (row maximum subtracted first)
                     m_v^r = concat_k sum_u alpha_u z_s[u]^k ;   empty neighbourhood -> 0
      fusion       per destination type d, over R_d = {r : dst(r) = d}:
                     w_r = (1/M_d) sum_v q . tanh(m_v^r W_s + b_s)    (all M_d rows, empty ones with m = 0)
                     beta = softmax_{r in R_d}(w)
                     pre_v = sum_r beta_r m_v^r + b_d ;  h = ReLU(pre) if relu
    No root term.  x: per type [N_t, F_t]; w_type[t]: [F_t, H]; a_src[r], a_dst[r]: [heads, D];
    w_sem [H, 128], b_sem [128], q_sem [128]; bias[t]: [H] or None.  Returns (h per type, cache)."""
    T, R = len(x), len(rel_src)
    x = [np.asarray(a, dtype=F64) for a in x]
    H = int(np.asarray(w_type[0]).shape[1])
    K = int(heads)
    D = H // K
    assert K * D == H
    z = [x[t] @ np.asarray(w_type[t], dtype=F64) for t in range(T)]          # feature projection
    ws, bs, q = np.asarray(w_sem, dtype=F64), np.asarray(b_sem, dtype=F64), np.asarray(q_sem, dtype=F64)
    nbrs, alphas, scores, m = [], [], [], []
    for r in range(R):                                                       # neighbour aggregation
        s, d = rel_src[r], rel_dst[r]
        M = int(n_dst[d])
        nb = _neighbour_lists(rel_edges[r][0], rel_edges[r][1], M)
        As, Ad = np.asarray(a_src[r], dtype=F64), np.asarray(a_dst[r], dtype=F64)
        mr = np.zeros((M, H), dtype=F64)
        al, sc = [None] * M, [None] * M
        for v in range(M):
            if not nb[v]:
                continue
            zu = z[s][nb[v]].reshape(len(nb[v]), K, D)
            zv = z[d][v].reshape(K, D)
            sv = (zu * As[None]).sum(axis=2) + (zv * Ad).sum(axis=1)[None, :]    # [n, K] before the LeakyReLU
            e = np.where(sv > 0, sv, LEAKY_SLOPE * sv)
            e = e - e.max(axis=0, keepdims=True)
            a = np.exp(e)
            a /= a.sum(axis=0, keepdims=True)
            mr[v] = (a[:, :, None] * zu).sum(axis=0).reshape(H)
            al[v], sc[v] = a, sv
        nbrs.append(nb); alphas.append(al); scores.append(sc); m.append(mr)
    pre, beta, tanhs = [], [None] * R, [None] * R
    for d in range(T):                                                       # semantic fusion
        M = int(n_dst[d])
        p = np.zeros((M, H), dtype=F64)
        Rd = [r for r in range(R) if rel_dst[r] == d]
        if M > 0 and Rd:
            w = np.zeros(len(Rd), dtype=F64)
            for i, r in enumerate(Rd):
                tanhs[r] = np.tanh(m[r] @ ws + bs[None, :])
                w[i] = (tanhs[r] @ q).sum() / M
            ew = np.exp(w - w.max())
            b = ew / ew.sum()
            for i, r in enumerate(Rd):
                beta[r] = float(b[i])
                p += b[i] * m[r]
        if M > 0 and bias[d] is not None:
            p += np.asarray(bias[d], dtype=F64)[None, :]
        pre.append(p)
    h = [np.maximum(p, 0.0) if relu else p.copy() for p in pre]
    cache = dict(x=x, z=z, nbrs=nbrs, alphas=alphas, scores=scores, m=m, beta=beta, tanhs=tanhs, pre=pre,
                 rel_src=rel_src, rel_dst=rel_dst, n_dst=list(n_dst), w_type=w_type, a_src=a_src, a_dst=a_dst,
                 w_sem=ws, b_sem=bs, q_sem=q, bias=bias, relu=relu, heads=K)
    return h, cache


def rgat_layer_backward(cache, grad_h, relu_mask=None):
    """Reverse of `rgat_layer_forward`, step by step.  Returns a dict with dx (per type), dw_type, da_src,
    da_dst, dw_sem, db_sem, dq_sem, dbias (None where the parameter is None)."""
    x, z, nbrs, alphas, scores, m = (cache[k] for k in ("x", "z", "nbrs", "alphas", "scores", "m"))
    beta, tanhs, pre = cache["beta"], cache["tanhs"], cache["pre"]
    rel_src, rel_dst, n_dst = cache["rel_src"], cache["rel_dst"], cache["n_dst"]
    ws, bs, q, K = cache["w_sem"], cache["b_sem"], cache["q_sem"], cache["heads"]
    T, R = len(x), len(rel_src)
    H = z[0].shape[1]
    D = H // K
    gp = []
    for t in range(T):
        g = np.asarray(grad_h[t], dtype=F64).reshape(pre[t].shape)
        if not cache["relu"]:
            gp.append(g.copy())
        elif relu_mask is not None:
            gp.append(g * np.asarray(relu_mask[t], dtype=bool).reshape(pre[t].shape))
        else:
            gp.append(g * (pre[t] > 0))
    dbias = [None if cache["bias"][t] is None else gp[t].sum(axis=0) for t in range(T)]
    dws, dbs, dq = np.zeros_like(ws), np.zeros_like(bs), np.zeros_like(q)
    dm = [np.zeros_like(a) for a in m]
    for d in range(T):                                                       # fusion, reversed
        M = int(n_dst[d])
        Rd = [r for r in range(R) if rel_dst[r] == d]
        if M == 0 or not Rd:
            continue
        dbeta = np.array([(gp[d] * m[r]).sum() for r in Rd])
        b = np.array([beta[r] for r in Rd])
        dw = b * (dbeta - (b * dbeta).sum())                                 # softmax over relations
        for i, r in enumerate(Rd):
            dm[r] += b[i] * gp[d]
            t = tanhs[r]
            dq += dw[i] / M * t.sum(axis=0)
            du = (dw[i] / M) * q[None, :] * (1.0 - t * t)
            dws += m[r].T @ du
            dbs += du.sum(axis=0)
            dm[r] += du @ ws.T
    dz = [np.zeros_like(a) for a in z]
    da_src, da_dst = [], []
    for r in range(R):                                                       # aggregation, reversed
        s, d = rel_src[r], rel_dst[r]
        As, Ad = np.asarray(cache["a_src"][r], dtype=F64), np.asarray(cache["a_dst"][r], dtype=F64)
        das, dad = np.zeros_like(As), np.zeros_like(Ad)
        for v in range(int(n_dst[d])):
            nb = nbrs[r][v]
            if not nb:
                continue
            a, sv = alphas[r][v], scores[r][v]
            zu = z[s][nb].reshape(len(nb), K, D)
            zv = z[d][v].reshape(K, D)
            g = dm[r][v].reshape(K, D)
            dalpha = (zu * g[None]).sum(axis=2)                              # [n, K]
            np.add.at(dz[s], nb, (a[:, :, None] * g[None]).reshape(len(nb), H))
            de = a * (dalpha - (a * dalpha).sum(axis=0, keepdims=True))      # softmax over the neighbours
            ds = de * np.where(sv > 0, 1.0, LEAKY_SLOPE)                     # LeakyReLU
            das += (ds[:, :, None] * zu).sum(axis=0)
            dad += ds.sum(axis=0)[:, None] * zv
            np.add.at(dz[s], nb, (ds[:, :, None] * As[None]).reshape(len(nb), H))
            dz[d][v] += (ds.sum(axis=0)[:, None] * Ad).reshape(H)
        da_src.append(das); da_dst.append(dad)
    dw_type = [x[t].T @ dz[t] for t in range(T)]                             # projection, reversed
    dx = [dz[t] @ np.asarray(cache["w_type"][t], dtype=F64).T for t in range(T)]
    return dict(dx=dx, dw_type=dw_type, da_src=da_src, da_dst=da_dst, dw_sem=dws, db_sem=dbs, dq_sem=dq, dbias=dbias)


def softmax_xent(logits, labels):
    """Mean softmax cross-entropy over the rows and its gradient w.r.t. the logits."""
    z = np.asarray(logits, dtype=F64)
    n = z.shape[0]
    zs = z - z.max(axis=1, keepdims=True)
    lse = np.log(np.exp(zs).sum(axis=1))
    logp = zs - lse[:, None]
    loss = -logp[np.arange(n), labels].mean()
    g = np.exp(logp)
    g[np.arange(n), labels] -= 1.0
    return loss, g / n


# --------------------------------------------------------------------------- #
# Whole model: layers stacked, each layer's output rows are the next layer's input
# --------------------------------------------------------------------------- #
def rgcn_model_forward(x0, blocks_sel, rel_src, rel_dst, blocks_n_dst, layers):
    """Layers stacked: returns per-layer outputs `h` and the per-layer caches."""
    xs, caches, hs = [x0], [], []
    for l, lw in enumerate(layers):
        if "w_type" in lw:      # attention variant
            h, c = rgat_layer_forward(xs[-1], blocks_sel[l], rel_src, rel_dst, blocks_n_dst[l], lw["w_type"],
                                      lw["a_src"], lw["a_dst"], lw["w_sem"], lw["b_sem"], lw["q_sem"], lw["bias"],
                                      lw["relu"], lw["heads"])
        else:
            h, c = rgcn_layer_forward(xs[-1], blocks_sel[l], rel_src, rel_dst, blocks_n_dst[l],
                                      lw["w_rel"], lw["w_root"], lw["bias"], lw["relu"])
        caches.append(c); hs.append(h); xs.append(h)
    return dict(h=hs, caches=caches)


def rgcn_model_forward_backward(x0, blocks_sel, rel_src, rel_dst, blocks_n_dst, layers, loss,
                                labels=None, grad_out=None, target_type=0, forward=None, relu_masks=None,
                                num_types=None):
    """x0: per type first-layer input; blocks_sel[l]: per-relation selected edges of
    layer l; layers[l]: dict(w_rel, w_root, bias, relu) for the mean layer or dict(w_type, a_src, a_dst,
    w_sem, b_sem, q_sem, bias, relu, heads) for the attention layer.  loss: "xent" (mean softmax
    cross-entropy of the target type's last-layer rows) or "dot" (sum of grad_out*h).
    `forward` may carry the result of `rgcn_model_forward` (then it is not recomputed);
    `relu_masks[l]` is passed to layer l's backward.
    Returns dict with per-layer outputs, loss value and all gradients."""
    fw = forward if forward is not None else rgcn_model_forward(x0, blocks_sel, rel_src, rel_dst, blocks_n_dst, layers)
    hs, caches = fw["h"], fw["caches"]
    T = len(x0) if x0 is not None else num_types
    if loss == "xent":
        val, g_t = softmax_xent(hs[-1][target_type], labels)
        g = [np.zeros_like(h) for h in hs[-1]]
        g[target_type] = g_t
    else:
        g = [np.asarray(grad_out[t], dtype=F64) for t in range(T)]
        val = sum(float((g[t] * hs[-1][t]).sum()) for t in range(T))
    grads = [None] * len(layers)
    for l in reversed(range(len(layers))):
        mask = None if relu_masks is None else relu_masks[l]
        if "w_type" in layers[l]:
            grads[l] = rgat_layer_backward(caches[l], g, mask)
            dx = grads[l]["dx"]
        else:
            dx, dw_rel, dw_root, dbias = rgcn_layer_backward(caches[l], g, mask)
            grads[l] = dict(dw_rel=dw_rel, dw_root=dw_root, dbias=dbias, dx=dx)
        g = dx
    return dict(h=hs, loss=val, grads=grads, dx0=g, caches=caches)
