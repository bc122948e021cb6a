"""Shared driver of the GPU parity tests: runs one configuration through the C-ABI path and
through the CPU oracle on the same seeded inputs and compares every output."""
import time

import numpy as np

from oracle import hgnn_oracle as O
from workloads import make_config, build_graph, sample_minibatch, init_weights, bf16_round
from workloads.synth import default_target_type

TOL = {"f32": 1e-4, "bf16": 2e-2}   # relative, per tensor: max-abs over max|ref| and L2 over ||ref||


def rel_errors(got, ref):
    got = np.asarray(got, dtype=np.float64).ravel()
    ref = np.asarray(ref, dtype=np.float64).ravel()
    if ref.size == 0:
        return 0.0, 0.0
    d = got - ref
    return (float(np.abs(d).max() / max(np.abs(ref).max(), 1e-30)),
            float(np.linalg.norm(d) / max(np.linalg.norm(ref), 1e-30)))


def prepare_inputs(index, scale=1.0, batch=None, graph=None):
    cfg = make_config(index, scale=scale, batch=batch)
    g = build_graph(cfg) if graph is None else graph
    mb = sample_minibatch(cfg, g)
    ws = init_weights(cfg, g)
    if cfg.dtype == "bf16":                       # both sides start from the same bf16-representable values
        g.stores = [bf16_round(s) for s in g.stores]
        for lw in ws:
            lw.w_rel = [bf16_round(w) for w in lw.w_rel]
            lw.w_root = [None if w is None else bf16_round(w) for w in lw.w_root]
            lw.bias = [None if b is None else bf16_round(b) for b in lw.bias]
            if cfg.kind == "rgat":
                lw.w_type = [bf16_round(w) for w in lw.w_type]
                lw.a_src = [bf16_round(a) for a in lw.a_src]
                lw.a_dst = [bf16_round(a) for a in lw.a_dst]
                lw.w_sem, lw.b_sem, lw.q_sem = bf16_round(lw.w_sem), bf16_round(lw.b_sem), bf16_round(lw.q_sem)
        if mb.grad_out is not None:
            mb.grad_out = [bf16_round(x) for x in mb.grad_out]
    return cfg, g, mb, ws


def storage_precision_pre(cache, dtype, round_input):
    """Pre-activation of the mean layer with the aggregate of the raw neighbour features rounded to the storage
    type (bf16 or fp32) before the projection, everything else in fp64: the precision in which the kernel takes
    the ReLU decision.  `cache` is the oracle's forward cache of the layer; `round_input`: the layer's input is an
    activation of the previous layer, stored in the storage type as well."""
    rnd = (lambda a: bf16_round(np.asarray(a, dtype=np.float32)).astype(np.float64)) if dtype == "bf16" else \
          (lambda a: np.asarray(a, dtype=np.float32).astype(np.float64))
    x = [rnd(a) if round_input else a for a in cache["x"]]
    n_dst, rel_src, rel_dst = cache["n_dst"], cache["rel_src"], cache["rel_dst"]
    pre = []
    for t in range(len(x)):
        H = cache["pre"][t].shape[1]
        p = np.zeros((int(n_dst[t]), H))
        if n_dst[t] > 0:
            if cache["w_root"][t] is not None:
                p += x[t][: n_dst[t]] @ np.asarray(cache["w_root"][t], dtype=np.float64)
            if cache["bias"][t] is not None:
                p += np.asarray(cache["bias"][t], dtype=np.float64)[None, :]
        pre.append(p)
    for r in range(len(rel_src)):
        s_, d = rel_src[r], rel_dst[r]
        nb = cache["nbrs"][r]
        M = int(n_dst[d])
        if M == 0:
            continue
        # the stored aggregate, formed as the kernel forms it: neighbours added one after the other in fp32, in the
        # row's edge order, the sum multiplied by the fp32 reciprocal of the degree, the product rounded to storage
        xs32 = x[s_].astype(np.float32)
        deg = np.array([len(a) for a in nb], dtype=np.int64)
        acc = np.zeros((M, xs32.shape[1]), dtype=np.float32)
        for k in range(int(deg.max()) if M else 0):
            rows = np.nonzero(deg > k)[0]
            cols = np.fromiter((nb[v][k] for v in rows), dtype=np.int64, count=len(rows))
            acc[rows] = acc[rows] + xs32[cols]
        inv = np.zeros(M, dtype=np.float32)
        inv[deg > 0] = np.float32(1.0) / deg[deg > 0].astype(np.float32)
        z = rnd(acc * inv[:, None])
        pre[d] += z @ np.asarray(cache["w_rel"][r], dtype=np.float64)
    return pre


def layer_dicts(cfg, ws):
    if cfg.kind == "rgat":
        return [dict(w_type=lw.w_type, a_src=lw.a_src, a_dst=lw.a_dst, w_sem=lw.w_sem, b_sem=lw.b_sem, q_sem=lw.q_sem,
                     bias=lw.bias, relu=lw.relu, heads=cfg.heads) for lw in ws]
    return [dict(w_rel=lw.w_rel, w_root=lw.w_root, bias=lw.bias, relu=lw.relu) for lw in ws]


def oracle_run(cfg, g, mb, ws, input_grad=None):
    sch = g.schema
    blocks_x, _, _, flat = O.merge_features(g.stores, mb.ids)
    sels, csrs = [], []
    for b in mb.blocks:
        sel = O.edge_index_select(b.edge_index, sch.num_rels, edge_id=b.edge_id, global_edge_type=g.edge_type)
        sels.append(sel)
        csrs.append(O.semantic_csr(sel, sch.rel_src, sch.rel_dst, b.n_src, b.n_dst,
                                   transpose_types=input_grad if len(csrs) == 0 else None))
    layers = layer_dicts(cfg, ws)
    loss = "xent" if cfg.loss == "xent" else "dot"
    res = O.rgcn_model_forward_backward(blocks_x, sels, sch.rel_src, sch.rel_dst, [b.n_dst for b in mb.blocks],
                                        layers, loss, labels=mb.labels, grad_out=mb.grad_out,
                                        target_type=mb.target_type)
    res["csr"] = csrs
    res["x0_flat"] = flat
    return res


def run_case(index, scale=1.0, batch=None, verbose=False, use_edge_id=True, check_naive=False, graph=None,
             input_grad=None, backward=True, cfg_edit=None, grad_tol=None, sampled=None, need_input_grad=True,
             check_two_step=False, build_permutation=False):
    """cfg_edit(cfg, g, mb, ws): optional hook that changes the prepared inputs (e.g. the storage type) before
    both sides run.  grad_tol: optional {substring of a gradient's name: tolerance or None}; a matching
    gradient is held to that tolerance in both norms against the tie-broken oracle (None: reported only).
    sampled: optional dict(seed=..., fanouts=...): the mini-batch of the same targets is sampled by the library's
    sampler on the HIP side and by the sampler oracle on the other.  need_input_grad=False: the first layer's
    backward gets no input-gradient buffer (its weight and bias gradients are still checked)."""
    import torch
    from paper_2408_08490_amd.runner import Model
    cfg, g, mb, ws = prepare_inputs(index, scale, batch, graph)
    if cfg_edit is not None:
        cfg_edit(cfg, g, mb, ws)
    sch = g.schema
    if sampled is not None:
        from oracle import sampler_oracle as SO
        from workloads.synth import Block
        nt = mb.blocks[-1].n_dst[mb.target_type]
        targets = mb.ids[mb.target_type][:nt].copy()
        fanouts = sampled.get("fanouts", cfg.fanouts)
        smb = SO.sample_minibatch(g.num_nodes, sch.rel_src, sch.rel_dst, g.in_indptr, g.in_nbr, g.edge_off,
                                  mb.target_type, targets, fanouts, sampled["seed"])
        mb.ids = smb["ids"]
        mb.blocks = [Block(b["n_src"], b["n_dst"], b["edge_index"], b["edge_id"], b["edge_type"]) for b in smb["blocks"]]
    t0 = time.time()
    ref = oracle_run(cfg, g, mb, ws, input_grad)
    t_oracle = time.time() - t0
    model = Model(sch, g.feat_dim, g.stores, ws, dtype=cfg.dtype, loss=("xent" if cfg.loss == "xent" else "dot"),
                  target_type=mb.target_type, first_layer_input_grad=input_grad, build_permutation=build_permutation)
    if sampled is not None:
        sampler = model.ctx.hgnn_sampler_create(g.num_nodes, g.in_indptr, g.in_nbr, g.edge_off)
        bt = model.prepare_sampled(sampler, targets, fanouts, sampled["seed"], labels=mb.labels, grad_out=mb.grad_out)
    else:
        bt = model.prepare(mb, g.edge_type, use_edge_id=use_edge_id)
    out = model.run(bt, backward=backward, need_input_grad=need_input_grad)
    torch.cuda.synchronize()
    tol = TOL[cfg.dtype]
    report, ok = {}, True

    def chk(name, got, want, exact=False):
        nonlocal ok
        if exact:
            good = np.array_equal(np.asarray(got), np.asarray(want))
            report[name] = "exact" if good else "MISMATCH"
        else:
            e = rel_errors(got, want)
            good = e[0] <= tol and e[1] <= tol
            report[name] = (round(e[0], 7), round(e[1], 7))
        if not good:
            ok = False
            if verbose:
                print("FAIL", name, report[name], flush=True)

    # integer outputs: bit-exact
    for l in range(len(mb.blocks)):
        view = bt.graph.host_view(l)
        for k in ("rel_row_off", "rel_edge_off", "rowptr", "colidx", "perm", "cptr", "crow", "cperm"):
            if view[k] is None:      # perm / cperm of a build without the permutations (the mean layers' default)
                assert k in ("perm", "cperm") and not build_permutation
                continue
            chk(f"L{l}.{k}", view[k], ref["csr"][l][k], exact=True)
    want_ro = np.concatenate([[0], np.cumsum([len(i) for i in mb.ids])]).astype(np.int32)
    want_eo = np.concatenate([[0], np.cumsum([len(i) * f for i, f in zip(mb.ids, g.feat_dim)])]).astype(np.int64)
    chk("row_off", out["row_off"], want_ro, exact=True)
    chk("elem_off", out["elem_off"], want_eo, exact=True)
    chk("x_merged", out["x0"].float().cpu().numpy(), ref["x0_flat"].astype(np.float32), exact=True)
    # floating point outputs.  A ReLU's backward needs a decision (unit active or not) that floating point takes;
    # both sides take it in the same precision, the kernel's: the mean layer keeps the aggregate of the raw
    # neighbour features in the storage type before it is projected, so the decision is taken on
    #   pre_k = x_v W_0 + b + sum_r round_storage(mean_u x_u) W_r
    # evaluated here in fp64 from the oracle's own inputs (`storage_precision_pre`).  The kernel accumulates the same
    # products in fp32, so its decision may still differ where pre_k is zero to within that rounding
    # (|pre_k| < AMBIG * rms): there the kernel's decision is taken over, after checking that it agrees everywhere
    # else.  The oracle's backward then runs with those decisions; forward values are compared with the plain oracle.
    AMBIG = {"f32": 1e-5, "bf16": 1e-4}[cfg.dtype]
    amb_max_frac = 1e-3
    if cfg.kind == "rgat" and cfg.dtype == "bf16":
        # the attention layer stores the projected features z and the per-relation aggregates m in bf16 (they are
        # gathered per edge, so their width is the layer's memory traffic): the pre-activation carries their
        # rounding, ~2^-8 of its scale, and a unit inside that band may take either decision
        AMBIG, amb_max_frac = 2.0 ** -7, 3e-2
    masks, n_amb, n_units = [], 0, 0
    for l in range(len(ws)):
        if not ws[l].relu:
            masks.append(None)
            continue
        hg = out["h"][l].float().cpu().numpy().reshape(-1, ws[l].out_dim)
        pre_k = ref["caches"][l]["pre"] if cfg.kind == "rgat" else storage_precision_pre(ref["caches"][l], cfg.dtype, l > 0)
        ml, r0 = [], 0
        for t in range(sch.num_types):
            pre = pre_k[t]
            hgt = hg[r0: r0 + pre.shape[0]]
            r0 += pre.shape[0]
            if pre.size == 0:
                ml.append(np.zeros(pre.shape, bool))
                continue
            amb = np.abs(pre) < AMBIG * np.sqrt(np.mean(pre * pre))
            if not np.array_equal((hgt > 0)[~amb], (pre > 0)[~amb]):
                ok = False
                report[f"L{l}.relu_decisions_type{t}"] = "MISMATCH"
            ml.append(np.where(amb, hgt > 0, pre > 0))
            n_amb += int(amb.sum()); n_units += amb.size
        masks.append(ml)
    report["ambiguous_relu_units"] = (n_amb, n_units)
    if n_units and n_amb > amb_max_frac * n_units:
        ok = False
    ref_tb = ref
    if any(m is not None for m in masks):
        layers = layer_dicts(cfg, ws)
        ref_tb = O.rgcn_model_forward_backward(None, None, sch.rel_src, sch.rel_dst, None, layers,
                                               "xent" if cfg.loss == "xent" else "dot", labels=mb.labels,
                                               grad_out=mb.grad_out, target_type=mb.target_type,
                                               forward=dict(h=ref["h"], caches=ref["caches"]), relu_masks=masks,
                                               num_types=sch.num_types)

    def chk2(name, got, want_plain, want_tb):
        nonlocal ok
        e_plain, e_tb = rel_errors(got, want_plain), rel_errors(got, want_tb)
        good = e_tb[0] <= tol and e_tb[1] <= tol     # against the oracle with the decisions of the storage precision
        for key, t2 in (grad_tol or {}).items():
            if key in name:
                good = True if t2 is None else (e_tb[0] <= t2 and e_tb[1] <= t2)
        report[name] = (round(e_tb[0], 7), round(e_plain[1], 7))
        if not good:
            ok = False
            if verbose:
                print("FAIL", name, "plain", e_plain, "tie-broken", e_tb, flush=True)

    for l in range(len(ws)):
        want = np.concatenate([h.ravel() for h in ref["h"][l]])
        chk(f"L{l}.h", out["h"][l].float().cpu().numpy(), want)
        if not backward:
            continue
        gr, gt, w = ref["grads"][l], ref_tb["grads"][l], model.weights[l]
        if cfg.kind == "rgat":
            for t in range(sch.num_types):
                chk2(f"L{l}.dw_type{t}", w["dattn"]["dw_type"][t].cpu().numpy(), gr["dw_type"][t], gt["dw_type"][t])
                if gr["dbias"][t] is not None:
                    chk2(f"L{l}.dbias{t}", w["dbias"][t].cpu().numpy(), gr["dbias"][t], gt["dbias"][t])
            for r in range(sch.num_rels):
                chk2(f"L{l}.da_src{r}", w["dattn"]["da_src"][r].cpu().numpy(), gr["da_src"][r], gt["da_src"][r])
                chk2(f"L{l}.da_dst{r}", w["dattn"]["da_dst"][r].cpu().numpy(), gr["da_dst"][r], gt["da_dst"][r])
            for k in ("dw_sem", "db_sem", "dq_sem"):
                chk2(f"L{l}.{k}", w["dattn"][k].cpu().numpy(), gr[k], gt[k])
        else:
            for r in range(sch.num_rels):
                chk2(f"L{l}.dw_rel{r}", w["dw_rel"][r].cpu().numpy(), gr["dw_rel"][r], gt["dw_rel"][r])
            for t in range(sch.num_types):
                if gr["dw_root"][t] is not None:
                    chk2(f"L{l}.dw_root{t}", w["dw_root"][t].cpu().numpy(), gr["dw_root"][t], gt["dw_root"][t])
                if gr["dbias"][t] is not None:
                    chk2(f"L{l}.dbias{t}", w["dbias"][t].cpu().numpy(), gr["dbias"][t], gt["dbias"][t])
        if out["dx"][l] is None:
            assert l == 0 and not need_input_grad
            continue
        got_dx = out["dx"][l].float().cpu().numpy()
        if l == 0 and input_grad is not None:          # rows of types without input gradients are left unwritten
            eo = np.concatenate([[0], np.cumsum([d.size for d in gr["dx"]])])
            keep = [t for t in range(sch.num_types) if input_grad[t]]
            chk2(f"L{l}.dx", np.concatenate([got_dx[eo[t]: eo[t + 1]] for t in keep]),
                 np.concatenate([gr["dx"][t].ravel() for t in keep]), np.concatenate([gt["dx"][t].ravel() for t in keep]))
        else:
            chk2(f"L{l}.dx", got_dx, np.concatenate([d.ravel() for d in gr["dx"]]),
                 np.concatenate([d.ravel() for d in gt["dx"]]))
    if cfg.loss == "xent":
        chk("loss", out["loss"].cpu().numpy(), np.array([ref["loss"]]))
    if check_naive:
        out2 = model.run(bt, backward=False, naive=True)
        torch.cuda.synchronize()
        for l in range(len(ws)):
            want = np.concatenate([h.ravel() for h in ref["h"][l]])
            chk(f"L{l}.h_naive", out2["h"][l].float().cpu().numpy(), want)
        report["naive_launches"] = out2["launches"]
        report["merged_launches"] = [model.ctx.hgnn_layer_launch_count(bt.graph, l, model.layers[l])
                                     for l in range(len(ws))]
    if check_two_step:
        # Algorithm 1 in its two stated steps (FeatureCat, then reduce): against the oracle like the fused path,
        # and bit for bit against the fused path's outputs
        fused = [h.clone() for h in out["h"]]
        out3 = model.run(bt, backward=False, two_step=True)
        torch.cuda.synchronize()
        for l in range(len(ws)):
            want = np.concatenate([h.ravel() for h in ref["h"][l]])
            chk(f"L{l}.h_two_step", out3["h"][l].float().cpu().numpy(), want)
            chk(f"L{l}.h_two_step_bits", out3["h"][l].view(torch.uint8).cpu().numpy(), fused[l].view(torch.uint8).cpu().numpy(),
                exact=True)
        report["two_step_launches"] = out3["launches"]
    bt.graph.release()
    model.close()
    report["ok"] = ok
    report["oracle_s"] = round(t_oracle, 3)
    report["sizes"] = [(sum(b.n_src), sum(b.n_dst), int(b.edge_index.shape[1])) for b in mb.blocks]
    if verbose:
        print({k: v for k, v in report.items() if not k.startswith("L")}, flush=True)
        worst = sorted(((v[0], k) for k, v in report.items() if isinstance(v, tuple) and len(v) == 2
                        and isinstance(v[0], float)), reverse=True)[:6]
        print("worst:", worst, flush=True)
        print("all:", {k: v for k, v in report.items() if isinstance(v, tuple) and len(v) == 2}, flush=True)
    return report


def train_case(index, scale=1.0, batch=None, steps=3, input_grad=None, verbose=False):
    """`steps` training steps (forward, loss, backward, Adam on every weight and on the embedding rows the
    mini-batch read) on one mini-batch: the C-ABI path against the same steps taken with the model oracle and the
    optimiser oracle.  Returns the losses of both sides and the relative rms distance of every updated tensor."""
    import torch
    from oracle import optim_oracle as P
    from paper_2408_08490_amd.runner import Model
    cfg, g, mb, ws = prepare_inputs(index, scale, batch)
    assert cfg.kind == "rgcn" and cfg.loss == "xent"
    sch = g.schema
    hp = {k: float(np.float32(x)) for k, x in dict(lr=1e-2, beta1=0.9, beta2=0.999, eps=1e-8).items()}
    model = Model(sch, g.feat_dim, g.stores, ws, dtype=cfg.dtype, loss="xent", target_type=mb.target_type,
                  first_layer_input_grad=input_grad)
    model.enable_training(**hp)
    bt = model.prepare(mb, g.edge_type, use_edge_id=True)
    got_loss = []
    for _ in range(steps):
        out = model.run(bt)
        got_loss.append(float(out["loss"].item()))
        model.optimizer_step(bt, out)
    torch.cuda.synchronize()
    # the oracle's loop
    learn = [t for t in range(sch.num_types) if input_grad is None or input_grad[t]]
    stores = [np.asarray(s, dtype=np.float64).copy() for s in g.stores]
    layers = layer_dicts(cfg, ws)
    for lw in layers:
        lw["w_rel"] = [np.asarray(w, np.float64) for w in lw["w_rel"]]
        lw["w_root"] = [None if w is None else np.asarray(w, np.float64) for w in lw["w_root"]]
        lw["bias"] = [None if b is None else np.asarray(b, np.float64) for b in lw["bias"]]
    mom = {}
    sels = [O.edge_index_select(b.edge_index, sch.num_rels, edge_id=b.edge_id, global_edge_type=g.edge_type)
            for b in mb.blocks]
    want_loss = []

    def upd(key, theta, grad, step):
        m, v = mom.get(key, (np.zeros_like(theta), np.zeros_like(theta)))
        theta, m, v = P.adam_step(theta, grad, m, v, step, **hp)
        mom[key] = (m, v)
        return theta

    for step in range(1, steps + 1):
        blocks_x, _, _, _ = O.merge_features(stores, mb.ids)
        res = O.rgcn_model_forward_backward(blocks_x, sels, sch.rel_src, sch.rel_dst, [b.n_dst for b in mb.blocks],
                                            layers, "xent", labels=mb.labels, grad_out=None, target_type=mb.target_type)
        want_loss.append(float(res["loss"]))
        for l, lw in enumerate(layers):
            gr = res["grads"][l]
            lw["w_rel"] = [upd((l, "r", r), w, gr["dw_rel"][r], step) for r, w in enumerate(lw["w_rel"])]
            lw["w_root"] = [None if w is None else upd((l, "0", t), w, gr["dw_root"][t], step) for t, w in enumerate(lw["w_root"])]
            lw["bias"] = [None if b is None else upd((l, "b", t), b, gr["dbias"][t], step) for t, b in enumerate(lw["bias"])]
        for t in learn:
            if len(mb.ids[t]) == 0:
                continue
            m, v = mom.get(("e", t), (np.zeros_like(stores[t]), np.zeros_like(stores[t])))
            stores[t], m, v = P.adam_rows_step(stores[t], mb.ids[t], res["dx0"][t], m, v, step, **hp)
            mom[("e", t)] = (m, v)

    def dist(got, want):
        want = np.asarray(want, np.float64)
        return float(np.sqrt(np.mean((np.asarray(got, np.float64) - want) ** 2)) / max(np.sqrt(np.mean(want ** 2)), 1e-30))

    dists = {}
    for l, (lw, w) in enumerate(zip(layers, model.weights)):
        for r in range(sch.num_rels):
            dists[f"L{l}.w_rel{r}"] = dist(w["w_rel"][r].float().cpu().numpy(), lw["w_rel"][r])
        for t in range(sch.num_types):
            if lw["w_root"][t] is not None:
                dists[f"L{l}.w_root{t}"] = dist(w["w_root"][t].float().cpu().numpy(), lw["w_root"][t])
            if lw["bias"][t] is not None:
                dists[f"L{l}.bias{t}"] = dist(w["bias"][t].float().cpu().numpy(), lw["bias"][t])
    for t in learn:
        if len(mb.ids[t]):
            dists[f"emb{t}"] = dist(model.stores[t][torch.from_numpy(mb.ids[t]).to(model.dev)].float().cpu().numpy(),
                                    stores[t][mb.ids[t]])
    for t in range(sch.num_types):
        if t not in learn:   # fixed features are never written
            assert np.array_equal(model.stores[t].float().cpu().numpy(), np.asarray(g.stores[t], np.float32))
    model.close()
    if verbose:
        print("losses", got_loss, want_loss, "max dist", max(dists.values()), flush=True)
    return dict(got_loss=got_loss, want_loss=want_loss, dists=dists)
