"""Drives the C-ABI entry points over one mini-batch: buffers and call order only.

Used by the GPU tests, the smoke check and bench.py.  All arithmetic happens in
libhgnn.so; PyTorch provides device memory and the stream.
"""
from __future__ import annotations

from typing import List, Optional

import numpy as np
import torch

from . import binding as B


def _tdtype(name):
    return torch.bfloat16 if name == "bf16" else torch.float32


def to_device(a: np.ndarray, dtype: str, dev) -> torch.Tensor:
    """float32 host array -> device tensor of the path's storage type (values must already be
    representable when dtype is bf16, so the conversion is exact)."""
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(dev).to(_tdtype(dtype)).contiguous()


class Batch:
    def __init__(self):
        self.ids_dev = None
        self.graph = None
        self.labels_dev = None
        self.grad_out_dev = None
        self.blocks = None
        self.n_rows = None
        self.sampled = False


class _DevIds:
    """Device id list that lives in a graph's buffers (what hgnn_merge_features needs of a tensor)."""

    def __init__(self, ptr, n):
        self._ptr, self._n = ptr, n

    def data_ptr(self):
        return self._ptr

    def numel(self):
        return self._n


class _Sizes:
    def __init__(self, n_src, n_dst):
        self.n_src, self.n_dst = n_src, n_dst


class Model:
    """Weights, feature stores and work buffers of one configuration on one GPU."""

    def __init__(self, schema, feat_dim, stores, layers, dtype="f32", loss="xent", target_type=0, device=0,
                 host_threads=0, first_layer_input_grad=None, concurrent_builds=0, build_permutation=False):
        """first_layer_input_grad: per type 0/1, which vertex types need gradients w.r.t. their input
        features in the first layer (learnable embeddings); None = all.
        build_permutation: whether the index build also writes perm / cperm, which the mean layers never read
        (the attention variant always gets them)."""
        self.dev = torch.device("cuda", device)
        torch.cuda.set_device(self.dev)
        self.dtype, self.loss, self.target_type = dtype, loss, target_type
        self.first_layer_input_grad = first_layer_input_grad
        self.T, self.R = schema.num_types, schema.num_rels
        self.attention = bool(layers) and len(getattr(layers[0], "w_type", []) or []) > 0
        heads = 1
        if self.attention:
            heads = int(layers[0].a_src[0].shape[0])
        self.ctx = B.Context(schema.rel_src, schema.rel_dst, schema.num_types, dtype, device, host_threads, concurrent_builds,
                             heads=heads, attention=self.attention)
        self.ctx.hgnn_set_build_permutation(bool(build_permutation))
        self.feat_dim = list(feat_dim)
        self.stores = [to_device(s, dtype, self.dev) for s in stores]
        self.layers: List[B.Layer] = []
        self.weights = []
        for lw in layers:
            if self.attention:
                f32 = dict(device=self.dev, dtype=torch.float32)
                dev = lambda a: to_device(a, dtype, self.dev)
                attn = dict(w_type=[dev(w) for w in lw.w_type], a_src=[dev(a) for a in lw.a_src], a_dst=[dev(a) for a in lw.a_dst],
                            w_sem=dev(lw.w_sem), b_sem=dev(lw.b_sem), q_sem=dev(lw.q_sem))
                bias = [None if b is None else dev(b) for b in lw.bias]
                dattn = dict(dw_type=[torch.empty(w.shape, **f32) for w in attn["w_type"]],
                             da_src=[torch.empty(a.shape, **f32) for a in attn["a_src"]],
                             da_dst=[torch.empty(a.shape, **f32) for a in attn["a_dst"]],
                             dw_sem=torch.empty(attn["w_sem"].shape, **f32), db_sem=torch.empty(attn["b_sem"].shape, **f32),
                             dq_sem=torch.empty(attn["q_sem"].shape, **f32))
                dbias = [None if b is None else torch.empty(b.shape, **f32) for b in bias]
                self.weights.append(dict(attn=attn, dattn=dattn, bias=bias, dbias=dbias))
                self.layers.append(B.Layer(self.ctx, lw.in_dim, lw.out_dim, lw.relu, None, None, bias, None, None, dbias,
                                           attn=attn, dattn=dattn))
                continue
            w_rel = [to_device(w, dtype, self.dev) for w in lw.w_rel]
            w_root = [None if w is None else to_device(w, dtype, self.dev) for w in lw.w_root]
            bias = [None if b is None else to_device(b, dtype, self.dev) for b in lw.bias]
            f32 = dict(device=self.dev, dtype=torch.float32)
            dw_rel = [torch.empty(w.shape, **f32) for w in w_rel]
            dw_root = [None if w is None else torch.empty(w.shape, **f32) for w in w_root]
            dbias = [None if b is None else torch.empty(b.shape, **f32) for b in bias]
            self.weights.append(dict(w_rel=w_rel, w_root=w_root, bias=bias, dw_rel=dw_rel, dw_root=dw_root, dbias=dbias))
            self.layers.append(B.Layer(self.ctx, lw.in_dim, lw.out_dim, lw.relu, w_rel, w_root, bias, dw_rel, dw_root, dbias,
                                       input_grad=first_layer_input_grad if not self.layers else None))
        self.loss_dev = torch.zeros(1, device=self.dev, dtype=torch.float32)
        self._buf = {}
        # default of run(gather=...): the first layer's aggregation reads the feature stores directly
        self.gather = False

    # ---- training: fp32 master copies and Adam moments of every weight and of the learnable embedding tables ----
    def enable_training(self, lr=1e-2, beta1=0.9, beta2=0.999, eps=1e-8, learnable_types=None):
        """learnable_types: vertex types whose feature store is an embedding table to be trained (default: the
        types whose first-layer input gradient is computed)."""
        f32 = dict(device=self.dev, dtype=torch.float32)
        params, grads = [], []
        for w in self.weights:
            if self.attention:
                a, d = w["attn"], w["dattn"]
                params += a["w_type"] + a["a_src"] + a["a_dst"] + [a["w_sem"], a["b_sem"], a["q_sem"]]
                grads += d["dw_type"] + d["da_src"] + d["da_dst"] + [d["dw_sem"], d["db_sem"], d["dq_sem"]]
            else:
                params += w["w_rel"] + [x for x in w["w_root"] if x is not None]
                grads += w["dw_rel"] + [x for x in w["dw_root"] if x is not None]
            params += [x for x in w["bias"] if x is not None]
            grads += [x for x in w["dbias"] if x is not None]
        masters = None if self.dtype == "f32" else [p.float() for p in params]
        ms, vs = [torch.zeros(p.shape, **f32) for p in params], [torch.zeros(p.shape, **f32) for p in params]
        self.adam = dict(lr=lr, beta1=beta1, beta2=beta2, eps=eps, step=0, params=params, masters=masters, m=ms, v=vs,
                         list=self.ctx.AdamList(params, masters, grads, ms, vs))
        if learnable_types is None:
            g = self.first_layer_input_grad
            learnable_types = [] if g is None else [t for t in range(self.T) if g[t]]
        self.emb = {}
        for t in learnable_types:
            st = self.stores[t]
            self.emb[t] = dict(master=None if self.dtype == "f32" else st.float(), m=torch.zeros(st.shape, **f32),
                               v=torch.zeros(st.shape, **f32))

    def optimizer_step(self, b: Batch, out):
        """Adam on all weights (one launch) and on the embedding rows this mini-batch read (one launch per type)."""
        a = self.adam
        a["step"] += 1
        hp = (a["lr"], a["beta1"], a["beta2"], a["eps"], a["step"])
        self.ctx.hgnn_adam_update(a["list"], *hp)
        dx, off = out["dx"][0], 0
        for t in range(self.T):
            n, F = b.n_rows[t], self.feat_dim[t]
            if t in self.emb and n > 0:
                e = self.emb[t]
                self.ctx.hgnn_adam_update_rows(self.stores[t], e["master"], e["m"], e["v"], b.ids_dev[t],
                                               dx[off: off + n * F], *hp)
            off += n * F

    def transpose_types(self, num_layers):
        """Per layer: which vertex types need transpose entries (the first layer skips the types whose input
        gradient is not wanted)."""
        if self.first_layer_input_grad is None or self.attention:
            return None
        return [list(self.first_layer_input_grad)] + [None] * (num_layers - 1)

    def close(self):
        self.ctx.close()

    def _get(self, name, nbytes):
        t = self._buf.get(name)
        if t is None or t.numel() < nbytes:
            t = torch.empty(max(nbytes, 256), device=self.dev, dtype=torch.uint8)
            self._buf[name] = t
        return t

    def _typed(self, name, numel):
        es = 2 if self.dtype == "bf16" else 4
        raw = self._get(name, numel * es)
        return raw[: numel * es].view(_tdtype(self.dtype))

    # ---- host side of a step: upload ids / labels, start the semantic graph build ----
    def prepare(self, mb, global_edge_type=None, use_edge_id=False, device_build=False) -> Batch:
        b = Batch()
        b.ids_dev = [torch.from_numpy(np.ascontiguousarray(i, dtype=np.int64)).to(self.dev) for i in mb.ids]
        b.n_rows = [len(i) for i in mb.ids]
        b.blocks = mb.blocks
        b.graph = self.ctx.hgnn_build_semantic_csr(mb.blocks, global_edge_type, use_edge_id, self.transpose_types(len(mb.blocks)),
                                                   on_device=device_build)
        if mb.labels is not None:
            b.labels_dev = torch.from_numpy(mb.labels.astype(np.int64)).to(self.dev)
        if mb.grad_out is not None:
            b.grad_out_dev = to_device(np.concatenate([g.reshape(-1) for g in mb.grad_out]), self.dtype, self.dev)
        return b

    def prepare_sampled(self, sampler, targets, fanouts, seed, labels=None, grad_out=None) -> Batch:
        """The mini-batch is sampled by the library's host threads (then built and uploaded, all one task)."""
        b = Batch()
        b.sampled = True
        b.graph = self.ctx.hgnn_sample_and_build(sampler, self.target_type, targets, fanouts, seed,
                                                 self.transpose_types(len(fanouts)))
        if labels is not None:
            b.labels_dev = labels if torch.is_tensor(labels) else torch.from_numpy(np.asarray(labels, np.int64)).to(self.dev)
        if grad_out is not None:
            b.grad_out_dev = to_device(np.concatenate([g.reshape(-1) for g in grad_out]), self.dtype, self.dev)
        return b

    def _resolve_sampled(self, b: Batch):
        """Sizes and device id lists of a sampled mini-batch (waits for its host task) and the stream dependency
        of the merge on the upload."""
        n_rows, _, dptr = b.graph.ids(device=True)
        b.n_rows = n_rows
        b.ids_dev = [_DevIds(p, n) for p, n in zip(dptr, n_rows)]
        b.blocks = [_Sizes(**b.graph.minibatch_view(l, arrays=False)) for l in range(len(self.layers))]
        b.graph.wait_stream()

    # ---- device side of a step ----
    def run(self, b: Batch, backward=True, naive=False, need_input_grad=True, two_step=False, layer_inputs=None,
            layer_grads=None, gather=None):
        """gather=True: the first layer's aggregation reads the feature stores directly (hgnn_layer_fwd_gather) and the
        feature merge copies the destination rows only.
        layer_inputs[l] (l >= 1) / layer_grads[l]: optional device tensors that take the place of layer l's input
        (the previous layer's output) and of its incoming gradient (the next layer's input gradient, or the loss
        gradient): every layer then runs on given tensors instead of its neighbour's results."""
        ctx, L = self.ctx, len(self.layers)
        gather = self.gather if gather is None else gather
        # the per-relation launch loop and the two-step aggregation read the fully merged input
        gather = bool(gather) and not naive and not two_step and not self.attention
        if b.sampled and b.ids_dev is None:
            self._resolve_sampled(b)
        if gather:
            nd0 = list(b.blocks[0].n_dst)
            x = self._typed("x0dst", sum(n * f for n, f in zip(nd0, self.feat_dim)))
            row_off, elem_off = ctx.hgnn_merge_features(self.stores, b.ids_dev, x, self.feat_dim, n_rows=nd0)
        else:
            n0 = sum(n * f for n, f in zip(b.n_rows, self.feat_dim))
            x = self._typed("x0", n0)
            row_off, elem_off = ctx.hgnn_merge_features(self.stores, b.ids_dev, x, self.feat_dim)
        xs, hs, saved = [x], [], []
        launches = []
        for l, lp in enumerate(self.layers):
            blk = b.blocks[l]
            if layer_inputs is not None and layer_inputs[l] is not None:
                xs[-1] = layer_inputs[l]
            sb, cb = ctx.hgnn_layer_workspace_bytes(b.graph, l, lp)
            sv = self._get(f"saved{l}", sb)
            sc = self._get("scratch", cb)
            h = self._typed(f"h{l}", sum(blk.n_dst) * lp.out_dim)
            if two_step:     # the materialising form of the aggregation (FeatureCat, then reduce)
                fc = self._typed("feature_cat", max(1, b.graph.num_edges(l)) * max(lp.in_dim))
                launches.append(ctx.hgnn_layer_fwd_two_step(b.graph, l, lp, xs[-1], h, sv, sc, fc))
            elif naive:
                launches.append(ctx.hgnn_layer_fwd_naive(b.graph, l, lp, xs[-1], h, sv, sc))
            elif gather and l == 0:
                ctx.hgnn_layer_fwd_gather(b.graph, l, lp, self.stores, b.ids_dev, xs[-1], h, sv, sc)
            else:
                ctx.hgnn_layer_fwd(b.graph, l, lp, xs[-1], h, sv, sc)
            hs.append(h); saved.append(sv); xs.append(h)
        out = dict(x0=x, h=hs, row_off=row_off, elem_off=elem_off, launches=launches)
        blk = b.blocks[-1]
        H = self.layers[-1].out_dim
        if self.loss == "xent":
            t = self.target_type
            r0 = sum(blk.n_dst[:t])
            logits = hs[-1].view(-1, H)[r0: r0 + blk.n_dst[t]]
            g = self._typed("g_last", sum(blk.n_dst) * H)
            if sum(blk.n_dst) != blk.n_dst[t]:   # rows of other types get no loss gradient
                g.zero_()
            gv = g.view(-1, H)[r0: r0 + blk.n_dst[t]]
            ctx.hgnn_softmax_xent(logits, b.labels_dev, self.loss_dev, gv)
            out["loss"] = self.loss_dev
        else:
            g = b.grad_out_dev
        out["g_last"] = g
        if not backward:
            return out
        dxs = [None] * L
        launches_bwd = [0] * L
        for l in reversed(range(L)):
            lp = self.layers[l]
            blk = b.blocks[l]
            sb, cb = ctx.hgnn_layer_workspace_bytes(b.graph, l, lp)
            sc = self._get("scratch", cb)
            want_dx = need_input_grad or l > 0
            if layer_grads is not None and layer_grads[l] is not None:
                g = layer_grads[l]
            dx = self._typed(f"dx{l}", sum(n * f for n, f in zip(blk.n_src, lp.in_dim))) if want_dx else None
            if naive and not self.attention:
                launches_bwd[l] = ctx.hgnn_layer_bwd_naive(b.graph, l, lp, xs[l], hs[l], saved[l], g, dx, sc)
            elif gather and l == 0:
                ctx.hgnn_layer_bwd_gather(b.graph, l, lp, xs[l], hs[l], saved[l], g, dx, sc)
            else:
                ctx.hgnn_layer_bwd(b.graph, l, lp, xs[l], hs[l], saved[l], g, dx, sc)
            dxs[l] = dx
            g = dx
        out["dx"] = dxs
        out["launches_bwd"] = launches_bwd
        return out
