#!/usr/bin/env python3
"""Benchmark of the merged HGNN layer path on one MI355X.

A "step" is one pass of the whole hot path over one pre-sampled synthetic mini-batch of the
headline workload (4-type / 8-relation academic-shaped graph, bf16, hidden 512, 4096 targets,
fanout [25, 20], 2 R-GCN layers 128 -> 512 -> 349, cross-entropy): type-first feature merge,
host semantic-CSR build (running on host threads and uploaded on a side stream while the GPU
works on the previous mini-batch), both layers forward, loss, both layers backward.

Prints ONE JSON line.  `value` is mini-batches/s of the pipelined loop; `gpu_only_mb_per_s` is
the same loop with the index arrays built beforehand.  `roofline` is for the dominant kernel,
timed with HIP event pairs inside the timed loop; `cpu_baseline` is the CPU oracle on a bounded
sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic_config2_bf16.txt")


def traffic_bytes():
    """HBM bytes per launch of the probed kernels on the default workload: the `traffic_bytes <kernel> <bytes>` lines of
    the rocprofv3 --pmc summary under profiles/ (FETCH_SIZE + WRITE_SIZE, scaled by the copy-kernel calibration stated
    there).  A kernel without such a line, or a missing file, reads as None (not measured)."""
    out = {}
    try:
        for line in open(TRAFFIC_FILE):
            f = line.split()
            if len(f) == 3 and f[0] == "traffic_bytes":
                out[f[1]] = float(f[2])
    except OSError:
        pass
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=2)
    ap.add_argument("--scale", type=float, default=1.0)
    ap.add_argument("--batches", type=int, default=4, help="distinct pre-sampled mini-batches cycled through")
    ap.add_argument("--probe", default="auto", help="kernel bracketed with HIP events for the roofline object "
                    "(auto: forward GEMM and gather-mean of layer 1)")
    ap.add_argument("--probe-layer", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sampler-loop", action="store_true", help="skip the run with the sampler in the loop")
    ap.add_argument("--no-train-loop", action="store_true", help="skip the run with the parameter update in the step")
    ap.add_argument("--ablation", action="store_true",
                    help="time the switchable pieces (the paper's Fig. 9 analogue: per-relation launch loop vs merged "
                         "launches, two-step vs fused aggregation, serial vs overlapped host build) over K/4 steps "
                         "instead of the 20 of the default line")
    ap.add_argument("--no-ablation", action="store_true", help="leave the ablation object out")
    ap.add_argument("--cpu-sample-batch", type=int, default=4096)
    ap.add_argument("--host-threads", type=int, default=0)
    ap.add_argument("--gather-from-stores", action="store_true",
                    help="merge the destination rows only and let the first layer's aggregation read the feature stores "
                         "(hgnn_layer_fwd_gather) instead of merging every source row into x_merged (hgnn_layer_fwd); the "
                         "default line times the other one of the two in its ablation object")
    ap.add_argument("--all-input-grads", action="store_true", help="also compute gradients w.r.t. the fixed T0 features")
    ap.add_argument("--calibrate", action="store_true",
                    help="also launch the merge kernel as a plain copy of known size (2^20 rows x 128, identity ids) "
                         "three times: reference for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE readings")
    ap.add_argument("--host-warmup-s", type=float, default=3.0,
                    help="seconds of further untimed pipelined steps after the W warm-up steps (0 with --warmup 0)")
    ap.add_argument("--build-permutation", action="store_true",
                    help="the index build also writes perm / cperm (input position of every CSR / transpose entry), which "
                         "the mean layers never read; the attention variant always gets them")
    ap.add_argument("--lookahead", type=int, default=24, help="mini-batches whose index build is started ahead of the GPU")
    ap.add_argument("--concurrent-builds", type=int, default=15,
                    help="host builders working on separate mini-batches at once (the host threads are split over them; "
                         "0: the library's low-latency default)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from workloads import make_config, build_graph, sample_minibatch, init_weights, bf16_round
    from workloads.synth import MASTER_SEED
    from paper_2408_08490_amd.runner import Model
    from paper_2408_08490_amd import binding as B

    t0 = time.time()
    cfg = make_config(args.config, scale=args.scale)
    g = build_graph(cfg)
    ws = init_weights(cfg, g)
    if cfg.dtype == "bf16":
        g.stores = [bf16_round(s) for s in g.stores]
        for lw in ws:
            lw.w_rel = [bf16_round(w) for w in lw.w_rel]
            lw.w_root = [None if w is None else bf16_round(w) for w in lw.w_root]
            lw.bias = [None if b is None else bf16_round(b) for b in lw.bias]
    mbs = [sample_minibatch(cfg, g, rng=np.random.default_rng([MASTER_SEED + cfg.index, 1000 + i]))
           for i in range(args.batches)]
    for mb in mbs:
        if mb.grad_out is not None and cfg.dtype == "bf16":
            mb.grad_out = [bf16_round(x) for x in mb.grad_out]
    t_setup = time.time() - t0

    model = Model(g.schema, g.feat_dim, g.stores, ws, dtype=cfg.dtype,
                  loss=("xent" if cfg.loss == "xent" else "dot"), target_type=mbs[0].target_type,
                  host_threads=args.host_threads or args.concurrent_builds, concurrent_builds=args.concurrent_builds,
                  build_permutation=args.build_permutation,
                  # T0 carries fixed input features; only the learnable embeddings of T1-T3 need input gradients
                  first_layer_input_grad=([0, 1, 1, 1] if cfg.index in (1, 2, 4) and not args.all_input_grads else None))
    ctx = model.ctx
    # first layer: the full feature merge by default.  Reading the stores directly saves the merge's copy (~34 us on the
    # default workload) but the gather then walks tables of GBs instead of a compact 100 MB buffer and takes ~20 us
    # longer; with the address pass the step comes out even.
    model.gather = args.gather_from_stores and cfg.kind != "rgat" and len(set(g.feat_dim)) == 1

    # inputs resident in HBM before the timed region: stores, weights, per-mini-batch id lists and labels
    class Slot:
        pass
    slots = []
    for mb in mbs:
        s = Slot()
        s.mb = mb
        s.ids_dev = [torch.from_numpy(np.ascontiguousarray(i, dtype=np.int64)).to(model.dev) for i in mb.ids]
        s.labels_dev = None if mb.labels is None else torch.from_numpy(mb.labels.astype(np.int64)).to(model.dev)
        s.grad_out_dev = None
        if mb.grad_out is not None:
            from paper_2408_08490_amd.runner import to_device
            s.grad_out_dev = to_device(np.concatenate([x.reshape(-1) for x in mb.grad_out]), cfg.dtype, model.dev)
        slots.append(s)

    from paper_2408_08490_amd.runner import Batch

    ctx.hgnn_set_edge_types(g.edge_type)        # graph-resident, like the feature stores: registered once

    def start_build(slot):
        return ctx.hgnn_build_semantic_csr(slot.mb.blocks, None, use_edge_id=True,
                                           transpose_types=model.transpose_types(len(slot.mb.blocks)))

    def batch_of(slot, graph):
        b = Batch()
        b.ids_dev, b.n_rows, b.blocks = slot.ids_dev, [len(i) for i in slot.mb.ids], slot.mb.blocks
        b.graph, b.labels_dev, b.grad_out_dev = graph, slot.labels_dev, slot.grad_out_dev
        return b

    class Pipeline:
        """Step i runs on the GPU while the host threads build the index arrays of the next `lookahead` steps (the
        sampler of a training loop runs that far ahead).  The look-ahead stays filled from one call of run() to the
        next, so a timed run() that follows an untimed one measures the loop, not its start-up; every step still
        starts exactly one build."""

        def __init__(self):
            self.ahead, self.next, self.pending = [], 0, []

        def fill(self):
            while len(self.ahead) < args.lookahead:
                self.ahead.append((self.next, start_build(slots[self.next % len(slots)])))
                self.next += 1

        def run(self, nsteps):
            for _ in range(nsteps):
                i, cur = self.ahead.pop(0)
                self.ahead.append((self.next, start_build(slots[self.next % len(slots)])))
                self.next += 1
                model.run(batch_of(slots[i % len(slots)], cur))
                ev = torch.cuda.Event()
                ev.record()
                self.pending.append((ev, cur))
                while len(self.pending) > 2:              # keep at most two finished-or-running steps alive
                    e, gr = self.pending.pop(0)
                    e.synchronize()
                    gr.release()

        def drain(self):
            for e, gr in self.pending:
                e.synchronize()
                gr.release()
            for _, gr in self.ahead:
                gr.wait()
                gr.release()
            self.ahead, self.pending = [], []

    W, K = args.warmup, args.steps
    # kernels bracketed with HIP event pairs inside the timed region: the dominant kernel (forward GEMM of
    # layer 1: projection + fusion) and the aggregation kernel of layer 1, or the one asked for
    probes = ([("gemm_fwd", 0), ("spmm_fwd", 0)] + ([] if cfg.kind == "rgat" else [("gemm_dw", 0)])
              if args.probe == "auto" else [(k_, args.probe_layer) for k_ in args.probe.split(",")])
    pipe = Pipeline()
    t_f = time.perf_counter()
    pipe.fill()
    pipe.run(1)
    torch.cuda.synchronize()
    t_fill = time.perf_counter() - t_f          # cold start: look-ahead builds started, first step through the GPU
    pipe.run(max(W - 1, 0))
    torch.cuda.synchronize()
    # the W steps above last ~20 ms: not enough for 16 host threads and their buffer pools to reach their steady
    # state on a machine that was idle a moment ago, so the same untimed loop runs on for a few seconds
    t_w = time.perf_counter()
    while W > 0 and time.perf_counter() - t_w < args.host_warmup_s:
        pipe.run(max(W, 50))
    torch.cuda.synchronize()
    # the probe brackets every selected launch with an event pair that the library creates on first use: an untimed
    # pass of the same length creates them all, so that the timed steps only reuse them
    for k_, l_ in probes:
        ctx.hgnn_probe_select(B.KERNEL_IDS[k_], l_)
    pipe.run(K)
    torch.cuda.synchronize()
    ctx.hgnn_probe_select(-1, -1)
    for k_, l_ in probes:
        ctx.hgnn_probe_select(B.KERNEL_IDS[k_], l_)
    t1 = time.perf_counter()
    pipe.run(K)
    torch.cuda.synchronize()
    t_pipe = time.perf_counter() - t1
    probe_res = {(k_, l_): ctx.hgnn_probe_read(B.KERNEL_IDS[k_], l_) for k_, l_ in probes}
    ctx.hgnn_probe_select(-1, -1)
    pipe.drain()

    # same loop with the index arrays built beforehand (GPU work only)
    graphs = [start_build(s) for s in slots]
    for gr in graphs:
        gr.wait()
    for i in range(W):
        model.run(batch_of(slots[i % len(slots)], graphs[i % len(slots)]))
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    for i in range(K):
        model.run(batch_of(slots[i % len(slots)], graphs[i % len(slots)]))
    torch.cuda.synchronize()
    t_gpu = time.perf_counter() - t2
    # the probed kernels once more with the GPU kept busy (in the pipelined loop the GPU idles while it waits for
    # the host, and a launch that follows an idle gap can run at a lower clock: those readings vary from run to run)
    for k_, l_ in probes:
        ctx.hgnn_probe_select(B.KERNEL_IDS[k_], l_)
    for i in range(max(20, K // 4)):
        model.run(batch_of(slots[i % len(slots)], graphs[i % len(slots)]))
    torch.cuda.synchronize()
    probe_busy = {(k_, l_): ctx.hgnn_probe_read(B.KERNEL_IDS[k_], l_) for k_, l_ in probes}
    ctx.hgnn_probe_select(-1, -1)

    # host build alone
    t3 = time.perf_counter()
    nb = 20
    for i in range(nb):
        gr = start_build(slots[i % len(slots)])
        gr.wait()
        gr.release()
    t_build = (time.perf_counter() - t3) / nb

    # sampling in the loop: every step's mini-batch is drawn, selected, built and uploaded by one task of the
    # library's host threads while the GPU works on earlier steps (fresh targets every step)
    sil = None
    if not args.no_sampler_loop:
        sampler = ctx.hgnn_sampler_create(g.num_nodes, g.in_indptr, g.in_nbr, g.edge_off)
        tt, nt = model.target_type, len(mbs[0].ids[mbs[0].target_type][: mbs[0].blocks[-1].n_dst[mbs[0].target_type]])
        order = np.random.default_rng([MASTER_SEED + cfg.index, 77]).permutation(g.num_nodes[tt])
        n_chunks = max(1, len(order) // nt)
        labels_all = order_dev = None
        if cfg.loss == "xent":
            labels_all = torch.from_numpy(np.random.default_rng([MASTER_SEED + cfg.index, 78])
                                          .integers(0, cfg.num_classes, g.num_nodes[tt])).to(model.dev)
            order_dev = torch.from_numpy(order).to(model.dev)

        def start_sampled(i):
            c = i % n_chunks
            labels = None if labels_all is None else labels_all[order_dev[c * nt:(c + 1) * nt]]
            b = model.prepare_sampled(sampler, order[c * nt:(c + 1) * nt], cfg.fanouts, seed=1_000_003 * i + 17, labels=labels)
            b.grad_out_dev = slots[0].grad_out_dev
            return b

        def sampled_loop(nsteps, first):
            ahead = [start_sampled(first + j) for j in range(min(args.lookahead, nsteps))]
            started, pending = len(ahead), []
            for i in range(nsteps):
                cur = ahead.pop(0)
                if started < nsteps:
                    ahead.append(start_sampled(first + started))
                    started += 1
                model.run(cur)
                ev = torch.cuda.Event()
                ev.record()
                pending.append((ev, cur.graph))
                while len(pending) > 2:
                    e, gr = pending.pop(0)
                    e.synchronize()
                    gr.release()
            for e, gr in pending:
                e.synchronize()
                gr.release()

        sampled_loop(W, 0)
        # as above: the pooled sample buffers are cold for the first passes, so the untimed loop runs on for a while
        t_w = time.perf_counter()
        while W > 0 and time.perf_counter() - t_w < args.host_warmup_s / 2:
            sampled_loop(max(W, 50), W)
        torch.cuda.synchronize()
        t4 = time.perf_counter()
        sampled_loop(K, W)
        torch.cuda.synchronize()
        t_sil = time.perf_counter() - t4
        t5 = time.perf_counter()
        for i in range(10):                          # one task at a time: its own duration
            b = start_sampled(W + K + i)
            b.graph.wait()
            b.graph.release()
        t_task = (time.perf_counter() - t5) / 10
        nb_conc = max(1, args.concurrent_builds)
        sil = dict(value=round(K / t_sil, 2), unit="mini-batches/s", ms_per_step=round(1e3 * t_sil / K, 4),
                   host_task_ms=round(1e3 * t_task, 3), host_tasks_in_parallel=nb_conc,
                   cpu_gpu_time_ratio=round((t_task / nb_conc) / (t_gpu / K), 3),
                   note="neighbour sampling + index arrays + upload per step on the host threads, fresh "
                        "targets every step; cpu_gpu_time_ratio = host time per mini-batch at that parallelism / "
                        "GPU time per mini-batch")
        sampler.close()

    # launches per layer: merged vs per-relation / per-type launch loop
    launches = []
    b0 = batch_of(slots[0], graphs[0])
    attention = cfg.kind == "rgat"   # the per-relation launch loop exists for the mean variant only
    out_naive = None if attention else model.run(b0, backward=True, naive=True)
    torch.cuda.synchronize()
    for l in range(len(model.layers)):
        f, bw = ctx.hgnn_layer_launch_count(graphs[0], l, model.layers[l])
        launches.append(dict(layer=l, merged_fwd=f, merged_bwd=bw,
                             naive_fwd=None if attention else out_naive["launches"][l],
                             naive_bwd=None if attention else out_naive["launches_bwd"][l]))

    # algorithmic traffic / flops of the probed kernels, from the first mini-batch's shapes
    es = 2 if cfg.dtype == "bf16" else 4
    mb = slots[0].mb
    sch = g.schema

    def roofline_of(kname, layer):
        probe_ms, probe_n = probe_res[(kname, layer)]
        avg_ms = probe_ms / max(probe_n, 1)
        blk, lw = mb.blocks[layer], ws[layer]
        view = graphs[0].host_view(layer)
        rows, E = int(view["rows"]), int(view["edges"])
        live = [view["rel_edge_off"][r + 1] > view["rel_edge_off"][r] for r in range(sch.num_rels)]
        if kname == "spmm_fwd" and attention:
            # attention aggregation over projected rows of width H: each referenced source row once per relation
            # segment, the destination's own row, index arrays, the aggregate and the softmax statistics
            H = lw.out_dim
            uniq = sum(len(np.unique(view["colidx"][view["rel_edge_off"][r]: view["rel_edge_off"][r + 1]]))
                       for r in range(sch.num_rels))
            alg = (uniq + 2 * rows) * H * es + 4 * E + 4 * (rows + 1) + 2 * rows * cfg.heads * 4
            ach = alg / (avg_ms * 1e-3) / 1e9 if avg_ms > 0 else 0.0
            return dict(kernel="attn_agg_kernel (layer %d: segment-softmax aggregation)" % (layer + 1), bound="hbm",
                        achieved=round(ach, 1), peak=HBM_PEAK_GBS, unit="GB/s", frac=round(ach / HBM_PEAK_GBS, 4),
                        traffic=None, algorithmic_bytes=int(alg), avg_kernel_us=round(avg_ms * 1e3, 2), launches_timed=probe_n)
        if kname == "gemm_fwd" and attention:
            flops = sum(2 * blk.n_src[t] * lw.in_dim[t] * lw.out_dim for t in range(sch.num_types))
            ach = flops / (avg_ms * 1e-3) / 1e12 if avg_ms > 0 else 0.0
            peak = MFMA_BF16_PEAK_TFLOPS if cfg.dtype == "bf16" else 157.3
            return dict(kernel="attn_proj_kernel (layer %d: per-type projection)" % (layer + 1), bound="mfma",
                        achieved=round(ach, 1), peak=peak, unit="TFLOP/s", frac=round(ach / peak, 4), traffic=None,
                        algorithmic_flops=int(flops), avg_kernel_us=round(avg_ms * 1e3, 2), launches_timed=probe_n)
        if kname == "spmm_fwd":
            # each referenced source row once per relation segment + index arrays + the output plane(s)
            uniq = sum(len(np.unique(view["colidx"][view["rel_edge_off"][r]: view["rel_edge_off"][r + 1]])) *
                       lw.in_dim[sch.rel_src[r]] for r in range(sch.num_rels))
            zel = sum(blk.n_dst[sch.rel_dst[r]] * lw.in_dim[sch.rel_src[r]] for r in range(sch.num_rels))
            nplanes = 1
            alg = uniq * es + 4 * E + 4 * (rows + 1) + zel * es * nplanes
            req = alg + (sum(lw.in_dim[sch.rel_src[r]] * int(view["rel_edge_off"][r + 1] - view["rel_edge_off"][r])
                             for r in range(sch.num_rels)) - uniq) * es
            ach = alg / (avg_ms * 1e-3) / 1e9 if avg_ms > 0 else 0.0
            return dict(kernel="spmm_fwd_kernel (layer %d: relation-segmented gather-mean)" % (layer + 1), bound="hbm",
                        achieved=round(ach, 1), peak=HBM_PEAK_GBS, unit="GB/s", frac=round(ach / HBM_PEAK_GBS, 4),
                        traffic=None, algorithmic_bytes=int(alg), requested_bytes=int(req),
                        avg_kernel_us=round(avg_ms * 1e3, 2), launches_timed=probe_n)
        if kname in ("gemm_fwd", "gemm_dw", "gemm_da"):
            # 2*M*K*N over the live K-segments (relations with edges + root)
            flops = 0
            for t in range(sch.num_types):
                k = sum(lw.in_dim[sch.rel_src[r]] for r in range(sch.num_rels) if sch.rel_dst[r] == t and live[r])
                k += lw.in_dim[t] if lw.w_root[t] is not None else 0
                flops += 2 * blk.n_dst[t] * k * lw.out_dim
            label = "%s_kernel (layer %d)" % (kname, layer + 1)
            if kname == "gemm_dw":
                # the weight-gradient tiles share their launch with the input-gradient tiles (dZ_s = G' W_s^T for
                # the segments whose source type wants an input gradient): count both
                ig = model.first_layer_input_grad if layer == 0 and model.first_layer_input_grad is not None \
                    else [1] * sch.num_types
                fl_da = sum(2 * blk.n_dst[sch.rel_dst[r]] * lw.in_dim[sch.rel_src[r]] * lw.out_dim
                            for r in range(sch.num_rels) if live[r] and ig[sch.rel_src[r]])
                fl_da += sum(2 * blk.n_dst[t] * lw.in_dim[t] * lw.out_dim for t in range(sch.num_types)
                             if lw.w_root[t] is not None and ig[t])
                if fl_da > 0:
                    flops += fl_da
                    label = "gemm_bwd_kernel (layer %d: weight-gradient and input-gradient GEMM tiles in one launch)" % (layer + 1)
            ach = flops / (avg_ms * 1e-3) / 1e12 if avg_ms > 0 else 0.0
            peak = MFMA_BF16_PEAK_TFLOPS if cfg.dtype == "bf16" else 157.3
            return dict(kernel=label, bound="mfma", achieved=round(ach, 1), peak=peak,
                        unit="TFLOP/s", frac=round(ach / peak, 4), traffic=None, algorithmic_flops=int(flops),
                        avg_kernel_us=round(avg_ms * 1e3, 2), launches_timed=probe_n)
        return dict(kernel=kname, bound="hbm", achieved=None, peak=HBM_PEAK_GBS, unit="GB/s", frac=None, traffic=None,
                    avg_kernel_us=round(avg_ms * 1e3, 2), launches_timed=probe_n)

    def with_busy(r, key):
        if r is not None:
            ms, n = probe_busy[key]
            r["avg_kernel_us_gpu_busy"] = round(1e3 * ms / max(n, 1), 2)
        return r
    roof_proj = roofline_of(*probes[0])
    roof_agg = roofline_of(*probes[1]) if len(probes) > 1 else None
    roof_dw = roofline_of(*probes[2]) if len(probes) > 2 else None
    if roof_agg is not None:
        # HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this command (profiles/)
        if cfg.index == 2 and args.scale == 1.0:     # measured on the default workload only
            tb = traffic_bytes()
            roof_proj["traffic"] = tb.get("gemm_fwd_layer1")
            roof_agg["traffic"] = tb.get("spmm_fwd_layer1")
            if roof_dw is not None:
                roof_dw["traffic"] = tb.get("gemm_bwd_layer1")
    with_busy(roof_proj, probes[0])
    if roof_agg is not None:
        with_busy(roof_agg, probes[1])
    if roof_dw is not None:
        with_busy(roof_dw, probes[2])
    # `roofline` is the dominant kernel, the longest launch of a step: the backward GEMM launch of layer 1 where it
    # exists (profiles/), else the projection
    roof = roof_dw if roof_dw is not None else roof_proj

    # ablation: what each piece buys on this machine
    abl = None
    if not args.no_ablation:
        def gpu_ms(fn, n):
            torch.cuda.synchronize()
            a, b_ = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for i in range(n):
                fn(i)
            b_.record()
            torch.cuda.synchronize()
            return a.elapsed_time(b_) / n

        def step_naive(i):
            model.run(batch_of(slots[i % len(slots)], graphs[i % len(slots)]), backward=True, naive=True)

        def step_merged(i):
            model.run(batch_of(slots[i % len(slots)], graphs[i % len(slots)]), backward=True)

        def fwd_only(naive, two_step=False):
            def f(i):
                model.run(batch_of(slots[i % len(slots)], graphs[i % len(slots)]), backward=False, naive=naive, two_step=two_step)
            return f
        n_ab = max(20, K // 4) if args.ablation else 20
        fwd_only(False)(0)
        merged_fwd_ms = gpu_ms(fwd_only(False), n_ab)
        naive_fwd_ms = two_step_fwd_ms = None
        if not attention:
            fwd_only(True)(0)
            naive_fwd_ms = gpu_ms(fwd_only(True), n_ab)
            if len(set(g.feat_dim)) == 1 and all(len(set(lw.in_dim)) == 1 for lw in model.layers):
                fwd_only(False, True)(0)
                two_step_fwd_ms = gpu_ms(fwd_only(False, True), n_ab)

        def serial_loop(n):          # build, wait, compute, wait: nothing overlaps
            t = time.perf_counter()
            for i in range(n):
                gr = start_build(slots[i % len(slots)])
                gr.wait()
                model.run(batch_of(slots[i % len(slots)], gr))
                torch.cuda.synchronize()
                gr.release()
            return (time.perf_counter() - t) / n
        serial_loop(3)
        serial_ms = 1e3 * serial_loop(n_ab)

        # the index arrays built by device kernels on the compute stream, in front of each step's compute
        dev_build_gpu_ms = []

        def device_build_loop(n):
            t = time.perf_counter()
            for i in range(n):
                sl = slots[i % len(slots)]
                gr = ctx.hgnn_build_semantic_csr_device(sl.mb.blocks, None, use_edge_id=True,
                                                        transpose_types=model.transpose_types(len(sl.mb.blocks)))
                dev_build_gpu_ms.append(gr.build_gpu_ms)
                model.run(batch_of(sl, gr))
                torch.cuda.synchronize()
                gr.release()
            return (time.perf_counter() - t) / n
        device_build_loop(3)
        del dev_build_gpu_ms[:]
        device_build_step_ms = 1e3 * device_build_loop(n_ab)
        step_naive_ms = None
        if not attention:
            step_naive(0)
            step_naive_ms = gpu_ms(step_naive, n_ab)
        step_merged(0)
        step_merged_ms = gpu_ms(step_merged, n_ab)
        step_other_merge_ms = None
        if cfg.kind != "rgat" and len(set(g.feat_dim)) == 1:
            def step_other(i):
                model.run(batch_of(slots[i % len(slots)], graphs[i % len(slots)]), backward=True, gather=not model.gather)
            step_other(0)
            step_other_merge_ms = gpu_ms(step_other, n_ab)
        # index-first feature layout: the rows of all types interleaved in one buffer, then a selection pass per step that
        # puts them type-first for the layer calls (the type-first merge does this in one pass)
        index_first_ms = type_first_merge_ms = None
        if len(set(g.feat_dim)) == 1:
            sl0 = slots[0]
            n0 = [len(i) for i in sl0.mb.ids]
            tot0, F0 = sum(n0), g.feat_dim[0]
            key = np.concatenate([(np.arange(k) + 0.5) / max(k, 1) for k in n0])
            rank = np.empty(tot0, np.int64)
            rank[np.argsort(key, kind="stable")] = np.arange(tot0)
            offs = np.concatenate([[0], np.cumsum(n0)])
            pos = [torch.from_numpy(rank[offs[t]: offs[t + 1]].astype(np.int32)).to(model.dev) for t in range(len(n0))]
            x_int = torch.empty(tot0 * F0, device=model.dev, dtype=model.stores[0].dtype)
            x_tf = torch.empty(tot0 * F0, device=model.dev, dtype=model.stores[0].dtype)

            def index_first(i):
                ctx.hgnn_merge_features_index_first(model.stores, sl0.ids_dev, pos, x_int, g.feat_dim)
                ctx.hgnn_select_type_first(x_int, pos, x_tf, g.feat_dim)

            def type_first(i):
                ctx.hgnn_merge_features(model.stores, sl0.ids_dev, x_tf, g.feat_dim)
            index_first(0)
            index_first_ms = gpu_ms(index_first, n_ab)
            type_first_merge_ms = gpu_ms(type_first, n_ab)
        abl = dict(steps_timed=n_ab, forward_merged_ms=round(merged_fwd_ms, 4),
                   feature_stage_type_first_ms=None if type_first_merge_ms is None else round(type_first_merge_ms, 4),
                   feature_stage_index_first_ms=None if index_first_ms is None else round(index_first_ms, 4),
                   step_merged_launches_ms=round(step_merged_ms, 4),
                   first_layer_input=("destination rows merged, aggregation reads the feature stores" if model.gather
                                      else "every source row merged"),
                   step_other_first_layer_input_ms=None if step_other_merge_ms is None else round(step_other_merge_ms, 4),
                   step_per_relation_launches_ms=None if step_naive_ms is None else round(step_naive_ms, 4),
                   forward_per_relation_launches_ms=None if naive_fwd_ms is None else round(naive_fwd_ms, 4),
                   forward_two_step_aggregation_ms=None if two_step_fwd_ms is None else round(two_step_fwd_ms, 4),
                   step_serial_build_then_compute_ms=round(serial_ms, 4),
                   step_device_build_then_compute_ms=round(device_build_step_ms, 4),
                   device_build_gpu_ms=round(float(np.mean(dev_build_gpu_ms)), 4),
                   step_overlapped_ms=round(1e3 * t_pipe / K, 4), step_gpu_only_ms=round(1e3 * t_gpu / K, 4),
                   host_builders=args.concurrent_builds,
                   note="forward_*: merge + all layers forward, index arrays resident (GPU time between events); step_*: "
                        "the same with loss and backward, merged launches against the per-relation / per-type launch loop; two_step: "
                        "the aggregation as Algorithm 1 states it (source rows of all semantic graphs gathered into "
                        "FeatureCat, then reduced by destination) instead of the fused gather-mean; "
                        "feature_stage_*: the feature merge alone, type-first in one pass (hgnn_merge_features) against an index-first "
                        "buffer (rows of all types interleaved) followed by the per-type selection the layer calls need; "
                        "serial: every step builds its index arrays with one builder, waits, computes, waits; "
                        "device_build: every step builds them with device kernels on the compute stream "
                        "(hgnn_build_semantic_csr_device: keys, two radix sorts, prefix sums), then computes; device_build_gpu_ms "
                        "is the GPU time of that build alone, input upload included; "
                        "overlapped: bench.py's `value` loop")

    # whole training steps (forward, loss, backward, Adam on all weights and on the embedding rows read), index
    # arrays resident: what the parameter update adds to a step.  Runs last: it changes weights and embeddings.
    train = None
    if not args.no_train_loop and not attention:
        model.enable_training()
        for i in range(W):
            b = batch_of(slots[i % len(slots)], graphs[i % len(slots)])
            model.optimizer_step(b, model.run(b))
        torch.cuda.synchronize()
        t6 = time.perf_counter()
        for i in range(K):
            b = batch_of(slots[i % len(slots)], graphs[i % len(slots)])
            model.optimizer_step(b, model.run(b))
        torch.cuda.synchronize()
        t_train = time.perf_counter() - t6
        n_par = sum(p.numel() for p in model.adam["params"])
        train = dict(gpu_only_mb_per_s=round(K / t_train, 2), gpu_only_ms_per_step=round(1e3 * t_train / K, 4),
                     optimizer="Adam: %d weights in one launch, embedding rows of the learnable types touched by the "
                               "mini-batch in one launch per type (fp32 masters and moments)" % n_par,
                     loss_after=round(float(model.loss_dev.item()), 4))

    for gr in graphs:
        gr.release()

    if args.calibrate:
        n_cal = 1 << 20
        tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
        src = torch.ones((n_cal, 128), device=model.dev, dtype=tdt)
        dst = torch.empty((n_cal, 128), device=model.dev, dtype=tdt)
        ids = torch.arange(n_cal, device=model.dev, dtype=torch.int64)
        T_ = sch.num_types
        for _ in range(3):
            ctx.hgnn_merge_features([src] + [None] * (T_ - 1), [ids] + [None] * (T_ - 1), dst, [128] * T_)
        torch.cuda.synchronize()

    cpu = None
    if not args.no_cpu_baseline:
        from tests.parity import oracle_run
        import copy
        cfg_s = make_config(args.config, scale=args.scale, batch=args.cpu_sample_batch)
        mb_s = sample_minibatch(cfg_s, g, rng=np.random.default_rng([MASTER_SEED + cfg.index, 999]))
        if mb_s.grad_out is not None and cfg.dtype == "bf16":
            mb_s.grad_out = [bf16_round(x) for x in mb_s.grad_out]
        tc = time.perf_counter()
        oracle_run(cfg_s, g, mb_s, ws)                # plain numpy fp64 oracle, whole mini-batch, fwd + bwd
        t_cpu = time.perf_counter() - tc
        frac = args.cpu_sample_batch / cfg.batch
        cpu = dict(value=round(frac / t_cpu, 5), unit="mini-batches/s", cores=os.cpu_count() if False else len(os.sched_getaffinity(0)),
                   kind="oracle",
                   sample="one mini-batch of %d targets (%.3g of the workload's %d): feature merge, index build, both "
                          "layers forward and backward in numpy fp64, %.1f s; rate scaled by the target fraction; "
                          "numpy's BLAS uses the host cores for the matmuls, the row loops are single-threaded" %
                          (args.cpu_sample_batch, frac, cfg.batch, t_cpu))

    sizes = [dict(src_rows=sum(b.n_src), dst_rows=sum(b.n_dst), edges=int(b.edge_index.shape[1])) for b in mb.blocks]
    line = dict(
        metric="HGNN layer fwd+bwd mini-batches/s (1 GPU)", value=round(K / t_pipe, 2), unit="mini-batches/s",
        n_gpus=1, steps=K, warmup=W, ms_per_step=round(1e3 * t_pipe / K, 4), higher_is_better=True, scaling="weak",
        vs_baseline=None, dtype=cfg.dtype, data="synthetic",
        config=dict(workload="configs[%d] %s: %d types / %d relations, %d targets, fanout %s, layers %s, scale %.3g" %
                    (cfg.index, cfg.name, sch.num_types, sch.num_rels, cfg.batch, cfg.fanouts[::-1],
                     [g.feat_dim[0]] + cfg.layer_out, cfg.scale),
                    minibatch_sizes=sizes, distinct_minibatches=len(slots),
                    first_layer_input=("feature merge of the destination rows; the aggregation reads the source rows in "
                                       "the per-type feature stores (hgnn_layer_fwd_gather / hgnn_layer_bwd_gather)"
                                       if model.gather else "feature merge of every source row (hgnn_layer_fwd / hgnn_layer_bwd)"),
                    index_build_outputs=("rowptr, colidx, cptr, crow, chunk lists" +
                                         (", perm, cperm" if args.build_permutation or attention else
                                          " (perm / cperm, which no kernel of this path reads, are left out)"))),
        gpu_only_mb_per_s=round(K / t_gpu, 2), gpu_only_ms_per_step=round(1e3 * t_gpu / K, 4),
        pipeline=dict(lookahead=args.lookahead, fill_ms=round(1e3 * t_fill, 3),
                      note="the look-ahead is filled before the timed region (fill_ms: cold start until the first step has "
                           "left the GPU); the K timed steps start K builds and run K steps"),
        host_build_ms=round(1e3 * t_build, 3), sampler_in_loop=sil, training_step=train, ablation=abl, launches_per_layer=launches,
        roofline=roof, roofline_projection=roof_proj, roofline_weight_grad=roof_dw, roofline_aggregation=roof_agg,
        cpu_baseline=cpu, setup_s=round(t_setup, 1))
    print(json.dumps(line))
    model.close()


if __name__ == "__main__":
    main()
