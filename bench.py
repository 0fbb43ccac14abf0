#!/usr/bin/env python3
"""Benchmark of one pipeline stage on one MI355X.

A step = one epoch's work of the stage: forward over all chunks (shuffled order), backward over
the chunks in reverse, then update_history.  The headline workload is configuration 4 of the
benchmark definition, the largest one that fits a GPU (R-MAT graph, 10 M vertices, 210 M entries,
4 GCN layers of width 256 in bf16, 32 chunks); configurations 1 to 3 are timed in the same run and
reported under "per_config".  Inputs are synthetic and resident in HBM before the timed region.
Prints one JSON line.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
BF16_MFMA_PEAK = 2.5e15
FP32_VALU_PEAK = 157.3e12
HEADLINE = "c4"
SECONDARY = ("c1", "c2", "c3")


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def pair_counts(row_ptr, col, chunk_ptr):
    """E[k][c] = entries of chunk k's rows whose column lies in chunk c; D[k][c] = distinct columns among them."""
    K = len(chunk_ptr) - 1
    n = len(row_ptr) - 1
    E = np.zeros((K, K), dtype=np.int64)
    D = np.zeros((K, K), dtype=np.int64)
    for k in range(K):
        cols = col[row_ptr[chunk_ptr[k]]:row_ptr[chunk_ptr[k + 1]]]
        mark = np.zeros(n, dtype=bool)
        mark[cols] = True
        cnt = np.bincount(np.searchsorted(chunk_ptr, cols, side="right") - 1, minlength=K)
        E[k] = cnt[:K]
        D[k] = np.add.reduceat(mark.astype(np.int64), chunk_ptr[:-1].clip(max=n - 1))[:K]
        for c in range(K):  # reduceat misreads empty ranges
            if chunk_ptr[c] == chunk_ptr[c + 1]:
                D[k, c] = 0
    return E, D


def copy_bandwidth(torch, dev, nbytes=2 << 30, reps=5):
    """What this machine's memory system gives a plain device-to-device copy (torch's copy kernel), read + written
    bytes per second: the yardstick for update_history."""
    a = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    b = torch.empty_like(a)
    b.copy_(a)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record()
    for _ in range(reps):
        b.copy_(a)
    ev1.record()
    torch.cuda.synchronize()
    ms = ev0.elapsed_time(ev1) / reps
    del a, b
    torch.cuda.empty_cache()
    return 2.0 * nbytes / (ms * 1e-3) / 1e9


def run_config(name, args, steps, warmup, with_cpu, copy_gbs):
    """Builds the workload, times `steps` steps and returns the result object of that configuration."""
    import torch
    import paper_2308_10087_amd as g
    from synth import values
    from synth.configs import CONFIGS, make_graph
    from synth.graphs import degree_stats, equal_chunks

    dev = "cuda:0"
    w = CONFIGS[name]
    t0 = time.time()
    row_ptr, col = make_graph(w)
    n, nnz = len(row_ptr) - 1, int(row_ptr[-1])
    chunk_ptr = equal_chunks(n, w.n_chunks)
    cut_note = ""
    if args.partition:
        t_p = time.time()
        part, perm, chunk_ptr = g.gnnstage_partition_chunks(row_ptr, col, w.n_chunks, by_entries=args.partition_by_entries)
        rows_all = np.repeat(np.arange(n, dtype=np.int64), np.diff(row_ptr))
        off = rows_all != col
        blind = (np.arange(n, dtype=np.int64) * w.n_chunks // n)
        cut_before = float(np.mean(blind[rows_all[off]] != blind[col[off]]))
        cut_after = float(np.mean(part[rows_all[off]] != part[col[off]]))
        del rows_all, off
        row_ptr, col = g.gnnstage_permute_csr(row_ptr, col, perm)
        cut_note = f" partitioned chunks (neighbours in other chunks {cut_before:.3f} -> {cut_after:.3f}, sizes {np.diff(chunk_ptr).min()}..{np.diff(chunk_ptr).max()})"
        log(f"[bench] partitioner: {time.time() - t_p:.1f}s,{cut_note}")
    K, L, dims = w.n_chunks, w.n_layers, list(w.dims)
    stats = degree_stats(row_ptr)
    log(f"[bench] graph {w.name}: {stats} built in {time.time() - t0:.1f}s")

    bf = w.dtype == "bf16"
    sdt = torch.bfloat16 if bf else torch.float32
    l0 = torch.float32 if (w.level0_f32 or not bf) else torch.bfloat16
    gcn = w.variant != "gcnii"  # layer types with a bias vector and no GCNII inputs
    sage, res = w.variant == "sage", w.variant == "resgcn"
    gen = torch.Generator(device=dev)
    gen.manual_seed(w.seed)

    def dev_normal(shape, dtype, absolute=False):
        # drawn on the device: the 10 M x 256 tables of the largest configuration take minutes on the host
        x = torch.randn(shape, generator=gen, device=dev)
        if absolute:
            x.abs_()
        return x.to(dtype)

    wrows = 2 if sage else 1  # GraphSage stacks [W_self ; W_neigh]
    W = [torch.from_numpy(np.concatenate([values.glorot_uniform(w.seed, 100 + 50 * h + j, dims[j], dims[j + 1]) for h in range(wrows)]))
         .to(dev, sdt) for j in range(L)]
    bias = [torch.zeros(dims[j + 1], device=dev) for j in range(L)] if gcn else None
    cur = [dev_normal((n, dims[0]), l0, absolute=not gcn)] + [torch.zeros((n, dims[j]), dtype=sdt, device=dev) for j in range(1, L + 1)]
    first_stage = (w.variant == "gcn") if w.first_stage is None else w.first_stage
    ln = [[torch.ones(dims[j], device=dev) for j in range(L)], [torch.zeros(dims[j], device=dev) for j in range(L)],
          [torch.zeros(dims[j], device=dev) for j in range(L)], [torch.zeros(dims[j], device=dev) for j in range(L)]] if res else [None] * 4
    hist = [cur[0] if first_stage else cur[0].clone()] + [torch.zeros((n, dims[j]), dtype=sdt, device=dev) for j in range(1, L)]
    dW = [torch.zeros((wrows * dims[j], dims[j + 1]), device=dev) for j in range(L)]
    dbias = [torch.zeros(dims[j + 1], device=dev) for j in range(L)] if gcn else None
    h0 = None if gcn else dev_normal((n, dims[0]), sdt)
    grad_h0 = None if gcn else torch.zeros((n, dims[0]), device=dev)
    grad_in = None if first_stage else torch.zeros((n, dims[0]), dtype=l0, device=dev)
    grad_out = dev_normal((n, dims[-1]), sdt)
    beta = None
    if not gcn:
        beta = np.array([math.log(0.5 / l + 1.0) for l in range(w.gcnii_first_layer, w.gcnii_first_layer + L)], np.float32)
    edge_val = None
    if args.caller_weights:  # the weights the library would compute itself: 1 / sqrt(D_v D_u), or 1 / D_v for the mean aggregator
        deg = np.diff(row_ptr).astype(np.float64)
        inv = 1.0 / np.maximum(deg, 1.0) if sage else 1.0 / np.sqrt(np.maximum(deg, 1.0))
        edge_val = (np.repeat(inv, np.diff(row_ptr)) * (1.0 if sage else inv[col])).astype(np.float32)
    t1 = time.time()
    st = g.GnnStage(row_ptr, col, chunk_ptr, dims, W=W, cur=cur, hist=hist, dW=dW, bias=bias, dbias=dbias, edge_val=edge_val,
                    variant={"gcn": g.GNNSTAGE_GCN, "gcnii": g.GNNSTAGE_GCNII, "sage": g.GNNSTAGE_SAGE,
                             "resgcn": g.GNNSTAGE_RESGCN}[w.variant], alpha=w.gcnii_alpha, beta=beta, h0=h0,
                    grad_h0=grad_h0, dtype=g.GNNSTAGE_BF16 if bf else g.GNNSTAGE_F32, level0_f32=w.level0_f32,
                    grad_in=grad_in, device=dev, ln_gamma=ln[0], ln_beta=ln[1], d_ln_gamma=ln[2], d_ln_beta=ln[3])
    log(f"[bench] gnnstage_create: {time.time() - t1:.1f}s, workspace {st.workspace_bytes / 2**30:.2f} GiB")

    def one_step(step_idx: int, swap: bool = args.history_swap):
        order = values.permutation(w.seed, 1000 + step_idx, K)
        for t in dW:
            t.zero_()
        if dbias:
            for t in dbias:
                t.zero_()
        if grad_h0 is not None:
            grad_h0.zero_()
        st.forward_pass(order)
        st.backward_pass(order, grad_out)
        if swap:
            st.gnnstage_update_history_swap()
        else:
            st.update_history()
        return order

    # historical buffers: one untimed epoch from zero history, refresh, then N(0, 0.01^2) noise
    one_step(-1)
    for j in range(L):
        if st.hist[j].data_ptr() != st.cur[j].data_ptr():  # the stage's lists: with --history-swap the buffers trade places
            rows_per = max(1, (1 << 28) // max(dims[j], 1))  # in slices: the noise of a whole 10 M x 256 level is 10 GB of fp32
            for r0 in range(0, n, rows_per):
                sl = st.hist[j][r0:r0 + rows_per]
                sl.add_((0.01 * torch.randn(sl.shape, generator=gen, device=dev)).to(sl.dtype))
    for i in range(warmup):
        one_step(i)
    torch.cuda.synchronize()

    # Inside the timed region only the launches of an aggregation (the dominant operation: gather kernels and
    # the reduce kernel that adds the partial rows of cut rows) carry HIP events, two event records per launch on
    # the launch stream, and only in every `event_every`-th step: an event pair costs a launch about a microsecond
    # and a half, which is a tenth of a step made of 2,000 launches of a few microseconds (configs[3]).  The per-kind
    # breakdown of a whole step comes from two further, untimed steps with every kind switched on.
    st.gnnstage_profile_reset()
    st.gnnstage_profile_enable(False)
    every = max(1, args.event_every)
    orders = []          # of the steps whose aggregations carried events
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for i in range(steps):
        if i % every == 0:
            st.gnnstage_profile_select(["spmm_fwd", "spmm_bwd", "spmm_reduce"])
        elif i % every == 1:
            st.gnnstage_profile_enable(False)
        order = one_step(warmup + i)
        if i % every == 0:
            orders.append(order)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start
    st.gnnstage_profile_enable(False)
    prof_layer = [st.gnnstage_profile_read(j) for j in range(L)]
    st.gnnstage_profile_reset()
    st.gnnstage_profile_enable(True)
    n_extra = 2
    for i in range(n_extra):
        one_step(warmup + steps + i)
    torch.cuda.synchronize()
    st.gnnstage_profile_enable(False)
    prof_all = st.gnnstage_profile_read(-1)
    # for comparison, not part of the line's value: the same steps with the history refreshed by trading buffers
    swap_ms = None
    if not args.history_swap and L > 1:
        n_swap = min(steps, 5)
        one_step(warmup + steps + n_extra, swap=True)
        torch.cuda.synchronize()
        t_sw = time.perf_counter()
        for i in range(n_swap):
            one_step(warmup + steps + n_extra + 1 + i, swap=True)
        torch.cuda.synchronize()
        swap_ms = round(1e3 * (time.perf_counter() - t_sw) / n_swap, 3)

    ms_per_step = 1e3 * elapsed / steps
    value = L * nnz / (elapsed / steps)

    # ---- roofline of the dominant operation ------------------------------------------------
    # Aggregations are grouped by the rows they gather (width, element type): one kernel instantiation and
    # launch shape per group, the same grouping rocprofv3 shows by kernel name.  One aggregation = the gather
    # kernels (dense blocks, sparse remainder) plus the reduce kernel; its duration is the sum of the three.
    # Algorithmic bytes of an aggregation over chunk k: every entry's packed index word (4 B) plus its weight
    # (4 B) when the caller gave weights - 0 B when the library computes the normalisation itself, as here -,
    # the chunk's row pointers, each DISTINCT gathered source row once, the output rows (+ the level rows a
    # masking epilogue reads).  Backward launches gather only entries whose reader chunk is already processed.
    E, D = pair_counts(row_ptr, col, chunk_ptr)
    rows = np.diff(chunk_ptr)
    elt = 2 if bf else 4
    tf = [st.gnnstage_layer_order(j) for j in range(L)]
    shared0 = hist[0].data_ptr() == cur[0].data_ptr()
    groups = {}

    def add(group, nbytes, gather, ms, launches):
        gr = groups.setdefault(group, [0.0, 0.0, 0.0, 0])
        gr[0] += nbytes
        gr[1] += gather
        gr[2] += ms
        gr[3] += launches

    def gname(d, e):
        return f"spmm gather width {d} {'f32' if e == 4 else 'bf16'}"

    entry_bytes = 8 if edge_val is not None else 4
    struct = [E[k].sum() * entry_bytes + 8 * (rows[k] + 1) for k in range(K)]
    for j in range(L):
        lvl_e = 4 if (j == 0 and l0 == torch.float32) else elt
        dg, eg = (dims[j + 1], elt) if tf[j] else (dims[j], lvl_e)       # what the forward gathers
        fb = sum(struct[k] + D[k].sum() * dg * eg + rows[k] * (dims[j + 1] if tf[j] else dims[j]) * elt
                 for k in range(K)) * len(orders)
        f_ms, f_n = prof_layer[j]["spmm_fwd"]
        b_ms, b_n = prof_layer[j]["spmm_bwd"]
        r_ms = prof_layer[j]["spmm_reduce"][0]
        # the reduce launches of a layer belong to its forward and backward aggregations alike: by launch count
        f_red = r_ms * f_n / max(f_n + b_n, 1)
        add(gname(dg, eg), fb, E.sum() * dg * eg * len(orders), f_ms + f_red, f_n)
        db_, eb = (dims[j + 1], elt) if tf[j] else (dims[j], elt)        # what the backward gathers
        bb = gb = 0.0
        masked = (j > 0 or grad_in is not None or res) and not (tf[j] and j == 0 and shared0 and grad_in is None)
        for order in orders:
            done = np.zeros(K, dtype=bool)
            for k in reversed(list(order)):
                done[k] = True
                if masked:
                    bb += struct[k] + D[k][done].sum() * db_ * eb + rows[k] * db_ * elt * (2 if (j > 0 and not tf[j]) else 1)
                    gb += E[k][done].sum() * db_ * eb
            if tf[j]:  # end-of-pass unmasked transposed aggregation of a transform-first layer
                bb += sum(struct[k] + D[k].sum() * db_ * eb + rows[k] * db_ * elt for k in range(K))
                gb += E.sum() * db_ * eb
            if res:  # end-of-pass aggregations over the readers that saw historical rows (LayerNorm parameters)
                earlier = np.zeros(K, dtype=bool)
                for pos, k in enumerate(order):
                    if pos > 0:
                        bb += struct[k] + D[k][earlier].sum() * db_ * eb + rows[k] * db_ * elt
                        gb += E[k][earlier].sum() * db_ * eb
                    earlier[k] = True
        if b_n > 0:
            add(gname(db_, eb), bb, gb, b_ms + (r_ms - f_red), b_n)
    dom_name, (dom_bytes, dom_gather, dom_ms, dom_launches) = max(groups.items(), key=lambda kv: kv[1][2])
    achieved = dom_bytes / (dom_ms * 1e-3) / 1e9 if dom_ms > 0 else 0.0
    traffic = None  # HBM-side bytes per aggregation from the committed rocprofv3 counter summary, if it covers this kernel
    tpath = os.path.join(ROOT, "profiles", f"stage_{w.name}_pmc_traffic.md")
    if os.path.exists(tpath) and not args.partition and not args.caller_weights:  # the counters were read on the benchmark configuration only
        for line in open(tpath):
            parts = [x.strip() for x in line.split("|")]
            if len(parts) == 3 and parts[0] == f"traffic {w.name}" and parts[1] == dom_name:
                traffic = float(parts[2])
    roofline = {
        "bound": "hbm", "kernel": dom_name, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
        "one_launch": "one aggregation over a chunk: gather kernels (dense blocks, sparse rows) + the reduce of cut rows",
        "algorithmic_bytes_per_launch": round(dom_bytes / max(dom_launches, 1)),
        "avg_launch_ms": round(dom_ms / max(dom_launches, 1), 4), "launches": dom_launches,
        "steps_with_events": len(orders),
        "gathered_bytes_per_launch": round(dom_gather / max(dom_launches, 1)),
        "gather_GBps": round(dom_gather / max(dom_ms * 1e-3, 1e-12) / 1e9, 1),
        "layer_order": ["transform-first" if t else "aggregate-first" for t in tf],
    }
    kernels_ms = {k: round(v[0] / n_extra, 3) for k, v in prof_all.items()}

    # ---- gemm side of the metric: achieved rate of the dense products against the matrix-core peak and against
    # the ceiling of their own shape, min(peak, arithmetic intensity x HBM bandwidth), operands from HBM once
    gemm_flops = gemm_bytes = 0.0
    for j in range(L):
        per = 2.0 * n * dims[j] * dims[j + 1]
        products = 3 if (j > 0 or not first_stage) else 2   # forward, weight gradient, input gradient
        gemm_flops += per * products
        in_e = 4 if (j == 0 and l0 == torch.float32) else elt
        gemm_bytes += products * (n * (dims[j] * in_e + dims[j + 1] * elt) + dims[j] * dims[j + 1] * elt)
    gemm_ms = sum(prof_all[k][0] for k in ("gemm_fwd", "gemm_dgrad", "gemm_wgrad")) / n_extra
    peak = BF16_MFMA_PEAK if bf else FP32_VALU_PEAK
    rate = gemm_flops / max(gemm_ms * 1e-3, 1e-12)
    ai = gemm_flops / gemm_bytes
    ceiling = min(peak, ai * HBM_PEAK_GBS * 1e9)
    gemm = {"tflops": round(rate / 1e12, 1), "ms_per_step": round(gemm_ms, 3),
            "frac_of_mfma_peak": round(rate / peak, 4),
            "flop_per_byte": round(ai, 1), "shape_ceiling_tflops": round(ceiling / 1e12, 1),
            "frac_of_shape_ceiling": round(rate / ceiling, 4),
            "bound": "hbm" if ceiling < peak else "mfma"}

    # ---- update_history against this box's plain copy bandwidth
    hist_bytes = sum(2.0 * n * dims[j] * (4 if (j == 0 and l0 == torch.float32) else elt)
                     for j in range(L) if hist[j].data_ptr() != cur[j].data_ptr())
    hms = kernels_ms.get("history_copy", 0.0)
    if args.history_swap:  # nothing is copied (but a level 0 with a history buffer of its own)
        hist_bytes = 2.0 * n * dims[0] * (4 if l0 == torch.float32 else elt) if hist[0].data_ptr() != cur[0].data_ptr() else 0.0
    history = {"mode": "swap" if args.history_swap else "copy", "step_ms_with_buffers_traded_instead": swap_ms,
               "bytes_per_step": round(hist_bytes), "ms_per_step": hms,
               "GBps": round(hist_bytes / max(hms * 1e-3, 1e-12) / 1e9, 1) if hms > 0 else None,
               "box_copy_GBps": round(copy_gbs, 1),
               "frac_of_box_copy": round(hist_bytes / max(hms * 1e-3, 1e-12) / 1e9 / copy_gbs, 3) if hms > 0 else None}

    # ---- optional: epochs of the whole training loop around the same stage ------------------
    trainer = None
    if args.train_epochs > 0 and w.variant == "gcn":
        n_classes = 41
        labels = torch.from_numpy(values._rng(w.seed, 7).integers(0, n_classes, size=n).astype(np.int32)).to(dev)
        master = [t.to(torch.float32) for t in W] if bf else W
        head_master = torch.from_numpy(values.glorot_uniform(w.seed, 900, dims[-1], n_classes)).to(dev)
        head_W = head_master.to(sdt) if bf else head_master
        head_b = torch.zeros(n_classes, device=dev)
        head_dW, head_db = torch.zeros((dims[-1], n_classes), device=dev), torch.zeros(n_classes, device=dev)
        params = [(master[j], W[j] if bf else None, dW[j]) for j in range(L)] + [(bias[j], None, dbias[j]) for j in range(L)]
        params += [(head_master, head_W if bf else None, head_dW), (head_b, None, head_db)]
        tr = g.GnnTrainer([st], head_W=head_W, head_b=head_b, head_dW=head_dW, head_db=head_db, labels=labels,
                          train_mask=None, params=params, optimizer=g.GNNTRAIN_ADAM, lr=1e-3, shuffle=True, seed=w.seed,
                          alpha_hist=1, device=dev)
        tr.gnntrain_epoch(0)
        torch.cuda.synchronize()
        t_tr = time.perf_counter()
        for e in range(1, args.train_epochs + 1):
            last_loss = tr.gnntrain_epoch(e, want_loss=(e == args.train_epochs))
        torch.cuda.synchronize()
        trainer = {"ms_per_epoch": round(1e3 * (time.perf_counter() - t_tr) / args.train_epochs, 3), "epochs": args.train_epochs,
                   "head_classes": n_classes, "optimizer": "adam", "loss": last_loss,
                   "step": "stage step + linear softmax cross-entropy head + Adam update of all weights"}
        del tr

    # ---- CPU baseline: the oracle on a bounded sample ---------------------------------------
    cpu = None
    if with_cpu and w.variant in ("gcn", "gcnii"):
        # level tables of a realistic range, drawn afresh (inputs, not what the library computed); this leg is timed, not compared
        tables = [cur[0]] + [dev_normal((n, dims[j]), sdt, absolute=True) for j in range(1, L)]
        cpu = cpu_baseline(w, row_ptr, col, tables, h0, dims, args.cpu_sample_rows if args.cpu_sample_rows > 0 else None)

    out = {
        "workload": f"configs[{name[1:]}] {w.name}: {'R-MAT' if w.kind == 'rmat' else 'Erdos-Renyi'} n={n} nnz={nnz} dims={dims} chunks={K} "
                    f"{w.variant} {'bf16 levels, fp32 level 0' if w.level0_f32 else w.dtype}{cut_note}{' edge weights given by the caller' if args.caller_weights else ''}",
        "max_degree": stats["max_degree"], "value": value, "unit": "edges/s", "ms_per_step": ms_per_step, "steps": steps,
        "dtype": "bf16" if bf else "f32",
        "kernel_ms_per_step": kernels_ms, "gemm": gemm, "roofline": roofline, "update_history": history, "cpu_baseline": cpu,
    }
    if trainer is not None:
        out["trainer"] = trainer
    st.gnnstage_destroy()
    del st, cur, hist, W, dW, grad_out, h0, grad_h0, grad_in
    torch.cuda.empty_cache()
    return out


def cpu_baseline(w, row_ptr, col, tables, h0, dims, sample_rows):
    """Times the CPU oracle (as it stands) on the first `sample_rows` destination rows of the same
    workload: all layers, forward + backward, half of the remaining vertices marked processed."""
    import ctypes

    import oracle
    from synth import values

    n = len(row_ptr) - 1
    L = len(dims) - 1
    if sample_rows is None:  # about 10 to 30 seconds of oracle time on the machine's cores
        sample_rows = {"c1": 131072, "c2": 306250, "c3": n // 2, "c4": 312500}.get(w.name, 131072)
    s = min(sample_rows, n // 2)
    chunk_ptr = np.array([0, s, (s + n) // 2, n], dtype=np.int64)
    t0 = time.time()
    val = oracle.gcn_norm(row_ptr, col)
    gcn = w.variant == "gcn"
    quant = w.dtype == "bf16"
    Wn = [values.glorot_uniform(w.seed, 100 + j, dims[j], dims[j + 1]) for j in range(L)]
    beta = None
    if not gcn:
        beta = np.array([math.log(0.5 / l + 1.0) for l in range(w.gcnii_first_layer, w.gcnii_first_layer + L)])
    h0n = None if h0 is None else h0.float().cpu().numpy()
    st = oracle.OracleStage(row_ptr, col, val, chunk_ptr, dims, Wn, None, variant=w.variant, a=w.gcnii_alpha,
                            beta=beta, h0=h0n, quant=quant, level0_f32=w.level0_f32)
    for j in range(L):  # one host array as current and historical level: nothing is compared here
        a = tables[j].float().cpu().numpy()
        st.cur[j] = a
        st.hist[j] = a
    st._refresh()
    log(f"[bench] oracle set-up {time.time() - t0:.1f}s")
    edges = int(row_ptr[s] - row_ptr[0])
    gout = values.normal(w.seed, 3, (s, dims[-1]))
    st.begin_pass()
    st.processed[2] = 1   # half of the other vertices count as already processed (read from cur)
    t1 = time.perf_counter()
    st.lib.oracle_forward_chunk(ctypes.byref(st._cs), 0)
    t_f = time.perf_counter() - t1
    st.bprocessed[2] = 1
    t2 = time.perf_counter()
    st.lib.oracle_backward_chunk(ctypes.byref(st._cs), 0, np.ascontiguousarray(gout).ctypes.data, 1)
    t_b = time.perf_counter() - t2
    total = t_f + t_b
    return {"value": L * edges / total, "unit": "edges/s", "cores": oracle.max_threads(), "kind": "oracle",
            "sample": f"first {s} destination rows ({edges} entries) of the same graph, all {L} layers, forward "
                      f"{t_f:.2f}s + backward {t_b:.2f}s, half of the other vertices marked processed",
            "seconds": round(total, 2)}


def cpu_full(name, threads):
    """Times the CPU oracle as it stands on ONE WHOLE configuration: a complete forward pass over all chunks (shuffled
    order) and the complete backward pass, at the configuration's own size, with `threads` host threads.  Level tables
    are random (the time does not depend on their values); nothing is compared here."""
    import oracle
    from synth import values
    from synth.configs import CONFIGS, make_graph
    from synth.graphs import equal_chunks

    w = CONFIGS[name]
    row_ptr, col = make_graph(w)
    n, nnz = len(row_ptr) - 1, int(row_ptr[-1])
    K, L, dims = w.n_chunks, w.n_layers, list(w.dims)
    chunk_ptr = equal_chunks(n, K)
    gcn = w.variant == "gcn"
    val = oracle.gcn_norm(row_ptr, col)
    Wn = [values.glorot_uniform(w.seed, 100 + j, dims[j], dims[j + 1]) for j in range(L)]
    beta = None if gcn else np.array([math.log(0.5 / l + 1.0) for l in range(w.gcnii_first_layer, w.gcnii_first_layer + L)])
    rng = np.random.default_rng(w.seed)
    h0 = None if gcn else rng.standard_normal((n, dims[0]), dtype=np.float32)
    if threads > 0:
        oracle.set_threads(threads)
    st = oracle.OracleStage(row_ptr, col, val, chunk_ptr, dims, Wn, None, variant=w.variant, a=w.gcnii_alpha, beta=beta,
                            h0=h0, quant=w.dtype == "bf16", level0_f32=w.level0_f32)
    for j in range(L):  # one host array as current and historical level
        a = np.abs(rng.standard_normal((n, dims[j]), dtype=np.float32))
        st.cur[j] = a
        st.hist[j] = a
    st._refresh()
    order = [int(k) for k in values.permutation(w.seed, 1000, K)]
    gout = rng.standard_normal((n, dims[-1]), dtype=np.float32)
    first_stage = gcn if w.first_stage is None else w.first_stage
    t0 = time.perf_counter()
    st.begin_pass()
    for k in order:  # a line per chunk: a whole pass takes minutes on the larger configurations
        st.forward_chunk(k)
        log(f"[bench]   {name} forward chunk {k} done at {time.perf_counter() - t0:.1f}s")
    t_f = time.perf_counter() - t0
    t1 = time.perf_counter()
    for k in reversed(order):
        st.backward_chunk(k, np.ascontiguousarray(gout[st.rows(k)]), need_input_grad=not first_stage)
        log(f"[bench]   {name} backward chunk {k} done at {time.perf_counter() - t1:.1f}s")
    t_b = time.perf_counter() - t1
    return {"workload": name, "n": n, "nnz": nnz, "layers": L, "chunks": K, "threads": oracle.max_threads(),
            "forward_s": round(t_f, 2), "backward_s": round(t_b, 2), "edges_per_s": L * nnz / (t_f + t_b), "kind": "oracle"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default=HEADLINE, help="headline configuration (default: the largest one, c4)")
    ap.add_argument("--only", action="store_true", help="time the headline configuration only (no per_config object)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--event-every", type=int, default=4,
                    help="the aggregation launches of every N-th timed step carry HIP events (1: of every step)")
    ap.add_argument("--cpu-sample-rows", type=int, default=0, help="0: a sample sized to about 10-30 s of oracle time")
    ap.add_argument("--partition", action="store_true",
                    help="chunks from the library's locality-aware partitioner instead of index ranges (not the benchmark configuration)")
    ap.add_argument("--partition-by-entries", action="store_true", help="with --partition: balance the chunks by entries")
    ap.add_argument("--caller-weights", action="store_true",
                    help="hand the edge weights to the library (edge_val) instead of letting it compute the normalisation: "
                         "dense blocks then run from stored weight tiles instead of bit patterns")
    ap.add_argument("--train-epochs", type=int, default=0,
                    help="also time this many epochs of the whole training loop (head + Adam) around the same stage")
    ap.add_argument("--history-swap", action="store_true",
                    help="refresh the history with gnnstage_update_history_swap (levels trade buffers, nothing is copied) "
                         "instead of update_history; not the default line")
    ap.add_argument("--cpu-full", default="",
                    help="no GPU work: time the CPU oracle on whole configurations instead (comma-separated names, "
                         "e.g. c0,c1,c2,c3; a name with ':1' appended runs on one thread) and print one JSON line")
    args = ap.parse_args()
    if args.cpu_full:
        import oracle
        all_threads = oracle.max_threads()
        res = []
        for item in args.cpu_full.split(","):
            nm, _, th = item.partition(":")
            log(f"[bench] CPU oracle on all of {nm} ...")
            res.append(cpu_full(nm, int(th) if th else all_threads))
            log(f"[bench] {res[-1]}")
        print(json.dumps({"cpu_baseline_full": res}))
        return
    if args.gpus != 1:
        sys.exit("bench.py measures one pipeline stage on ONE GPU; this build has no multi-GPU path (--gpus must be 1)")

    import torch
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    copy_gbs = copy_bandwidth(torch, "cuda:0")
    log(f"[bench] plain device copy on this box: {copy_gbs:.0f} GB/s (read + written)")

    head = run_config(args.workload, args, args.steps, args.warmup, not args.no_cpu_baseline, copy_gbs)
    per_config = {}
    if not args.only and args.workload == HEADLINE and not (args.partition or args.caller_weights or args.train_epochs or args.history_swap):
        for name in SECONDARY:
            r = run_config(name, args, args.steps, args.warmup, False, copy_gbs)
            per_config[name] = {k: r[k] for k in ("workload", "value", "unit", "ms_per_step", "steps", "dtype", "kernel_ms_per_step",
                                                  "gemm", "roofline", "update_history")}
    out = {
        "metric": "layer-stage fwd+bwd edges/sec per MI355X", "value": head["value"], "unit": "edges/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": head["dtype"], "data": "synthetic",
        "config": {"workload": head["workload"], "max_degree": head["max_degree"],
                   "step": "forward all chunks + backward all chunks + " +
                           ("gnnstage_update_history_swap (levels trade buffers)" if args.history_swap else "update_history")},
        "kernel_ms_per_step": head["kernel_ms_per_step"],
        "gemm": head["gemm"],
        "update_history": head["update_history"],
        "roofline": head["roofline"],
        "cpu_baseline": head["cpu_baseline"],
    }
    if per_config:
        out["per_config"] = per_config
    if "trainer" in head:
        out["trainer"] = head["trainer"]
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
