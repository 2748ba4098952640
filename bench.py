#!/usr/bin/env python3
"""Benchmark of the whole mini-batch step (sdt_train_loop / sdt_train_step) on one MI355X.

A "step" is one pass of the hot path -- sample, gather, forward, loss, backward,
SGD -- over one seeded synthetic mini-batch.  The default workload is the
dense-neighbourhood one (Chung-Lu 2^18 nodes, degree ~470, F=602, 41 classes,
2-layer GraphSAGE-mean with hidden 256, fan-out [25,10], 1024 seeds): the largest
fp32 step, where the kernels are long enough for their bandwidth and matrix-core
fractions to mean something; the products-shaped step (latency-bound everywhere)
is measured after it and reported under "also"; `--workload` selects any other.
Graph, features, labels, weights and all seed batches are resident in HBM before
a timed region starts.  The value is the median of `--reps` repetitions of one
K-step loop call, each from the same initial weights, and every loss of the
timed loops is checked against K sequential single-step calls.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_FP32_PEAK_TFLOPS = 157.3  # MI355X dense fp32 matrix, published
MFMA_BF16_PEAK_TFLOPS = 2500.0 # MI355X dense bf16 matrix, published

STEP_WORKLOADS = ["tiny", "products", "products_spring", "dense", "sparse_bf16"]


def log(msg):
    print(msg, file=sys.stderr, flush=True)


def measured_traffic(workload, kernel, rank=0):
    """HBM bytes per launch (read + written) of `kernel` from profiles/traffic.json: the rocprofv3 --pmc
    FETCH_SIZE / WRITE_SIZE figures that paper_2404_02300_amd/profile_summary.py wrote from a counter run
    of this workload.  The file names the hash of the kernel sources it was measured with; when the tree's
    sources hash differently (or there is no entry) the answer is None: a figure from another build is not
    reported as this run's.  `rank`: which of the kernel's launch sizes, largest first (layer 0 is the largest)."""
    try:
        from paper_2404_02300_amd import profile_summary as ps
        if not os.path.exists(ps.TRAFFIC):
            return None
        e = json.load(open(ps.TRAFFIC)).get(workload)
        if not e or e.get("sources_hash") != ps.sources_hash():
            return None
        hits = sorted(((v["read_bytes"] + v["written_bytes"], k) for k, v in e["kernels"].items()
                       if k.startswith(kernel)), reverse=True)
        if rank >= len(hits):
            return None
        return {"bytes": round(hits[rank][0]), "kernel": hits[rank][1], "from": e.get("summary")}
    except Exception as ex:       # a broken table must not break the measurement
        log(f"[bench] traffic table unreadable: {ex}")
        return None


def measured_traffic_sum(workload, prefix):
    """The same for every launch size of every kernel whose name starts with `prefix`, summed (a stage made
    of several launches)."""
    total, names, k = 0, [], 0
    while True:
        t = measured_traffic(workload, prefix, k)
        if t is None:
            break
        total += t["bytes"]
        names.append(t["kernel"])
        src = t["from"]
        k += 1
    return {"bytes": total, "kernel": " + ".join(names), "from": src} if names else None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None,
                    help="timed steps per repetition (default: the number the workload prescribes: 100, or 200 for sparse_bf16)")
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--reps", type=int, default=3,
                    help="repetitions of the timed region, each from the same initial weights; the median is reported")
    ap.add_argument("--workload", default="dense",
                    choices=STEP_WORKLOADS + ["fullgraph", "sampling", "gather"],
                    help="default: dense, the largest fp32 training step (where the bandwidth and matrix-core fractions "
                         "show); 'sampling' / 'gather' time that stage alone at a size where it is bandwidth-bound")
    ap.add_argument("--also", default="products",
                    help="comma-separated further step workloads measured after the main one (steps/s and the loss check only; "
                         "'none' to skip); ignored unless the main workload is the default")
    ap.add_argument("--model", default="sage", choices=["sage", "gcn", "gat"],
                    help="gcn / gat: the same step with the GCN or GAT model kind (not the headline metric)")
    ap.add_argument("--lr", type=float, default=0.01)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--serial", action="store_true", help="no auxiliary stream: every step strictly in sequence")
    ap.add_argument("--aux", type=int, default=2, help="auxiliary streams the sampling phase alternates between")
    ap.add_argument("--cpu-seconds", type=float, default=12.0,
                    help="the oracle is timed on whole steps until this many seconds have passed (at least one step)")
    ap.add_argument("--roofline-stage", default=None,
                    help="kernel-level stage to time inside the loop instead of the longest one, as kind:layer "
                         "(e.g. linear_fwd:0, bwd_weight:0); for diagnosis")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="first run one plain 1 GiB device copy (a reference dispatch for rocprofv3 --pmc runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on ONE GPU (the per-worker step has no collectives); --gpus must be 1")
        sys.exit(2)

    import torch
    import sdt_gen as gen

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    wl = gen.WORKLOADS["products" if args.workload in ("sampling", "gather", "products_spring") else args.workload]
    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")     # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if args.workload == "fullgraph":
        args.steps = args.steps or 20
        return bench_fullgraph(args, wl)
    if args.workload in ("sampling", "gather"):
        args.steps = args.steps or 20
        return bench_stage_at_scale(args, wl)
    # the auxiliary streams are created once and shared by every workload of the run: a process has four
    # hardware queues, and a fifth stream would share one with the main stream
    args.aux_streams = None if args.serial else [torch.cuda.Stream() for _ in range(max(1, min(3, args.aux)))]
    out = bench_step(args, args.workload, full=True)
    also = [w for w in args.also.split(",") if w and w != "none"]
    if args.workload == "dense" and args.model == "sage" and also:
        out["also"] = []
        for w in also:
            if w not in STEP_WORKLOADS or w == args.workload:
                continue
            r = bench_step(args, w, full=False)
            out["also"].append({k: r[k] for k in ("value", "unit", "steps", "repetitions", "ms_per_step", "dtype", "config",
                                                  "loss_check", "sampled_edges_per_s", "roofline")})
    print(json.dumps(out), flush=True)


def bench_step(args, workload, full):
    """Steps/s of `workload` through sdt_train_loop (median of args.reps repetitions of K steps, each from
    the same initial weights), the loss check against K sequential sdt_train_step calls, per-kernel HIP-event
    times, the roofline entry of the longest kernel and (full) the oracle on the host."""
    import numpy as np
    import torch
    import sdt_gen as gen
    import paper_2404_02300_amd as sdt

    t0 = time.time()
    # products_spring: the products-shaped graph cut into four partitions by the paper's streaming
    # partitioner; the step runs on partition 0 (owned nodes + replicas), seeds from its owned nodes
    spring = workload == "products_spring"
    wl = gen.WORKLOADS["products" if spring else workload]
    K = args.steps if args.steps is not None else (wl.steps if wl.steps > 1 else 100)
    Wm, R = args.warmup, max(1, args.reps)
    inst = gen.make_partition_instance(wl, p=4, which=0) if spring else gen.make_instance(wl)
    nnz_graph = int(inst.indptr[-1])
    log(f"[bench] generated {workload}: N={inst.n_nodes} nnz={nnz_graph} avg_deg={nnz_graph / inst.n_nodes:.2f} "
        f"in {time.time() - t0:.1f}s" + (f" {inst.info}" if spring else ""))

    graph = sdt.Csr(torch.from_numpy(inst.indptr).cuda(), torch.from_numpy(inst.indices).cuda())
    if wl.bf16:
        X = torch.from_numpy(inst.X.view(np.int16)).cuda().view(torch.bfloat16)
    else:
        X = torch.from_numpy(inst.X).cuda()
    y = torch.from_numpy(inst.y).cuda()
    gat = args.model == "gat"
    gcn = args.model == "gcn" or gat      # one weight matrix per layer
    att_h = att = None
    if gcn:     # one [in, out] matrix per layer, Glorot-uniform from the workload's seed
        rng = np.random.default_rng(wl.seed)
        Wh = [(rng.uniform(-1, 1, size=(wl.dims[l], wl.dims[l + 1])) *
               np.sqrt(6.0 / (wl.dims[l] + wl.dims[l + 1]))).astype(np.float32) for l in range(len(wl.fanouts))]
        if gat:  # attention vectors [a_src | a_dst] per layer
            att_h = [(rng.uniform(-1, 1, size=2 * wl.dims[l + 1]) * np.sqrt(6.0 / (wl.dims[l + 1] + 1))).astype(np.float32)
                     for l in range(len(wl.fanouts))]
            att = [torch.from_numpy(v).cuda() for v in att_h]
    else:
        Wh = inst.W
    W = [torch.from_numpy(w).cuda() for w in Wh]
    b = [torch.from_numpy(v).cuda() for v in inst.b]
    params = W + b + (att or [])
    params0 = [p.clone() for p in params]

    def restore():
        for p, p0 in zip(params, params0):
            p.copy_(p0)

    model = sdt.make_model(wl.dims, W, b, kind=sdt.SDT_MODEL_GAT if gat else sdt.SDT_MODEL_GCN if gcn else sdt.SDT_MODEL_SAGE_MEAN,
                           att=att)
    code = sdt.SDT_BF16 if wl.bf16 else sdt.SDT_F32
    lay = sdt.sdt_train_step_layout(graph.n_nodes, wl.batch, wl.fanouts, model, code)
    ws = torch.empty(sdt.sdt_train_loop_workspace_bytes(graph.n_nodes, wl.batch, wl.fanouts, model, code),
                     dtype=torch.uint8, device="cuda")
    loss = torch.zeros(1, dtype=torch.float32, device="cuda")
    losses = torch.zeros(Wm + K, dtype=torch.float32, device="cuda")
    seeds_all = torch.from_numpy(np.stack([inst.batch(s) for s in range(Wm + K)])).cuda()
    aux = args.aux_streams
    L = len(wl.fanouts)
    es = 2 if wl.bf16 else 4

    def run_loop(first, count, timing=None):
        # one native call enqueues `count` whole steps; the sampling phase of a step runs on the
        # auxiliary streams, ahead of the forward/backward phase of the previous ones
        sdt.sdt_train_loop(graph, X, y, seeds_all[first:first + count], wl.fanouts, model, wl.seed, first, args.lr,
                           losses[first:first + count], ws, aux, timing)

    # ---- stages: the coarse ones (a stage may span several launches) and the single launches inside them
    coarse = [("sample", l) for l in range(L)] + [("loss", 0)] + [("linear_bwd", l) for l in range(L)]
    kernels = [("sample_rows", l) for l in range(L)] + [("front_scan", l) for l in range(L)] + \
              [("front_apply", l) for l in range(L)] + [("relabel", l) for l in range(L)] + \
              ([] if gcn and not gat else [("gather", 0)]) + [("aggregate_fwd", l) for l in range(L)] + \
              [("linear_fwd", l) for l in range(L)] + [("head", L - 1)] + [("bwd_weight", l) for l in range(L)] + \
              [("bwd_input", l) for l in range(1, L)] + [("update", 0)]
    if not gat:
        kernels += [("aggregate_bwd", l) for l in range(1, L)]
        # the transposed block of a small layer is one launch (the general path, five launches, stays a coarse stage)
        small_t = [l for l in range(1, L) if lay.cap_nnz[l] <= (1 << 14)]
        kernels += [("transpose", l) for l in small_t]
        coarse += [("transpose", l) for l in range(1, L) if l not in small_t]
    else:
        coarse += [("aggregate_bwd", l) for l in range(L)] + [("transpose", l) for l in range(L)]
    stages = coarse + kernels

    def staged_pass(first, count, timed, with_counts):
        """`count` sequential sdt_train_step calls (untimed by the wall clock); the first `timed` of them with
        every stage bracketed by HIP events.  Returns mean stage times, block sizes of the timed steps, all losses."""
        t = sdt.Timing(max(1, timed), stages)
        cnts, ls = [], torch.zeros(count, dtype=torch.float32, device="cuda")
        for i in range(first, first + count):
            sdt.sdt_train_step(graph, X, y, seeds_all[i], wl.fanouts, model, wl.seed, i, args.lr, ls[i - first:], ws,
                               t if i - first < timed else None)
            if with_counts and i - first < timed:
                torch.cuda.synchronize()
                cnts.append([sdt.ws_view(ws, lay.counts[l], (4,), torch.int32).cpu().tolist() for l in range(L)])
        torch.cuda.synchronize()
        ms = {}
        for k, l in stages:
            try:
                ms[(k, l)] = float(np.mean(t.read(k, l)))
            except sdt.SdtError:    # stage not run separately (e.g. folded into the fused last layer)
                pass
        t.close()
        return ms, np.array(cnts), ls.cpu().tolist()

    # ---- warm-up (W pipelined steps, then a short staged pass that finds the longest kernel)
    run_loop(0, Wm)
    pre_ms, _, _ = staged_pass(0, min(5, Wm + K), min(5, Wm + K), False)
    dominant = max((k for k in pre_ms if k in kernels), key=pre_ms.get)   # the longest single launch of a step
    if args.roofline_stage and full:
        kind, layer = args.roofline_stage.split(":")
        dominant = (kind, int(layer))
        assert dominant in pre_ms, f"stage {dominant} did not run; stages: {sorted(pre_ms)}"

    # one untimed pass of the same K steps first: a short loop after an idle stretch (graph generation, the
    # host oracle of an earlier workload) would otherwise be timed while the clocks are still coming up
    run_loop(Wm, K)
    torch.cuda.synchronize()

    # ---- the timed region, R times from the same initial weights: exactly K steps between two
    # synchronisations; only the dominant kernel is bracketed by HIP events (on the stream it is launched on)
    elapsed, dom_ms, rep_losses = [], [], []
    for r in range(R):
        restore()
        tim = sdt.Timing(K, [dominant], stride=8)    # every 8th launch: an event record costs the stream microseconds
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run_loop(Wm, K, tim)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        elapsed.append(t1 - t0)
        dom_ms.append(float(np.mean(tim.read(*dominant))))
        tim.close()
        rep_losses.append(losses[Wm:Wm + K].cpu().tolist())
    order = sorted(range(R), key=lambda r: elapsed[r])
    med = order[R // 2]
    t_med = elapsed[med]
    assert all(rl == rep_losses[0] for rl in rep_losses), "the repetitions of the timed loop did not reproduce each other's losses"
    final_loss = rep_losses[0][-1]

    # ---- loss check + diagnostic pass (untimed): the same K batches from the same initial weights through
    # K sequential sdt_train_step calls; every loss must equal the timed loop's bit for bit
    restore()
    nd = min(K, 20)
    stage_t, counts, seq_losses = staged_pass(Wm, K, nd, True)        # counts: [nd, L, 4] = n_dst, n_src, nnz, 0
    bad = [i for i in range(K) if seq_losses[i] != rep_losses[0][i]]
    assert not bad, (f"losses of the timed loop differ from {K} sequential sdt_train_step calls at steps {bad[:8]}: "
                     f"{[rep_losses[0][i] for i in bad[:4]]} vs {[seq_losses[i] for i in bad[:4]]}")
    loss_check = (f"all {K} losses of each of the {R} timed repetitions bit-equal to {K} sequential sdt_train_step calls "
                  f"from the same initial weights (final loss {final_loss:.6f})")
    mean_cnt = counts.mean(axis=0)
    edges_per_step = float(counts[:, :, 2].sum(axis=1).mean())
    n_src0 = mean_cnt[0][1]
    d = wl.dims
    N = inst.n_nodes

    # fp32 GraphSAGE layers with a wide output, a long reduction and few row tiles run on the bf16 matrix cores through
    # exact three-way splits (csrc/linear_x3.hip; the predicates are x3_fwd_wanted / x3_dw_wanted there)
    def x3_fwd(l):
        return (not wl.bf16 and not gcn and not gat and l < L - 1 and 128 < d[l + 1] <= 256 and d[l + 1] % 4 == 0
                and d[l] >= 256 and lay.cap_dst[l] >= 2048 and (lay.cap_dst[l] + 127) // 128 <= 256)

    def x3_dw(l):
        return (not wl.bf16 and not gcn and not gat and 128 < d[l + 1] <= 256 and d[l] >= 128 and lay.cap_dst[l] >= 2048
                and 2 * ((d[l] + 127) // 128) <= 64 and not (l == L - 1 and ("head", l) in stage_t))

    def work(kind, l):
        """Algorithmic work of one launch of a stage: (bound, amount, kernel name)."""
        n_dst, n_src, nnz = mean_cnt[l][:3]
        wf = 1.0 if gcn else 2.0      # rows of W per input feature: GraphSAGE stacks a self and a neighbour block
        if gat:     # every frontier row is gathered and projected; the attention passes read projected rows
            F = d[l + 1]
            if kind == "gather":
                return "hbm", n_src * (2 * d[0] * es + 4), "k_gather"
            if kind == "aggregate_fwd":   # scores over every source row, then two score passes and one row pass per edge
                return "hbm", n_src * F * es + nnz * (F * es + 12) + n_dst * (2 * F * es + 16), "k_gat_scores + k_gat_fwd"
            if kind == "aggregate_bwd":   # two dot-product passes per edge on each side + the weighted sums
                return "hbm", nnz * (5 * F * es + 16) + n_src * 3 * F * es + n_dst * 3 * F * es, \
                       "k_gat_mask_bias + k_gat_bwd_dst + k_gat_bwd_src + k_gat_vec_partials"
            if kind == "linear_fwd":
                return "mfma", 2.0 * n_src * d[l] * F, "k_linear_fwd"
            if kind in ("linear_bwd", "bwd_weight", "bwd_input"):
                f = 2.0 * n_src * d[l] * F
                return "mfma", f * (2 if l > 0 and kind == "linear_bwd" else 1), \
                       {"linear_bwd": "k_linear_bwd_weight (+ _input)", "bwd_weight": "k_linear_bwd_weight",
                        "bwd_input": "k_linear_bwd_input"}[kind]
        if kind == "sample":      # 16 B of row offsets per destination, 4 B read + 4 B written per sampled edge
            return "hbm", n_dst * 16 + nnz * 8, "k_sample_rows + frontier scan + relabel (+ transposed block)"
        if kind == "sample_rows":     # + one mark byte per sampled edge
            return "hbm", n_dst * 16 + nnz * 9, "k_sample_rows"
        if kind == "front_scan":      # mark bytes and state bits of every node, and the per-row counts, read once
            return "hbm", N * 1.25 + n_dst * 4, "k_front_partials"
        if kind == "front_apply":     # the same again, plus row offsets, the new frontier ids and their map entries
            return "hbm", N * 1.25 + n_dst * 12 + (n_src - n_dst) * 8, "k_front_apply"
        if kind == "relabel":         # global id in, state word and rank (or map entry) in, local id out
            return "hbm", nnz * 16, "k_relabel"
        if kind == "transpose":       # row offsets and column ids in, source offsets and destination rows out
            return "hbm", nnz * 8 + n_dst * 4 + n_src * 8, "k_transpose_parts" if lay.cap_nnz[l] <= (1 << 14) else \
                   "k_scan_partials + k_scan_apply + k_transpose_fill + k_sort_short + k_sort_long"
        if kind == "update":          # every layer's partial products read once, weights and gradients written
            return "hbm", float(sum(wf * d[j] * d[j + 1] * 4 * 8 for j in range(L))), "k_reduce_partials"
        if kind == "gather":      # only the destination prefix is copied; the rest is read by the aggregation
            return "hbm", n_dst * (2 * d[0] * es + 4), "k_gather"
        if kind == "aggregate_fwd":   # layer 0 reads X through src_nodes: 4 more index bytes per edge
            return "hbm", nnz * (d[l] * es + (8 if l == 0 else 4)) + n_dst * (d[l] * es + 8), \
                   "k_gcn_aggregate_fwd" if gcn else "k_aggregate_fwd"
        if kind == "aggregate_bwd":
            return "hbm", nnz * (d[l] * es + 4) + n_src * (d[l] * es + 8) + n_dst * d[l] * es, \
                   "k_gcn_aggregate_bwd" if gcn else "k_aggregate_bwd"
        if kind == "linear_fwd":
            # bf16 workloads: the products run on the bf16 matrix cores, but the layer is below their ridge
            # (2.5 PFLOP/s / 8 TB/s = 312 flop/B against ~128 flop/B here), so it is priced by the bytes it
            # must move: both operands and the weights in, the output rows out
            if wl.bf16:
                return "hbm", n_dst * (wf * d[l] + d[l + 1]) * es + wf * d[l] * d[l + 1] * 2, \
                       "k_linear_fwd (bf16 operands widened on the way into LDS)" if gcn else "k_fwd_bf16"
            return "mfma", 2.0 * n_dst * wf * d[l] * d[l + 1], \
                   "k_linear_fwd_x3 (+ k_linear_fwd_x3_finish after it; k_x3_transpose_w before it in a step on its own)" \
                   if x3_fwd(l) else "k_linear_fwd"
        if kind in ("linear_bwd", "bwd_weight", "bwd_input"):
            f = 2.0 * n_dst * wf * d[l] * d[l + 1]
            if wl.bf16:   # as the forward: operands in, partial products / input gradients out
                by_w = n_dst * (2 * d[l] + d[l + 1]) * es + 2 * d[l] * d[l + 1] * 4
                by_i = n_dst * (d[l + 1] + 2 * d[l]) * es + 2 * d[l] * d[l + 1] * 2
                return "hbm", {"linear_bwd": by_w + (by_i if l > 0 else 0), "bwd_weight": by_w, "bwd_input": by_i}[kind], \
                       {"linear_bwd": "k_bwd_weight_bf16 (+ k_bwd_input_bf16)", "bwd_weight": "k_bwd_weight_bf16",
                        "bwd_input": "k_bwd_input_bf16"}[kind]
            if kind == "linear_bwd" and l == L - 1 and ("head", l) in stage_t:   # projection + softmax + dW + input gradients
                return "mfma", f * (3 if l > 0 else 2), "k_head"
            wname = "k_linear_bwd_weight_x3" if x3_dw(l) else "k_linear_bwd_weight"
            return "mfma", f * (2 if l > 0 and kind == "linear_bwd" else 1), \
                   {"linear_bwd": wname + " (+ _input)", "bwd_weight": wname, "bwd_input": "k_linear_bwd_input"}[kind]
        if kind == "head":        # projection + dW (+ input gradients) of the last layer, one launch
            return "mfma", 2.0 * n_dst * wf * d[l] * d[l + 1] * (3 if l > 0 else 2), "k_head"
        return "hbm", wl.batch * d[L] * 8, "k_softmax_xent"

    def rate(kind, l, seconds):
        bound, amount, kname = work(kind, l)
        if bound == "hbm":
            ach, peak, unit = amount / seconds / 1e9, HBM_PEAK_GBS, "GB/s"
        else:
            ach, peak, unit = amount / seconds / 1e12, MFMA_FP32_PEAK_TFLOPS, "TFLOP/s"
        r = {"stage": f"{kind}[{l}]", "kernel": kname, "bound": bound, "achieved": round(ach, 2), "peak": peak,
             "unit": unit, "frac": round(ach / peak, 4), "algorithmic_per_launch": float(amount),
             "avg_launch_us": round(seconds * 1e6, 2)}
        if "_x3" in kname:   # priced as what it computes: the fp32 product, against the fp32 matrix peak
            r["matrix_path"] = ("fp32 operands as exact sums of three bf16, six v_mfma_f32_32x32x16_bf16 per fp32 product "
                                "block; algorithmic fp32 flops over the published fp32 matrix peak")
        return r

    # roofline of the longest kernel, from the events recorded inside the timed region (median repetition)
    roofline = rate(dominant[0], dominant[1], dom_ms[med] * 1e-3)
    roofline["avg_launch_us_serial"] = round(stage_t.get(dominant, float("nan")) * 1e3, 2)   # the same kernel with nothing beside it
    tr = None
    if args.model == "sage":
        same = sorted((l for (k, l) in stage_t if k == dominant[0]), key=lambda l: -work(dominant[0], l)[1])
        tr = measured_traffic(workload, work(*dominant)[2].split()[0], same.index(dominant[1]) if dominant[1] in same else 0)
    roofline["traffic"] = tr["bytes"] if tr else None
    roofline["traffic_from"] = (f"{tr['from']}: {tr['kernel']}" if tr else
                                "no counter run of this build's kernel sources in profiles/traffic.json")
    stage_ms = {f"{k}[{l}]": v for (k, l), v in stage_t.items()}
    others = [rate(k, l, v * 1e-3) for (k, l), v in stage_t.items() if (k, l) in kernels]

    # ---- CPU baseline: the oracle as it stands, one thread, on a bounded sample of the same workload
    cpu = None
    if full and not args.no_cpu_baseline:
        from oracle import sdt_oracle as orc
        ns = 0
        tc = time.perf_counter()
        while ns == 0 or (time.perf_counter() - tc < args.cpu_seconds and ns < min(K, 32)):
            s = ns
            if gat:
                orc.gat_train_step(inst.indptr, inst.indices, inst.X, inst.y, inst.batch(s), wl.fanouts, Wh, inst.b, att_h,
                                   wl.seed, s, args.lr, bf16=wl.bf16)
            elif gcn:
                orc.gcn_train_step(inst.indptr, inst.indices, inst.X, inst.y, inst.batch(s), wl.fanouts, Wh, inst.b,
                                   wl.seed, s, args.lr, bf16=wl.bf16)
            else:
                orc.train_step(inst.indptr, inst.indices, inst.X, inst.y, inst.batch(s), wl.fanouts, inst.W, inst.b,
                               wl.seed, s, args.lr, bf16=wl.bf16)
            ns += 1
        tc = time.perf_counter() - tc
        cores = 1
        if gcn:     # the GCN oracle's projections are numpy matrix products: count the BLAS threads
            try:
                from threadpoolctl import threadpool_info
                cores = max([1] + [int(p.get("num_threads", 1)) for p in threadpool_info()])
            except Exception:
                cores = os.cpu_count()
        cpu = {"value": round(ns / tc, 4), "unit": "steps/s", "cores": cores, "kind": "oracle",
               "sample": f"{ns} full mini-batch steps of the same workload (batches 0..{ns - 1}, initial weights), {tc:.1f} s",
               "host_cpus": os.cpu_count()}

    return {
        "metric": "train steps/s per GPU (sample + gather + forward + backward + SGD)" + (" [GAT model kind]" if gat else " [GCN model kind]" if gcn else ""),
        "value": round(K / t_med, 2), "unit": "steps/s", "n_gpus": 1, "steps": K, "warmup": Wm, "repetitions": R,
        "ms_per_step": round(t_med / K * 1e3, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16" if wl.bf16 else "f32", "data": "synthetic",
        "config": {"workload": (f"{wl.name}: {wl.kind} 2^{wl.log2n} nodes, {nnz_graph} CSR entries, " if not spring else
                                f"products_spring: partition 0 of 4 of the {wl.kind} 2^{wl.log2n} graph without isolated nodes "
                                f"(streaming partitioner, beta 1.05): {inst.n_owned} owned + {inst.n_nodes - inst.n_owned} replica "
                                f"nodes, {nnz_graph} CSR entries, ") + f"F={wl.feat}, "
                               f"C={wl.classes}, {L}-layer {'GAT' if gat else 'GCN' if gcn else 'GraphSAGE-mean'} hidden {wl.hidden}, fanout {wl.fanouts}, "
                               f"batch {wl.batch}, seeds from " + ("the owned nodes" if spring else f"the first {wl.owned_frac:g} of the ids"),
                   "lr": args.lr, "seed": wl.seed},
        "value_is": f"median of {R} repetitions of one {K}-step sdt_train_loop call",
        "steps_per_s_all_repetitions": [round(K / e, 2) for e in elapsed],
        "sampled_edges_per_s": round(edges_per_step * K / t_med, 1),
        "sampled_edges_per_step": round(edges_per_step, 1),
        "frontier_rows_per_step": round(float(n_src0), 1),
        "final_loss": round(final_loss, 6), "loss_check": loss_check,
        "overlap": "serial" if args.serial else f"sampling of the next steps on {len(aux)} auxiliary stream(s)",
        "roofline": roofline, "cpu_baseline": cpu,
        "stage_ms": {k: round(v, 4) for k, v in stage_ms.items()}, "kernel_rates": others,
    }


def bench_stage_at_scale(args, wl):
    """The sampling stage (sdt_sample_csr: neighbour sampling, frontier, relabelling) or the feature
    gather alone, with every owned node of the products-shaped graph as a destination: the mini-batch
    steps move so little per launch that these stages are latency-bound there; this shows what the
    same kernels sustain once a launch is large."""
    import numpy as np
    import torch
    import sdt_gen as gen
    import paper_2404_02300_amd as sdt

    K, Wm = min(args.steps, 20), min(args.warmup, 3)
    indptr, indices = gen.make_graph(wl)
    N, nnz = wl.n_nodes, int(indptr[-1])
    n_dst = int(N * wl.owned_frac)
    fanout = wl.fanouts[0]
    g = sdt.Csr(torch.from_numpy(indptr).cuda(), torch.from_numpy(indices).cuda())
    dst = torch.arange(n_dst, dtype=torch.int32, device="cuda")
    blk = sdt.Block(n_dst, fanout, N, "cuda", transposed=False)
    ws = torch.empty(sdt.sdt_sample_workspace_bytes(N, n_dst, fanout), dtype=torch.uint8, device="cuda")
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(K)]
    if args.workload == "sampling":
        def run(i):
            sdt.sdt_sample_csr(g, dst, fanout, wl.seed, i, 0, blk, ws)
    else:
        sdt.sdt_sample_csr(g, dst, fanout, wl.seed, 0, 0, blk, ws)      # a frontier to gather
        torch.cuda.synchronize()
        n_src = int(blk.counts[1].item())
        X = torch.from_numpy(gen.normal_features(N, wl.feat, wl.seed)).cuda()
        out = torch.empty(n_src, wl.feat, dtype=torch.float32, device="cuda")
        idx = blk.src_nodes[:n_src]

        def run(i):
            sdt.sdt_gather_features(X, idx, out)
    for i in range(Wm):
        run(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(K):
        ev[i][0].record()
        run(Wm + i)
        ev[i][1].record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    sec = float(np.mean([e[0].elapsed_time(e[1]) for e in ev])) * 1e-3
    cnt = blk.counts.cpu().tolist()
    if args.workload == "sampling":
        amount = cnt[0] * 16 + cnt[2] * 8          # two row offsets per destination, 4 B read + 4 B written per edge
        units, unit_name, kern = cnt[2], "sampled edges/s", "k_sample_rows + frontier scan + relabel"
    else:
        amount = cnt[1] * (2 * wl.feat * 4 + 4)
        units, unit_name, kern = cnt[1], "gathered rows/s", "k_gather"
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import sdt_oracle as orc
        m = 1 << 15          # a bounded sample: the first 2^15 destinations
        tc = time.perf_counter()
        b = orc.sample_block(indptr, indices, np.arange(m, dtype=np.int32), fanout, wl.seed, 0, 0)
        if args.workload == "gather":
            orc.gather_rows(gen.normal_features(N, wl.feat, wl.seed), b.src_nodes)
        tc = time.perf_counter() - tc
        cpu = {"value": round((b.nnz if args.workload == "sampling" else b.n_src) / tc, 1), "unit": unit_name, "cores": 1,
               "kind": "oracle", "sample": f"the first {m} destination rows of the same launch", "host_cpus": os.cpu_count()}
    tr = measured_traffic_sum(args.workload, "k_")
    out_json = {
        "metric": f"{unit_name} of the {args.workload} stage alone ({cnt[0]} destination rows, fan-out {fanout})",
        "value": round(units / sec, 1), "unit": unit_name, "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": round(elapsed / K * 1e3, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int32" if args.workload == "sampling" else "f32", "data": "synthetic",
        "config": {"workload": f"{args.workload} stage on products: {wl.kind} 2^{wl.log2n} nodes, {nnz} CSR entries, "
                               f"{cnt[0]} destinations, {cnt[1]} frontier rows, {cnt[2]} sampled edges"},
        "roofline": {"kernel": kern, "bound": "hbm", "achieved": round(amount / sec / 1e9, 1), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(amount / sec / 1e9 / HBM_PEAK_GBS, 4),
                     "traffic": tr["bytes"] if tr else None,
                     "traffic_from": f"{tr['from']}: {tr['kernel']}" if tr else "no counter run of this build's kernel sources in profiles/traffic.json",
                     "algorithmic_bytes_per_launch": int(amount), "avg_launch_us": round(sec * 1e6, 1)},
        "cpu_baseline": cpu,
    }
    print(json.dumps(out_json), flush=True)


def bench_fullgraph(args, wl):
    """One full-neighbour GraphSAGE-mean layer over every node of the graph (layer-wise
    inference): segmented-mean SpMM over the whole CSR, then the [x | mean] projection."""
    import numpy as np
    import torch
    import sdt_gen as gen
    import paper_2404_02300_amd as sdt

    K, Wm = min(args.steps, 20), min(args.warmup, 3)
    t0 = time.time()
    indptr, indices = gen.make_graph(wl)
    Xh = gen.normal_features(wl.n_nodes, wl.feat, wl.seed)
    Wh, bh = gen.glorot_sage_weights(wl.dims, wl.seed)
    N, F, O, nnz = wl.n_nodes, wl.dims[0], wl.dims[1], int(indptr[-1])
    log(f"[bench] generated {wl.name}: N={N} nnz={nnz} in {time.time() - t0:.1f}s")
    g = sdt.Csr(torch.from_numpy(indptr).cuda(), torch.from_numpy(indices).cuda())
    X = torch.from_numpy(Xh).cuda()
    W, b = torch.from_numpy(Wh[0]).cuda(), torch.from_numpy(bh[0]).cuda()
    A = torch.empty(N, F, dtype=torch.float32, device="cuda")
    Y = torch.empty(N, O, dtype=torch.float32, device="cuda")
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(K)]
    for _ in range(Wm):
        sdt.sdt_sage_aggregate_csr_fwd(g, X, A)
        sdt.sdt_sage_linear_fwd(X, A, W, b, True, Y)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(K):          # events sit on torch's current stream, the one the kernels are launched on
        ev[i][0].record()
        sdt.sdt_sage_aggregate_csr_fwd(g, X, A)
        ev[i][1].record()
        sdt.sdt_sage_linear_fwd(X, A, W, b, True, Y)
        ev[i][2].record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    agg_s = float(np.mean([e[0].elapsed_time(e[1]) for e in ev])) * 1e-3
    gemm_s = float(np.mean([e[1].elapsed_time(e[2]) for e in ev])) * 1e-3
    # the same layer in one launch (aggregated rows stay in LDS)
    Yf = torch.empty(N, O, dtype=torch.float32, device="cuda")
    fev = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(K)]
    for _ in range(Wm):
        sdt.sdt_sage_layer_csr_fwd(g, X, W, b, True, Yf)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(K):
        fev[i][0].record()
        sdt.sdt_sage_layer_csr_fwd(g, X, W, b, True, Yf)
        fev[i][1].record()
    torch.cuda.synchronize()
    fused_elapsed = time.perf_counter() - t0
    fused_s = float(np.mean([e[0].elapsed_time(e[1]) for e in fev])) * 1e-3
    fused_equal = bool(torch.equal(Y, Yf))
    log(f"[bench] two launches {agg_s * 1e3:.2f} + {gemm_s * 1e3:.2f} ms; one launch {fused_s * 1e3:.2f} ms; "
        f"results bit-equal: {fused_equal}")
    agg_bytes = nnz * (F * 4 + 4) + N * (F * 4 + 8)          # every neighbour row read once per edge
    compulsory = 2 * N * F * 4 + nnz * 4 + N * 8            # each row read once, A written once
    flops = 2.0 * N * (2 * F) * O
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import sdt_oracle as orc
        rows = np.random.default_rng(wl.seed).choice(N, size=1 << 13, replace=False)
        deg = np.diff(indptr)
        sub_ip = np.zeros(len(rows) + 1, dtype=np.int64)
        sub_ip[1:] = np.cumsum(deg[rows])
        sub_cols = np.concatenate([indices[indptr[r]:indptr[r + 1]] for r in rows]).astype(np.int32)
        X64 = Xh.astype(np.float64)
        tc = time.perf_counter()
        refA = orc.aggregate_fwd(sub_ip, sub_cols, X64)
        orc.linear_fwd(X64[rows], refA, Wh[0], bh[0], relu=True)
        tc = time.perf_counter() - tc
        cpu = {"value": round(len(rows) / tc, 1), "unit": "nodes/s", "cores": 1, "kind": "oracle",
               "sample": f"{len(rows)} seeded random rows of the same layer (SpMM + projection), rows are independent",
               "host_cpus": os.cpu_count()}
    tr_agg = measured_traffic_sum(wl.name, "k_aggregate")
    tr_gemm = measured_traffic(wl.name, "k_linear_fwd")
    out = {
        "metric": "full-neighbour GraphSAGE-mean layer, nodes/s (SpMM over the whole CSR + projection)",
        "value": round(N * K / elapsed, 1), "unit": "nodes/s", "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": round(elapsed / K * 1e3, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{wl.name}: rmat 2^{wl.log2n} nodes, {nnz} CSR entries, F={F} -> {O}, one layer, "
                               f"no sampling", "seed": wl.seed},
        # the SpMM's fraction of the HBM roofline is taken from the counters (bytes that crossed the L2) when a counter
        # run of this build exists; the gather-side algorithmic figure (every neighbour row once per edge) is beside it
        "roofline": {"kernel": "k_aggregate_fwd<float,4,64,long> + k_aggregate_long (whole CSR, hub rows in the second launch)",
                     "bound": "hbm",
                     "achieved": round((tr_agg["bytes"] if tr_agg else agg_bytes) / agg_s / 1e9, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round((tr_agg["bytes"] if tr_agg else agg_bytes) / agg_s / 1e9 / HBM_PEAK_GBS, 4),
                     "basis": "rocprofv3 FETCH_SIZE + WRITE_SIZE bytes per launch" if tr_agg else "algorithmic (gather-side) bytes: no counter run of this build",
                     "traffic": tr_agg["bytes"] if tr_agg else None,
                     "traffic_from": f"{tr_agg['from']}: {tr_agg['kernel']}" if tr_agg else None,
                     "algorithmic_GBps": round(agg_bytes / agg_s / 1e9, 1), "algorithmic_frac": round(agg_bytes / agg_s / 1e9 / HBM_PEAK_GBS, 4),
                     "algorithmic_bytes_per_launch": int(agg_bytes), "compulsory_bytes_per_launch": int(compulsory),
                     "compulsory_GBps": round(compulsory / agg_s / 1e9, 1), "avg_launch_us": round(agg_s * 1e6, 1)},
        "gemm": {"kernel": "k_linear_fwd<float, float, Tile<128, 256, 16, 2, 4>, 4, 4, false>", "bound": "mfma",
                 "TFLOPs": round(flops / gemm_s / 1e12, 2), "traffic": tr_gemm["bytes"] if tr_gemm else None,
                 "peak": MFMA_FP32_PEAK_TFLOPS, "frac": round(flops / gemm_s / 1e12 / MFMA_FP32_PEAK_TFLOPS, 4),
                 "flops_per_launch": flops, "avg_launch_us": round(gemm_s * 1e6, 1)},
        # the same layer through sdt_sage_layer_csr_fwd (aggregated rows kept in LDS, no N x F buffer)
        "one_launch": {"kernel": "k_sage_layer_fused<256>", "nodes_per_s": round(N * K / fused_elapsed, 1),
                       "avg_launch_us": round(fused_s * 1e6, 1), "bit_equal_to_two_launches": fused_equal,
                       "hbm_buffer_saved_bytes": int(N * F * 4),
                       "algorithmic_GBps": round((agg_bytes + N * O * 4) / fused_s / 1e9, 1)},
        "cpu_baseline": cpu,
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
