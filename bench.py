#!/usr/bin/env python3
"""Benchmark of the degree-split SpMM hot path on one MI355X.

One "step" = one full aggregation Y = A_hat X (LD kernel + HD kernel + split-row
reduction) over the whole workload graph, inputs resident in HBM.  Prints ONE
JSON line: throughput in GFLOP/s (2*nnz*F per step), the effective HBM rate,
the roofline of the dominant (LD) kernel measured with HIP events, and the CPU
oracle timed on a bounded sample of the same workload.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0

# name -> (multiplier bits, batch copies, F, feature seed, degree threshold)
WORKLOADS = {
    "csa1024_b16_F64": (1024, 16, 64, 3, 32),    # the headline graph: 134,103,040 nodes
    "csa1024_b16_F32": (1024, 16, 32, 3, 32),    # embedding width of the paper's kernel evaluation
    "csa1024_b16_F128": (1024, 16, 128, 3, 32),
    "csa1024_b1_F64": (1024, 1, 64, 2, 32),
    "csa256_b1_F64": (256, 1, 64, 1, 32),
    "csa32_b1_F32": (32, 1, 32, 0, 32),
    # degree profile of the paper's Booth dataset at its kernel-evaluation sizes (64-512 bit, embedding 32):
    # radix-4 Booth multipliers, batched so that the graph is large enough to time
    "booth512_b16_F32": (512, 16, 32, 4, 32),
    "booth256_b16_F32": (256, 16, 32, 4, 32),
    "booth64_b16_F32": (64, 16, 32, 4, 32),
    "booth512_b16_F64": (512, 16, 64, 4, 32),
    # shape of the 4-LUT-mapped carry-save multiplier (rows of 7 entries; adjacency only, via groot_graph_from_csr)
    "lut4csa512_b16_F32": (512, 16, 32, 5, 32),
    "lut4csa256_b16_F32": (256, 16, 32, 5, 32),
    # shape of the standard-cell-mapped carry-save multiplier (AND2 rows of 4 entries, full-adder rows of 6)
    "cellcsa512_b16_F32": (512, 16, 32, 6, 32),
    "cellcsa1024_b16_F32": (1024, 16, 32, 6, 32),
    # polarized stress graph: 2^24 rows, 1 % heavy rows of 64..262,144 entries (Zipf 1.2), F = 128, thresholds swept
    # (first field: log2 of the row count; batch field unused)
    "stress16m_F128": (24, 1, 128, 4, 32),
    "stress1m_F128": (20, 1, 128, 4, 32),
}
STRESS_THRESHOLDS = (16, 32, 64, 128)


# HBM-side traffic of one launch of the LD kernel in bytes, from rocprofv3 FETCH_SIZE + WRITE_SIZE runs (the
# summaries under profiles/ give the commands and the scaling against a copy of known size).  Each entry is
# stamped with the hash of the kernel sources it was measured on (kernel_sources_sha16 below): when the
# sources have changed since, the figure no longer describes the kernel that is timed and the line reports
# traffic null instead.
TRAFFIC = {
    # FETCH_SIZE 26,515,835 KiB x 2.000 (scale of the 34.33 GB device copy in the same run), WRITE_SIZE 33,513,871 KiB x 1.000
    ("csa1024_b16_F64", "ld_pipe_kernel"): {"bytes": 88.62e9, "read": 54.30e9, "written": 34.32e9,
                                            "sources_sha16": "19684d826dc72e3c"},
}
KERNEL_SOURCES = ("groot_device.h", "groot_kernels.hip", "groot_ld_pipe.hip", "groot_compress.hip")


def kernel_sources_sha16():
    """Hash of the code of the aggregation kernels (the files a traffic measurement depends on), comments and
    white space left out: a reworded comment does not make a measurement stale, a changed statement does."""
    import hashlib
    import re

    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2511_18297_amd", "csrc", name), "r") as f:
            text = f.read()
        text = re.sub(r"/\*.*?\*/", " ", text, flags=re.S)         # none of these sources holds "//" or "/*" in a string
        text = re.sub(r"//[^\n]*", " ", text)
        h.update(" ".join(text.split()).encode())
    return h.hexdigest()[:16]


def measured_traffic(workload, kernel):
    """-> (bytes or None, note)"""
    entry = TRAFFIC.get((workload, kernel))
    if entry is None:
        return None, "no counter run recorded for this workload and kernel"
    now = kernel_sources_sha16()
    if entry["sources_sha16"] != now:
        return None, f"counter run was made on kernel sources {entry['sources_sha16']}, the timed ones are {now}"
    return entry["bytes"], f"FETCH_SIZE + WRITE_SIZE on kernel sources {now}"


def algorithmic_bytes(n, nnz, F):
    """The per-step byte count by definition: row pointers (int64) + column indices + weights + X read once +
    Y written once."""
    return 8 * (n + 1) + 4 * nnz + 4 * nnz + 4 * n * F + 4 * n * F


def bytes_needed(csr_bytes, n_in, n_out, F):
    """What a launch has to move at least, given the data structures the kernels really read: the device CSR as
    the library keeps it (groot_plan_query "csr_bytes": no weight array when the weights are row-uniform,
    compressed arrays where the library compresses) + the feature rows read once + the result rows written once."""
    return csr_bytes + 4 * n_in * F + 4 * n_out * F


def partitioned_bench(args, G, torch, np, g, view, X, Y, n, nnz, F, T, name, props):
    """Partitioned mode (Algorithm 1 of the paper): per part, gather the rows of S_p+ and aggregate on the
    sub-graph; the owned rows go straight to their global positions (groot_spmm_execute_rows), or, for
    comparison, all local rows are computed and the owned ones scattered back.  Reports the time of one
    pass over all parts with every sub-plan resident, and the device footprint one part needs when parts
    are processed one at a time."""
    P = args.partitioned
    t0 = time.time()
    parts = G.groot_partition_regrow(g, P)
    t_partition = time.time() - t0
    items, foot, cross = [], [], 0
    t0 = time.time()
    for p in range(P):
        pv = G.groot_parts_view(parts, p)
        sub = G.groot_graph_view(pv["sub"])
        ids = torch.from_numpy(pv["global_id"].copy()).cuda()
        plan = G.groot_spmm_plan(pv["sub"], T)
        G.groot_plan_upload(plan, F)
        n_loc = ids.shape[0]
        items.append((plan, ids, pv["n_owned"], n_loc))
        cross += pv["n_crossing"]
        # rowptr + col (mean weights are not stored on the device) + ids + X_p + the owned rows of Y
        # (boundary rows are not computed: groot_spmm_execute_rows)
        foot.append(8 * (n_loc + 1) + 4 * sub["nnz"] + 8 * n_loc + 4 * n_loc * F + 4 * pv["n_owned"] * F)
    torch.cuda.synchronize()
    t_plans = time.time() - t0
    max_loc = max(it[3] for it in items)
    Xp = torch.empty((max_loc, F), dtype=torch.float32, device="cuda")
    Yp = torch.empty_like(Xp)
    Yout = torch.full_like(Y, float("nan"))

    def one_pass_copies():
        """gather, SpMM on all local rows, scatter of the owned rows"""
        for plan, ids, n_owned, n_loc in items:
            G.groot_rows_gather(ids, X, Xp[:n_loc], F)
            G.groot_spmm_execute(plan, Xp[:n_loc], Yp[:n_loc], F)
            G.groot_rows_scatter(ids[:n_owned], Yp[:n_loc], Yout, F)

    def one_pass():
        """gather, then only the owned rows, written straight to their global positions"""
        for plan, ids, n_owned, n_loc in items:
            G.groot_rows_gather(ids, X, Xp[:n_loc], F)
            G.groot_spmm_execute_rows(plan, Xp[:n_loc], Yout, F, n_owned, ids)

    def timed(fn):
        for _ in range(max(1, args.warmup)):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / args.steps

    ms_copies = timed(one_pass_copies)
    Yout.fill_(float("nan"))
    ms = timed(one_pass)
    full_plan = G.groot_spmm_plan(g, T)
    G.groot_plan_upload(full_plan, F)
    G.groot_spmm_execute(full_plan, X, Y, F)
    torch.cuda.synchronize()
    worst = 0.0
    for lo in range(0, n, 1 << 24):
        worst = max(worst, float((Yout[lo:lo + (1 << 24)] - Y[lo:lo + (1 << 24)]).abs().max()))
    # the same partition built on the device: re-growth of every part from the full graph's resident CSR, and a
    # plan from the part's device arrays; one pass with those plans must give the same result
    items.clear()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    dev_items = []
    for p in range(P):
        part = G.groot_partition_regrow_device(full_plan, P, p)
        pv = G.groot_dev_part_view(part)
        plan = G.groot_dev_part_plan(part, T, F)
        dev_items.append((plan, pv["global_id"], pv["n_owned"], pv["n_owned"] + pv["n_halo"], part))
    torch.cuda.synchronize()
    t_partition_dev = time.perf_counter() - t0
    assert max(it[3] for it in dev_items) == max_loc
    items.extend(it[:4] for it in dev_items)
    Yout.fill_(float("nan"))
    ms_dev = timed(one_pass)
    worst_dev = 0.0
    for lo in range(0, n, 1 << 24):
        worst_dev = max(worst_dev, float((Yout[lo:lo + (1 << 24)] - Y[lo:lo + (1 << 24)]).abs().max()))
    # the same device-built plans with their columns renamed to global rows: no gather, X read in place
    for plan, ids, n_owned, n_loc in items:
        G.groot_plan_use_global_columns(plan, ids, n)
    torch.cuda.synchronize()

    def one_pass_in_place():
        for plan, ids, n_owned, n_loc in items:
            G.groot_spmm_execute_rows(plan, X, Yout, F, n_owned, ids)

    Yout.fill_(float("nan"))
    ms_in_place = timed(one_pass_in_place)
    worst_in_place = 0.0
    for lo in range(0, n, 1 << 24):
        worst_in_place = max(worst_in_place, float((Yout[lo:lo + (1 << 24)] - Y[lo:lo + (1 << 24)]).abs().max()))
    full_foot = 8 * (n + 1) + 4 * nnz + 2 * 4 * n * F
    undirected = (nnz - n) // 2
    print(json.dumps({
        "metric": "partitioned-mode SpMM (per part: the owned rows computed into place from the resident feature "
                  "matrix), 1024-bit CSA AIG, F=64",
        "value": round(2.0 * nnz * F / (ms_in_place * 1e-3) / 1e9, 1), "unit": "GFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_in_place, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": name + f"_partitioned{P}", "N": n, "nnz": nnz, "F": F, "parts": P},
        "max_abs_diff_vs_full_graph_in_place": worst_in_place,
        "ms_per_step_with_gather_pass": round(ms, 4),
        "ms_per_step_with_gather_and_scatter_pass": round(ms_copies, 4),
        "boundary_edge_fraction": round(cross / 2 / undirected, 4),
        "rows_with_boundary": sum(it[3] for it in items), "largest_part_rows": max_loc,
        "device_bytes_full_graph": full_foot, "device_bytes_largest_part": max(foot),
        "memory_reduction_pct": round(100.0 * (1.0 - max(foot) / full_foot), 2),
        "max_abs_diff_vs_full_graph": worst, "partition_seconds": round(t_partition, 2),
        "host_plans_and_upload_seconds": round(t_plans, 2),
        "device_built": {"partition_and_plans_seconds": round(t_partition_dev, 3), "ms_per_step": round(ms_dev, 4),
                         "max_abs_diff_vs_full_graph": worst_dev},
        "device": props.name}))


def sage_layer_bench(args, G, torch, np, aig, g, T, plan, X, H, n, nnz, F, batch, name, props, placement):
    """Fused layer (X -> H, the pair of buffers the placement search kept) against the unfused form (library SpMM
    into a buffer of its own, then torch for the dense part)."""
    assert F in (32, 64), "the fused layer is built for F = 64 and F = 32"
    gen = torch.Generator(device="cuda").manual_seed(2)
    Wn, Ws = ((torch.rand((F, F), generator=gen, device="cuda") - 0.5) * 0.25 for _ in range(2))
    b = (torch.rand(F, generator=gen, device="cuda") - 0.5) * 0.25
    Y = torch.empty_like(X)

    def fused():
        G.groot_sage_layer_forward(plan, X, Wn, Ws, b, True, H, F)

    def unfused():
        G.groot_spmm_execute(plan, X, Y, F)
        out = torch.addmm(b, Y, Wn)
        out.addmm_(X, Ws)
        return torch.relu_(out)

    def timed(fn, steps, warmup):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps

    ms_fused = timed(fused, args.steps, args.warmup)
    ms_unfused = timed(unfused, max(3, args.steps // 4), 1)
    ref = unfused()
    fused()
    torch.cuda.synchronize()
    worst = 0.0
    for lo in range(0, n, 1 << 24):
        worst = max(worst, float((H[lo:lo + (1 << 24)] - ref[lo:lo + (1 << 24)]).abs().max()))
    del ref

    # The layer's input gradient, dX = A_hat^T (dZ Wn^T) + dZ Ws^T, through the same kernel (X plays dZ, H takes
    # dX), against the unfused form: one dense product, the library's SpMM on the transposed graph, a second dense
    # product added to it.
    WnT, WsT = Wn.t().contiguous(), Ws.t().contiguous()
    Xs = Y                                                   # dZ / deg; the unfused forward's buffer is free again
    G.groot_rows_over_degree(plan, X, Xs, F)

    def fused_backward():
        G.groot_sage_layer_backward_data(plan, Xs, WnT, WsT, H, F, F)

    ms_backward = timed(fused_backward, args.steps, args.warmup)
    backward = {"ms_per_step": round(ms_backward, 4), "unfused_ms_per_step": None, "speedup_vs_unfused": None,
                "max_abs_diff_vs_unfused": None}
    torch.cuda.empty_cache()                                 # the unfused forward's result is still cached
    if torch.cuda.mem_get_info()[0] > 2.6 * X.numel() * 4:   # two more matrices and the transposed graph's plan
        plan_t = G.groot_spmm_plan(G.groot_graph_transpose(g), T)
        G.groot_plan_upload(plan_t, F)
        G1, out = torch.empty_like(X), torch.empty_like(X)

        def unfused_backward():
            torch.mm(X, WnT, out=G1)
            G.groot_spmm_execute(plan_t, G1, out, F)
            return out.addmm_(X, WsT)

        ms_unfused_backward = timed(unfused_backward, max(3, args.steps // 4), 1)
        unfused_backward()
        fused_backward()
        torch.cuda.synchronize()
        worst_b = 0.0
        for lo in range(0, n, 1 << 24):
            worst_b = max(worst_b, float((H[lo:lo + (1 << 24)] - out[lo:lo + (1 << 24)]).abs().max()))
        backward.update(unfused_ms_per_step=round(ms_unfused_backward, 4),
                        speedup_vs_unfused=round(ms_unfused_backward / ms_backward, 3), max_abs_diff_vs_unfused=worst_b)
        del G1, out, plan_t
    # The gradients of the two weight matrices, dWn = (A_hat X)^T dZ and dWs = X^T dZ (H plays dZ), in one pass
    # against the unfused form: the library's SpMM, then two products with N as the contraction length.
    torch.cuda.empty_cache()
    ws = torch.empty((G.groot_sage_layer_backward_weights_workspace(plan, F) // 4,), dtype=torch.float32, device="cuda")
    dW = torch.empty((2, F, F), dtype=torch.float32, device="cuda")

    def fused_wgrad():
        G.groot_sage_layer_backward_weights(plan, X, H, dW[0], dW[1], ws, F)

    def unfused_wgrad():
        G.groot_spmm_execute(plan, X, Y, F)
        return torch.mm(Y.t(), H), torch.mm(X.t(), H)

    ms_wgrad = timed(fused_wgrad, args.steps, args.warmup)
    ms_unfused_wgrad = timed(unfused_wgrad, 2, 1)
    ref_n, ref_s = unfused_wgrad()
    fused_wgrad()
    torch.cuda.synchronize()
    weights = {"ms_per_step": round(ms_wgrad, 4), "unfused_ms_per_step": round(ms_unfused_wgrad, 4),
               "speedup_vs_unfused": round(ms_unfused_wgrad / ms_wgrad, 3),
               "max_rel_diff_vs_unfused": float(max((dW[0] - ref_n).abs().max() / ref_n.abs().max(),
                                                    (dW[1] - ref_s).abs().max() / ref_s.abs().max()))}

    flops = 2.0 * nnz * F + 2.0 * n * (2 * F) * F
    tflops = flops / (ms_fused * 1e-3) / 1e12
    # The dense products run as bf16 piece products (a sixteenth of the fp32 matrix instruction's time per
    # multiply-add, six per fp32 product), so the layer is bound like the aggregation alone: by the bytes of X,
    # of the CSR and of H.
    # the layer kernel reads the plain CSR (8-byte row pointers, 4-byte column indices; no weight array for the
    # row-uniform weights of these graphs), X once, and writes H once
    bytes_layer = bytes_needed(8 * (n + 1) + 4 * nnz, n, n, F)
    gbps = bytes_layer / (ms_fused * 1e-3) / 1e9
    print(json.dumps({
        "metric": f"GraphSAGE-mean layer forward H = relu((A_hat X) Wn + X Ws + b), fused, 1024-bit CSA AIG, F={F}",
        "value": round(tflops * 1e3, 1), "unit": "GFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_fused, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": name + "_sage_layer", "batch": batch, "N": n, "nnz": nnz, "F": F},
        "roofline": {"bound": "hbm", "kernel": "sage_pipe_kernel (+ hd_kernel)", "achieved": round(gbps, 1),
                     "peak": 8000.0, "unit": "GB/s", "frac": round(gbps / 8000.0, 4), "traffic": None,
                     "algorithmic_bytes": bytes_layer},
        "bf16_pieces_per_operand": next((int(t.partition("=")[2]) for t in args.tune if t.startswith("sage_pieces=")), 3),
        "fp32_equivalent_tflops": round(tflops, 2), "fp32_mfma_peak_tflops": 157.3,
        "unfused_ms_per_step": round(ms_unfused, 4), "speedup_vs_unfused": round(ms_unfused / ms_fused, 3),
        "max_abs_diff_vs_unfused": worst, "backward_data": backward, "backward_weights": weights, "placement": placement, "device": props.name}))


def place_features(G, torch, wl, plan, seed, n, F, tries, fixed=None):
    """Where the feature matrices lie in device memory changes the step time by up to 10 % on this machine, the same
    kernels on the same data: slowest when X and Y lie in address ranges of the same one of two classes that
    alternate every 64 GiB or so (the first two allocations of a process), fastest when each of them straddles a
    boundary between the classes.  The library has a call that finds a good place
    by measuring, `groot_feature_placement`; a caller that reuses its feature buffers over many layers and epochs
    makes it once.  Here, before any feature matrix exists: one arena of `tries` + 3 matrix sizes is allocated, the
    call picks the offsets of X and Y in it, and the features are generated into the X it picked.  With `tries` = 0
    X and Y are plain allocations, one after the other.  -> X, Y, log"""
    numel = n * F
    slots, arena = 0, None
    if tries > 0:
        free, _ = torch.cuda.mem_get_info()
        slots = min(tries + 3, int(0.75 * free // (numel * 4)))      # a quarter of the memory stays free for the rest
    while slots >= 3 and arena is None:
        try:
            arena = torch.empty((slots * numel,), dtype=torch.float32, device="cuda")
            arena.uniform_(-1.0, 1.0)                    # values like the features': the times depend a little on the data
        except RuntimeError:                             # out of memory after all: a smaller arena
            torch.cuda.empty_cache()
            slots -= 1
    if arena is None:
        X = wl.uniform_features(seed, 0, n, F, device="cuda")
        return X, torch.empty_like(X), (None if tries <= 0 else {"arena_matrices": 0, "note": "no room for an arena"})
    t0 = time.perf_counter()
    if fixed:                                            # offsets of an earlier search (they repeat from box to box)
        assert max(fixed) + numel * 4 <= arena.numel() * 4 and abs(fixed[0] - fixed[1]) >= numel * 4 \
            and fixed[0] % 16 == 0 and fixed[1] % 16 == 0, "offsets outside the arena, overlapping or unaligned"
        place = {"x_offset": fixed[0], "y_offset": fixed[1], "best_ms": float("nan"), "first_ms": float("nan")}
    else:
        place = G.groot_feature_placement(plan, arena, F)
    seconds = time.perf_counter() - t0
    ox, oy = place["x_offset"] // 4, place["y_offset"] // 4
    X, Y = arena[ox:ox + numel].view(n, F), arena[oy:oy + numel].view(n, F)
    wl.uniform_features(seed, 0, n, F, out=X)
    return X, Y, {"arena_matrices": slots, "x_offset_bytes": place["x_offset"], "y_offset_bytes": place["y_offset"],
                  "back_to_back_ms": None if fixed else round(place["first_ms"], 3),
                  "kept_ms": None if fixed else round(place["best_ms"], 3),
                  "search_seconds": None if fixed else round(seconds, 2)}


def stress_bench(args, G, torch, np, wl, name, props):
    """The polarized stress workload: N = 2^24 rows, 99 % light rows (3-5 entries within +-4096), 1 % heavy rows
    of 64 .. 262,144 entries with uniformly random columns, F = 128; one SpMM per degree threshold of the sweep.
    The gathers of the heavy rows (4 F bytes per stored entry, spread uniformly over the whole feature matrix,
    34 times the size of the last-level cache) cannot be served from any cache, so the bound of this workload is
    the gather demand 4 F nnz against the HBM peak, not the read-once byte count."""
    log2n, _, F, seed, T_default = WORKLOADS[name]
    n = 1 << log2n
    thresholds = tuple(args.thresholds) if args.thresholds else STRESS_THRESHOLDS
    t0 = time.time()
    s = wl.stress_graph(seed, n, window=4096, dmin=64, dmax=262144, verbose=True)
    nnz = int(s.rowptr[-1])
    deg = np.diff(s.rowptr)
    t_gen = time.time() - t0
    t0 = time.time()
    g = G.groot_graph_from_csr(s.rowptr, s.col, s.val)
    X = wl.uniform_features(seed, 0, n, F, device="cuda")
    Y = torch.empty_like(X)
    torch.cuda.synchronize()
    t_setup = time.time() - t0
    flops = 2.0 * nnz * F
    gather_bytes = 4.0 * F * nnz

    sweep, headline, cpu, parity = [], None, None, None
    T_head = T_default if T_default in thresholds else thresholds[0]
    for T in thresholds:
        plan = G.groot_spmm_plan(g, T)
        pv = G.groot_plan_view(plan)
        G.groot_plan_upload(plan, F)
        for _ in range(max(1, args.warmup)):
            G.groot_spmm_execute(plan, X, Y, F)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            G.groot_spmm_execute(plan, X, Y, F)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / args.steps

        def timed_phase(phases):
            G.groot_spmm_execute_phases(plan, X, Y, F, phases)
            start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            start.record()
            for _ in range(args.steps):
                G.groot_spmm_execute_phases(plan, X, Y, F, phases)
            stop.record()
            stop.synchronize()
            return start.elapsed_time(stop) / args.steps

        ms_ld = timed_phase(G.GROOT_PHASE_LD)
        ms_hd = timed_phase(G.GROOT_PHASE_HD) if pv["n_hd"] else 0.0
        ms_fin = timed_phase(G.GROOT_PHASE_FINISH) if pv["n_hd"] else 0.0
        nnz_hd = G.groot_plan_query(plan, "nnz_hd")
        csr_bytes = G.groot_plan_query(plan, "csr_bytes")
        item = {"degree_threshold": T, "n_hd_rows": pv["n_hd"], "nnz_hd": nnz_hd, "ms_per_step": round(ms, 3),
                "gflops": round(flops / (ms * 1e-3) / 1e9, 1),
                "gather_demand_gbps": round(gather_bytes / (ms * 1e-3) / 1e9, 1),
                "ld_ms": round(ms_ld, 3), "hd_ms": round(ms_hd, 3), "finish_ms": round(ms_fin, 3),
                "hd_gather_gbps": round(4.0 * F * nnz_hd / (ms_hd * 1e-3) / 1e9, 1) if ms_hd else None,
                "hd_pieces": G.groot_plan_query(plan, "hd_pieces"), "csr_bytes": csr_bytes,
                "weight_mode": G.groot_plan_query(plan, "weight_mode")}
        sweep.append(item)
        print(f"stress T={T}: {item}", file=sys.stderr, flush=True)
        if T == T_head:
            headline = item
            G.groot_spmm_execute(plan, X, Y, F)
            torch.cuda.synchronize()
            # ---- CPU oracle on sampled rows (light rows at random, heavy rows at random, the eight longest)
            if not args.no_cpu_baseline:
                import oracle

                rng = np.random.default_rng(5)
                heavy = np.nonzero(deg >= 16)[0]
                rows = np.unique(np.concatenate([rng.integers(0, n, 20000), rng.choice(heavy, min(600, heavy.shape[0]), replace=False),
                                                 heavy[np.argsort(deg[heavy])[-8:]], [0, n - 1]]))
                sub_rowptr = np.concatenate([[0], np.cumsum(deg[rows])])
                idx = np.concatenate([np.arange(s.rowptr[v], s.rowptr[v + 1]) for v in rows])
                uniq, inv = np.unique(s.col[idx], return_inverse=True)
                Xs = X[torch.from_numpy(uniq.astype(np.int64)).cuda()].cpu().numpy()
                sub_col, sub_val = inv.astype(np.int32), s.val[idx]
                threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
                t0 = time.perf_counter()
                Y64, _ = oracle.spmm_f64(sub_rowptr, sub_col, sub_val, Xs, want_abs=False)
                t_cpu = time.perf_counter() - t0
                _, S = oracle.spmm_f64(sub_rowptr, sub_col, sub_val, Xs, want_abs=True)
                got = Y[torch.from_numpy(rows).cuda()].cpu().numpy().astype(np.float64)
                parity = float(np.max(np.abs(got - Y64) / (1e-5 * S + 1e-6)))
                cpu = {"value": round(2.0 * idx.shape[0] * F / t_cpu / 1e9, 3), "unit": "GFLOP/s", "cores": threads,
                       "kind": "oracle", "seconds": round(t_cpu, 3),
                       "sample": f"{rows.shape[0]} sampled rows (20,000 random, 600 heavy, the 8 longest) with "
                                 f"{idx.shape[0]} stored entries of the {n}-row graph, their {uniq.shape[0]} feature "
                                 f"rows gathered into a compact matrix first, F={F} (fp64, row-parallel OpenMP)"}
        del plan
    out = {
        "metric": "SpMM GFLOP/s and achieved HBM GB/s (% of peak), polarized stress graph, F=128",
        "value": headline["gflops"], "unit": "GFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": headline["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": name, "N": n, "nnz": nnz, "F": F, "degree_threshold": headline["degree_threshold"],
                   "heavy_rows": int((deg >= 64).sum()), "longest_row": int(deg.max())},
        "hbm_gbps": round(algorithmic_bytes(n, nnz, F) / (headline["ms_per_step"] * 1e-3) / 1e9, 1),
        "algorithmic_bytes_per_step": algorithmic_bytes(n, nnz, F),
        "bytes_needed_per_step": bytes_needed(headline["csr_bytes"], n, n, F),
        "roofline": {"bound": "hbm", "kernel": "hd_kernel", "achieved": headline["hd_gather_gbps"], "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": round(headline["hd_gather_gbps"] / HBM_PEAK_GBPS, 4) if headline["hd_gather_gbps"] else None,
                     "traffic": None, "ms": headline["hd_ms"],
                     "algorithmic_bytes": 4.0 * F * headline["nnz_hd"],
                     "note": "gather demand of the high-degree rows (4 F bytes per stored entry; uniformly random "
                             "columns over a feature matrix 34 times the last-level cache) over the HD kernel's time"},
        "threshold_sweep": sweep,
        "cpu_baseline": cpu, "parity_max_err_over_tol": parity,
        "generation_seconds": round(t_gen, 1), "setup_seconds": round(t_setup, 1), "device": props.name}
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default=None, choices=sorted(WORKLOADS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-copies", type=int, default=16, help="copies of the batch the CPU oracle runs (and checks)")
    ap.add_argument("--placement-tries", type=int, default=3,
                    help="groot_feature_placement looks for a good place for X and Y in an arena of this many matrix sizes + 3; "
                         "0: take the first allocations as they come")
    ap.add_argument("--placement-offsets", type=int, nargs=2, default=None, metavar=("X", "Y"),
                    help="byte offsets of X and Y in the arena, as an earlier run reported them: no search (for profiles)")
    ap.add_argument("--thresholds", type=int, nargs="*", default=None, help="stress workload: degree thresholds to sweep")
    ap.add_argument("--transposed", action="store_true", help="time dX = A_hat^T dY (backward pass) instead")
    ap.add_argument("--partitioned", type=int, default=0, metavar="P",
                    help="time the partitioned mode instead: P parts with re-grown boundary, gather -> SpMM -> scatter")
    ap.add_argument("--sage-layer", action="store_true",
                    help="time the fused GraphSAGE-mean layer H = relu((A_hat X) Wn + X Ws + b) instead (F = 64)")
    ap.add_argument("--xcd-remap", type=int, default=None)
    ap.add_argument("--hd-chunk", type=int, default=None)
    ap.add_argument("--ld-pipeline", type=int, default=None, help="LD kernel choice: 1 pipelined, 0 plain, -1 auto")
    ap.add_argument("--sage-gap", type=int, default=None, help="pacing of the fused layer's matrix wavefronts (0..4)")
    ap.add_argument("--tune", action="append", default=[], metavar="NAME=VALUE",
                    help="any other groot_set_tuning knob (repeatable), e.g. uniform_detect=0")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (the path is single-GPU by design); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2511_18297_amd import build as groot_build

    if not os.path.exists(groot_build.LIB_PATH):
        groot_build.build()
    import paper_2511_18297_amd as G
    import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    props = torch.cuda.get_device_properties(0)
    if args.xcd_remap is not None:
        G.groot_set_tuning("xcd_remap", args.xcd_remap)
    if args.hd_chunk is not None:
        G.groot_set_tuning("hd_chunk", args.hd_chunk)
    if args.ld_pipeline is not None:
        G.groot_set_tuning("ld_pipeline", args.ld_pipeline)
    if args.sage_gap is not None:
        G.groot_set_tuning("sage_gap", args.sage_gap)
    for item in args.tune:
        name, _, value = item.partition("=")
        G.groot_set_tuning(name, int(value))

    name = args.workload
    if name is None:
        # the headline graph needs ~76 GB of HBM; fall back to one copy on smaller parts
        name = "csa1024_b16_F64" if props.total_memory > 100e9 else "csa1024_b1_F64"
    bits, batch, F, seed, T = WORKLOADS[name]
    if name.startswith("stress"):
        stress_bench(args, G, torch, np, wl, name, props)
        return

    t0 = time.time()
    shape_only = wl.lut4_csa_graph if name.startswith("lut4") else wl.cellmap_csa_graph if name.startswith("cell") else None
    if shape_only is not None:
        if args.transposed or args.partitioned or args.sage_layer:
            sys.exit("the mapped-netlist shape workloads run the plain SpMM only")
        aig = None
        g = G.groot_graph_from_csr(*(lambda b: (b.rowptr, b.col, b.val))(shape_only(bits, batch)))
    else:
        aig = wl.booth_multiplier_aig(bits) if name.startswith("booth") else wl.csa_multiplier_aig(bits)
        g = G.groot_graph_build(aig.type, aig.fanin0, aig.fanin1, batch)
    if args.transposed:
        g = G.groot_graph_transpose(g)
    view = G.groot_graph_view(g)
    n, nnz = view["n"], view["nnz"]
    plan = G.groot_spmm_plan(g, T)
    pv = G.groot_plan_view(plan)
    n_hd, n_ld = pv["n_hd"], pv["n_ld"]
    nnz_hd = int(np.diff(view["rowptr"])[pv["hd_rows"]].sum()) if n_hd else 0
    G.groot_plan_upload(plan, F)
    t_setup = time.time() - t0
    tries = 0 if args.partitioned else min(args.placement_tries, 1) if args.sage_layer else args.placement_tries
    X, Y, placement = place_features(G, torch, wl, plan, seed, n, F, tries, args.placement_offsets)
    torch.cuda.synchronize()

    def run(phases, count):
        for _ in range(count):
            G.groot_spmm_execute_phases(plan, X, Y, F, phases)

    if args.partitioned:
        partitioned_bench(args, G, torch, np, g, view, X, Y, n, nnz, F, T, name, props)
        return
    if args.sage_layer:                                  # X and the layer's output where the aggregation runs fastest
        sage_layer_bench(args, G, torch, np, aig, g, T, plan, X, Y, n, nnz, F, batch, name, props, placement)
        return

    # ---- whole path: W warm-up steps, then exactly K timed steps
    run(G.GROOT_PHASE_ALL, args.warmup)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(G.GROOT_PHASE_ALL, args.steps)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps

    flops = 2.0 * nnz * F
    bytes_all = algorithmic_bytes(n, nnz, F)                 # by the definition (int64 row pointers, weights counted)
    bytes_min = bytes_needed(G.groot_plan_query(plan, "csr_bytes"), n, n, F)   # what the kernels have to move
    gflops = flops / (ms_per_step * 1e-3) / 1e9
    gbps = bytes_min / (ms_per_step * 1e-3) / 1e9
    gbps_formula = bytes_all / (ms_per_step * 1e-3) / 1e9

    # ---- dominant kernel (LD) alone, HIP events on the launch stream
    def timed_phase(phases):
        run(phases, 2)
        start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        start.record()
        run(phases, args.steps)
        stop.record()
        stop.synchronize()
        return start.elapsed_time(stop) / args.steps

    ms_ld = timed_phase(G.GROOT_PHASE_LD)
    ms_hd = timed_phase(G.GROOT_PHASE_HD) if n_hd else 0.0
    ms_fin = timed_phase(G.GROOT_PHASE_FINISH) if n_hd else 0.0
    # LD launch: the bytes it has to move (the LD part of the device CSR as the kernels read it, X once, the LD
    # rows of Y), and the same by the definition's formula (all row pointers as int64, index and weight of every
    # LD entry) for comparison
    bytes_ld = bytes_needed(G.groot_plan_query(plan, "csr_bytes_ld"), n, n_ld, F)
    bytes_ld_formula = 8 * (n + 1) + 8 * (nnz - nnz_hd) + 4 * n * F + 4 * n_ld * F
    ld_gbps = bytes_ld / (ms_ld * 1e-3) / 1e9

    # ---- device copy of the same N x F matrix: the practical streaming ceiling of this machine
    Z = torch.empty_like(X)
    for _ in range(2):
        Z.copy_(X)
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    start.record()
    for _ in range(5):
        Z.copy_(X)
    stop.record()
    stop.synchronize()
    copy_gbps = 2 * 4 * n * F / (start.elapsed_time(stop) / 5 * 1e-3) / 1e9
    del Z

    # ---- CPU oracle (fp64, row-parallel) on the same workload, copy by copy; its output doubles as an
    # element-wise parity check of the timed configuration.  --cpu-copies bounds the sample.
    cpu = None
    parity = None
    if not args.no_cpu_baseline:
        import oracle

        lut = shape_only(bits, 1) if shape_only is not None else None
        n1 = lut.n if lut is not None else aig.num_nodes
        if lut is not None:
            rp, col, val = lut.rowptr, lut.col, lut.val
        else:
            rp, col, val, _ = oracle.csr_build(aig.type, aig.fanin0, aig.fanin1, 1)
        if args.transposed:
            rp, col, val = oracle.csr_transpose(rp, col, val)
        threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
        copies = min(batch, args.cpu_copies)
        run(G.GROOT_PHASE_ALL, 1)
        torch.cuda.synchronize()
        t_cpu, parity = 0.0, 0.0
        for c in range(copies):
            Xc = X[c * n1:(c + 1) * n1].cpu().numpy()
            t0 = time.perf_counter()
            Y64, _ = oracle.spmm_f64(rp, col, val, Xc, want_abs=False)
            t_cpu += time.perf_counter() - t0
            _, S = oracle.spmm_f64(rp, col, val, Xc, want_abs=True)          # untimed: error scale
            err = np.abs(Y[c * n1:(c + 1) * n1].cpu().numpy().astype(np.float64) - Y64)
            parity = max(parity, float(np.max(err / (1e-5 * S + 1e-6))))
            del Y64, S, err, Xc
        cpu = {"value": round(2.0 * rp[-1] * copies * F / t_cpu / 1e9, 3), "unit": "GFLOP/s", "cores": threads,
               "kind": "oracle", "seconds": round(t_cpu, 3),
               "sample": f"copies 0..{copies - 1} of {batch}: {n1 * copies} rows, {int(rp[-1]) * copies} nnz, F={F} "
                         f"(fp64, row-parallel OpenMP, one copy at a time)"}

    # which LD kernel the library picked for this plan and F
    mode = G.groot_plan_query(plan, "ld_pipelined")
    ld_name = "ld_pipe_kernel" if (mode == 2 and F in (32, 64, 128)) or (mode == 1 and F in (64, 128)) else "ld_kernel"
    traffic, traffic_note = (None, "not measured for the transposed graph") if args.transposed else \
        measured_traffic(name, ld_name)
    out = {
        "metric": "SpMM GFLOP/s and achieved HBM GB/s (% of peak), 1024-bit CSA AIG, F=64",
        "value": round(gflops, 2),
        "unit": "GFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": name + ("_transposed" if args.transposed else ""), "multiplier_bits": bits, "batch": batch, "N": n, "nnz": nnz, "F": F,
                   "degree_threshold": T, "n_hd_rows": n_hd, "nnz_hd": nnz_hd,
                   "xcd_remap": args.xcd_remap if args.xcd_remap is not None else 1},
        "hbm_gbps": round(gbps, 1),
        "hbm_pct_of_peak": round(100.0 * gbps / HBM_PEAK_GBPS, 2),
        "bytes_needed_per_step": bytes_min,
        "formula": {"algorithmic_bytes_per_step": bytes_all, "hbm_gbps": round(gbps_formula, 1),
                    "hbm_pct_of_peak": round(100.0 * gbps_formula / HBM_PEAK_GBPS, 2),
                    "note": "8(N+1) + 4 nnz + 4 nnz + 4NF + 4NF: counts a weight array and 8-byte row pointers "
                            "whether or not the kernels read them; hbm_gbps / hbm_pct_of_peak above use "
                            "bytes_needed_per_step"},
        "roofline": {"bound": "hbm", "kernel": ld_name, "achieved": round(ld_gbps, 1), "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": round(ld_gbps / HBM_PEAK_GBPS, 4),
                     "traffic": traffic, "traffic_note": traffic_note,
                     "ms": round(ms_ld, 4), "algorithmic_bytes": bytes_ld, "formula_bytes": bytes_ld_formula},
        "weight_mode": G.groot_plan_query(plan, "weight_mode"),
        "kernel_sources_sha16": kernel_sources_sha16(),
        "hd_ms": round(ms_hd, 4),
        "finish_ms": round(ms_fin, 4),
        "copy_kernel_gbps": round(copy_gbps, 1),
        "placement": placement,
        "cpu_baseline": cpu,
        "parity_max_err_over_tol": parity,
        "setup_seconds": round(t_setup, 2),
        "device": props.name,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
