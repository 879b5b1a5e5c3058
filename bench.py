#!/usr/bin/env python3
"""Benchmark: full-batch GCN training epochs per second on one partition, one MI355X.

One step = one epoch = gcn_forward + gcn_loss_acc + gcn_backward + gcn_sgd_step over the whole
partition (graph creation is outside the timed region; all inputs are resident in HBM).
Prints ONE JSON line with
  * the epoch rate, timed with no event between launches;
  * a second timed region of the same epochs in which the library brackets every launch with HIP events on the
    stream it is launched on: per-kernel times, the dominant kernel and its roofline position;
  * the ceilings that position is measured against, taken in this process on this chip: the gather ceiling
    (every gather an L2 hit, on a table of the aggregated matrix's size), the same gather without locality, the
    streaming-copy rate and the rate of the tile product's matrix instruction;
  * the CPU oracle timed on this machine's host cores (all of them, and one) as a baseline.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0       # MI355X HBM3E peak
FP32_PEAK_TFLOPS = 157.3


def gather_bytes(E: int, n: int, w: int, s: int = 4) -> int:
    """Algorithmic traffic of one aggregation of width w: every nonzero pulls a 4-byte column index
    and one feature row, every output row is written once, plus the row pointers and d^-1/2."""
    return E * (4 + w * s) + n * w * s + 8 * (n + 1) + 4 * n


BF16_MFMA_PEAK_TFLOPS = 2500.0


def compulsory_bytes(E: int, n: int, w: int, s: int = 4) -> int:
    """Every array of one aggregation touched once: the floor for traffic past the caches."""
    return 4 * E + 2 * n * w * s + 8 * (n + 1) + 4 * n


def read_traffic(workload: str, kernel: str, width: int):
    """Bytes leaving L2 per launch of `kernel` at this width, and its L2 hit rate, from the rocprofv3 counter summary
    committed under profiles/ (lines: workload kernel w<width> fetch_bytes write_bytes l2_hit_rate commit), else None."""
    path = os.path.join(ROOT, "profiles", "spmm_traffic.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        parts = line.split()
        if len(parts) >= 6 and parts[0] == workload and parts[1] == kernel and parts[2] == "w%d" % width:
            try:
                return {"fetch_bytes": float(parts[3]), "write_bytes": float(parts[4]), "l2_hit_rate": float(parts[5]),
                        "source": "profiles/spmm_traffic.txt" + (" @ " + parts[6] if len(parts) > 6 else "")}
            except ValueError:
                return None
    return None


def gpu_graph(B, torch, np, wl, dtype):
    """The workload's arrays as device tensors in the types the C ABI takes, and the graph made from them."""
    dev = lambda a, t: torch.from_numpy(np.ascontiguousarray(a, dtype=t)).cuda()
    return B.gcn_graph_create(dev(wl.rowptr, np.int64), dev(wl.col, np.int32), dev(wl.x, np.float32),
                              dev(wl.labels, np.int32), dev(wl.mask, np.uint8), wl.dims[-1], store_dtype=dtype)


def event_time(torch, fn, reps):
    """Average milliseconds of fn() over reps launches on the current stream (after one warm-up)."""
    fn()
    torch.cuda.synchronize()
    s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    s.record()
    for _ in range(reps):
        fn()
    e.record()
    torch.cuda.synchronize()
    return s.elapsed_time(e) / reps


def ceilings(B, torch, n_rows: int, row_floats: int):
    """The ceilings of this chip, measured here: see the module docstring."""
    out = {}
    table = torch.randn((n_rows, row_floats), dtype=torch.float32, device="cuda")
    waves, per_wave = 256 * 4 * 7, 2048                       # seven waves per SIMD, 2,048 rows each
    gathered = waves * per_wave * row_floats * 4
    for name, spread in (("gather_l2_hits_GBps", False), ("gather_no_locality_GBps", True)):
        ms = event_time(torch, lambda: B.gcn_ceiling_gather(table, waves, per_wave, spread), 5)
        out[name] = round(gathered / ms / 1e6, 1)
    out["gather_table"] = "%d rows x %d float32 = %.1f MB" % (n_rows, row_floats, n_rows * row_floats * 4 / 1e6)
    src = torch.ones(1 << 30, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    ms = event_time(torch, lambda: B.gcn_calibration_copy(src, dst), 5)
    out["copy_1GiB_read_plus_write_GBps"] = round(2 * (1 << 30) / ms / 1e6, 1)
    del src, dst
    mw, per = 256 * 4 * 4, 4096
    ms = event_time(torch, lambda: B.gcn_ceiling_mfma_bf16(mw, per), 5)
    out["mfma_bf16_32x32x16_TFLOPs"] = round(mw * per * 4 * 32768 / ms / 1e9, 1)
    return out


def sage_leg(B, torch, np, g, wl, args, cpu_baseline):
    """One pass over the train vertices in batches of 256 (hidden 128, S1 = 25, S2 = 10, Adam lr 1e-4): sample,
    both layers, loss, backward, update per batch.  Batches come from a seeded permutation, resident in HBM."""
    from synth import rng
    hidden, s1, s2, bsz = 128, 25, 10, 256
    f, classes = wl.x.shape[1], wl.dims[-1]
    model = B.gcn_sage_create(g, hidden, s1, s2, bsz, seed=args.seed)
    a1, a2 = np.sqrt(6.0 / (2 * f + hidden)), np.sqrt(6.0 / (2 * hidden + classes))
    w1 = ((rng.uniform(args.seed, 901, 2 * f * hidden) * 2 - 1) * a1).astype(np.float32).reshape(2 * f, hidden)
    w2 = ((rng.uniform(args.seed, 902, 2 * hidden * classes) * 2 - 1) * a2).astype(np.float32).reshape(2 * hidden, classes)
    B.gcn_sage_set_weights(model, w1, w2)
    train = np.nonzero(wl.mask)[0]
    order = train[rng.permutation(args.seed, 903, len(train))].astype(np.int32)
    batches = [torch.from_numpy(order[i:i + bsz]).cuda() for i in range(0, len(order), bsz)]

    def one_pass(first_step):
        for k, b in enumerate(batches):
            B.gcn_sage_forward(model, b, first_step + k)
            B.gcn_sage_loss_acc(model, sync=False)
            B.gcn_sage_backward(model)
            B.gcn_sage_adam_step(model, 1e-4)

    one_pass(0)                                        # warm-up pass
    torch.cuda.synchronize()
    B.gcn_timing_reset()
    B.gcn_timing_enable(True)
    t0 = time.perf_counter()
    one_pass(len(batches))
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    B.gcn_timing_enable(False)
    cnt, ms = B.gcn_timing_read(0, B.GCN_TIME_SAGE_GATHER)
    n1 = bsz * (1 + s2)
    ldf = (f + 15) // 16 * 16
    # algorithmic bytes of one full-batch gather: (1 + S1) feature rows read per instance, ids, two rows written
    by = n1 * ((1 + s1) * f * 4 + (1 + s1) * 4 + 2 * ldf * 4)
    full = [1 for b in batches if b.numel() == bsz]
    avg = ms / cnt if cnt else float("nan")
    out = {"workload": wl.name, "hidden": hidden, "S1": s1, "S2": s2, "batch": bsz, "batches": len(batches),
           "lr": 1e-4, "ms_per_batch": round(1e3 * wall / len(batches), 4),
           "epochs_per_s": round(1.0 / wall, 3), "targets_per_s": round(len(order) / wall, 1),
           "gather": {"kernel": "k_sage_concat1", "bound": "hbm", "launches": cnt, "avg_launch_ms": round(avg, 5),
                      "bytes_per_full_launch": by,
                      "achieved": round(by * len(full) / max(len(batches), 1) / avg / 1e6, 1) if cnt else None,
                      "peak": HBM_PEAK_GBS, "unit": "GB/s"}}
    if out["gather"]["achieved"]:
        out["gather"]["frac"] = round(out["gather"]["achieved"] / HBM_PEAK_GBS, 4)
    if cpu_baseline:
        from oracle import gcn_oracle as O
        from oracle import sage_oracle as SO
        og = O.canonicalise(wl.n, wl.rowptr, wl.col)
        ws, state = [w1.astype(np.float64), w2.astype(np.float64)], {}
        t0 = time.perf_counter()
        done = 0
        for k in range(len(batches)):
            b = order[k * bsz:(k + 1) * bsz]
            t = SO.forward(og.rowptr, og.col, wl.x, ws[0], ws[1], b, s1, s2, args.seed, k)
            d1, d2 = SO.backward(t, ws[1], wl.labels[b], s2)
            ws = O.adam(ws, [d1, d2], state, 1e-4)
            done += 1
            if time.perf_counter() - t0 > 10.0:
                break
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": round(done / dt, 3), "unit": "batches/s", "kind": "oracle",
                               "cores": int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)),
                               "sample": "%d batches of %d in %.1f s (numpy fp64)" % (done, bsz, dt),
                               "gpu_batches_per_s": round(len(batches) / wall, 1)}
    del model
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None,
                    help="timed epochs; default: about 2 s of them (the chip's clock under a training loop settles "
                         "within a few tenths of a second, and it is the settled rate that a training run sees)")
    ap.add_argument("--warmup", type=int, default=None,
                    help="untimed epochs before them; default: about 0.5 s of them")
    ap.add_argument("--workload", default="c3", choices=["c1", "c2", "c3", "c4", "c5"])
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--dtype", default=None, choices=["f32", "bf16"],
                    help="storage type of features, activations and gradients (sums are always float32); default: the "
                         "workload's own (f32, c5: bf16).  The parity bar is 1e-4 in f32 and 2e-2 in bf16")
    ap.add_argument("--optimizer", default="sgd", choices=["sgd", "adam"],
                    help="update rule of the timed epochs (the paper trains with Adam, lr 0.02)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibration-copy-mib", type=int, default=0,
                    help="also run one plain copy kernel of this many MiB (scales rocprofv3 byte counters)")
    ap.add_argument("--cache-ax", type=int, default=1, choices=[0, 1, 2],
                    help="layer 1 as (A_hat X) W_1 from a cached A_hat X: 0 never, 1 the library's default (when the "
                         "input is not wider than the first hidden layer), 2 always; the headline run is the default")
    ap.add_argument("--no-alt-mode", action="store_true",
                    help="skip the extra timed runs (cache_ax switch flipped; vertex ids shuffled)")
    ap.add_argument("--no-kernel-timing", action="store_true",
                    help="skip the second timed region with events around every launch, and the ceiling kernels")
    ap.add_argument("--sage", action="store_true",
                    help="also time the second network of the paper, GraphSAGE-mean in batches of 256 (Section 4.1), "
                         "over one pass of the train vertices; reported under \"sage\" in the same line")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (one partition = one worker's share of the "
              "data-parallel scheme); --gpus %d is not supported" % args.gpus, file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2012_04930_amd import binding as B
    from synth import workloads

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    B.lib()

    t0 = time.perf_counter()
    wl = workloads.BY_NAME[args.workload](seed=args.seed)
    t_gen = time.perf_counter() - t0
    if args.dtype:
        wl.dtype = args.dtype
    dtype = B.GCN_BF16 if wl.dtype == "bf16" else B.GCN_F32
    esize = 2 if dtype == B.GCN_BF16 else 4

    t0 = time.perf_counter()
    g = gpu_graph(B, torch, np, wl, dtype)
    torch.cuda.synchronize()
    t_create = time.perf_counter() - t0
    info = B.gcn_graph_info(g)
    tile_info = B.gcn_graph_tile_info(g)

    def timed_run(model, lr, steps, timing_level):
        def epoch():
            B.gcn_forward(model, True)
            B.gcn_loss_acc(model, sync=False)     # loss, accuracy and dLoss/dlogits are computed; the two scalars
            B.gcn_backward(model)                 # are read back once, after the timed region
            if args.optimizer == "adam":
                B.gcn_adam_step(model, lr)
            else:
                B.gcn_sgd_step(model, lr)

        for _ in range(warmup):
            epoch()
        torch.cuda.synchronize()
        B.gcn_timing_reset()
        B.gcn_timing_enable(timing_level)
        start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        start.record()
        for _ in range(steps):
            epoch()
        stop.record()
        torch.cuda.synchronize()
        wall_s = time.perf_counter() - t0
        B.gcn_timing_enable(0)
        return wall_s, start.elapsed_time(stop)

    # the library's default decides whether layer 1 runs from a cached A_hat X (it does when the input is
    # not wider than the first hidden layer); the headline number is that default
    B.gcn_set_tunable("cache_ax", args.cache_ax)
    m = B.gcn_model_create(g, wl.dims, dtype=dtype)
    B.gcn_set_weights(m, wl.weights)
    warmup = 3
    rough_ms = timed_run(m, wl.lr, 5, 0)[1] / 5          # sizes the defaults only
    warmup = args.warmup if args.warmup is not None else max(5, int(500.0 / rough_ms))
    args.steps = args.steps if args.steps is not None else max(20, int(2000.0 / rough_ms))
    wall, ev_ms = timed_run(m, wl.lr, args.steps, 0)

    if args.calibration_copy_mib > 0:
        src = torch.ones(args.calibration_copy_mib << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        B.gcn_calibration_copy(src, dst)
        torch.cuda.synchronize()
        del src, dst

    # final state, read after the timed region
    B.gcn_forward(m, False)
    loss, acc = B.gcn_loss_acc(m)

    E, n = info["nnz"], info["n"]
    E_res = E - tile_info["nnz_dense"] if tile_info["in_use"] else E
    widths = sorted(set(wl.dims[1:]), reverse=True)
    kernels, roofline, ceil, timed_ms = {}, None, None, None
    if not args.no_kernel_timing:
        # second timed region: the same epochs with events around every launch
        k_steps = max(5, min(args.steps, 50))
        _, timed_ev = timed_run(m, wl.lr, k_steps, 2)
        timed_ms = timed_ev / k_steps
        names = {B.GCN_TIME_AGGREGATE: "aggregation", B.GCN_TIME_GATHER: "gather", B.GCN_TIME_TILES: "tiles",
                 B.GCN_TIME_PLANES: "planes", B.GCN_TIME_JOIN: "join", B.GCN_TIME_GEMM_NN: "gemm_nn",
                 B.GCN_TIME_GEMM_TN: "gemm_tn", B.GCN_TIME_GEMM_NT: "gemm_nt", B.GCN_TIME_LOSS: "loss"}
        for part, name in names.items():
            for w in sorted(set(wl.dims[1:])):
                cnt, ms = B.gcn_timing_read(w, part)
                if cnt:
                    kernels["%s.w%d" % (name, w)] = {"launches_per_epoch": round(cnt / k_steps, 2),
                                                     "avg_ms": round(ms / cnt, 5),
                                                     "ms_per_epoch": round(ms / k_steps, 5)}
        # the gather ceilings are taken on a table of the widest aggregated matrix's size and row length in bytes
        w_top = max(d for d in wl.dims[1:])
        ceil = ceilings(B, torch, n + 1, (w_top + 15) // 16 * 16 * esize // 4)
        # the dominant kernel: the one with the most time per epoch among the parts (not the wholes)
        parts = {k: v for k, v in kernels.items() if not k.startswith("aggregation.")}

        def roofline_of(dom):
            kind, w = dom.split(".w")
            w = int(w)
            avg = parts[dom]["avg_ms"]
            ld = (w + 15) // 16 * 16
            if kind == "gather":
                # forward launches gather over the (residual) pattern, the last layer's backward one over the masked
                # pattern: `avg` averages both, so do the bytes
                by = gather_bytes(E_res, n, ld, esize)
                achieved = by / avg / 1e6
                # a gathered matrix that fits the last-level cache (256 MB) is served by the caches: the ceiling is the
                # measured all-L2-hit gather rate; a larger one is served by HBM: the ceiling is the HBM peak
                cached = (n + 1) * ld * esize <= (256 << 20)
                peak = ceil["gather_l2_hits_GBps"] if cached else HBM_PEAK_GBS
                traffic = read_traffic(wl.name, "gather", w) if args.dtype is None else None
                return {"bound": "cache" if cached else "hbm", "kernel": "k_spmm_phased | k_spmm_wave + k_spmm_group: gather over the "
                        + ("%d entries outside the dense tiles" % E_res if tile_info["in_use"] else "whole pattern")
                        + ", width %d" % w,
                        "achieved": round(achieved, 1), "peak": peak, "unit": "GB/s",
                        "frac": round(achieved / peak, 4),
                        "peak_is": ("gather ceiling measured in this run: every gather an L2 hit, table of the "
                                    "aggregated matrix's size (gcn_ceiling_gather)") if cached else
                                   "HBM peak: the gathered matrix is larger than the last-level cache",
                        "bytes_per_launch": by, "avg_launch_ms": avg,
                        "traffic": (traffic["fetch_bytes"] + traffic["write_bytes"]) if traffic else None,
                        "traffic_detail": traffic,
                        "hbm_frac": round((traffic["fetch_bytes"] + traffic["write_bytes"]) / avg / 1e6 / HBM_PEAK_GBS, 4)
                        if traffic else None,
                        "compulsory_GBps": round(compulsory_bytes(E_res, n, ld, esize) / avg / 1e6, 1),
                        "alu_frac_fp32": round(2.0 * E_res * w / (avg * 1e-3) / (FP32_PEAK_TFLOPS * 1e12), 4),
                        "frac_of_no_locality_ceiling": round(achieved / ceil["gather_no_locality_GBps"], 4)}
            if kind == "tiles":
                planes = 1 if dtype == B.GCN_BF16 else 3
                flops = tile_info["n_tiles"] * planes * 2.0 * 128 * 32 * ((w + 31) // 32 * 32)
                achieved = flops / (avg * 1e-3) / 1e12
                traffic = read_traffic(wl.name, "tiles", w) if args.dtype is None else None
                return {"bound": "mfma", "kernel": "k_tiles: %d dense tiles of 128 x 32, %d bfloat16 plane(s), "
                        "width %d" % (tile_info["n_tiles"], planes, w),
                        "achieved": round(achieved, 1), "peak": BF16_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                        "frac": round(achieved / BF16_MFMA_PEAK_TFLOPS, 4),
                        "traffic": (traffic["fetch_bytes"] + traffic["write_bytes"]) if traffic else None,
                        "traffic_detail": traffic,
                        "flops_per_launch": flops, "avg_launch_ms": avg,
                        "frac_of_measured_mfma_ceiling": round(achieved / ceil["mfma_bf16_32x32x16_TFLOPs"], 4)}
            if kind.startswith("gemm"):
                # dense products on the float32 (or bfloat16) matrix instruction: flops of the layers of this width
                ls = [l for l in range(1, len(wl.dims)) if wl.dims[l] == w] if kind != "gemm_nt" else \
                     [l for l in range(1, len(wl.dims) - 1) if wl.dims[l] == w]
                fl = [2.0 * n * wl.dims[l - 1] * wl.dims[l] if kind != "gemm_nt" else 2.0 * n * wl.dims[l] * wl.dims[l + 1]
                      for l in ls]
                flops = sum(fl) / max(len(fl), 1)
                peak = BF16_MFMA_PEAK_TFLOPS if dtype == B.GCN_BF16 else FP32_PEAK_TFLOPS
                achieved = flops / (avg * 1e-3) / 1e12
                return {"bound": "mfma", "kernel": "k_gemm (%s), output width %d" % (kind, w),
                        "achieved": round(achieved, 2), "peak": peak, "unit": "TFLOP/s",
                        "frac": round(achieved / peak, 4), "traffic": None, "flops_per_launch": flops,
                        "avg_launch_ms": avg}
            return {"bound": "hbm", "kernel": dom, "achieved": None, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": None, "traffic": None, "avg_launch_ms": avg}

        if parts:
            dom = max(parts, key=lambda k: parts[k]["ms_per_epoch"])
            # The tile product and the gather of one aggregation run side by side on two streams, each one's time
            # taken while it shares the chip with the other (the two times differ by a tenth and which one is longer
            # changes from run to run).  The pair is reported as one: the gather first (it moves nine tenths of the
            # pair's bytes), the tile product under "runs_beside".
            kind, w = dom.split(".w")
            if kind == "tiles" and "gather.w%s" % w in parts:
                kind = "gather"
            roofline = roofline_of("%s.w%s" % (kind, w))
            roofline["longest_part_by_time"] = dom
            beside = {"tiles": "gather", "gather": "tiles"}.get(kind)
            if beside and "%s.w%s" % (beside, w) in parts:
                roofline["runs_beside"] = roofline_of("%s.w%s" % (beside, w))

    default_cached = len(wl.dims) > 2 and (args.cache_ax == 2 or (args.cache_ax == 1 and wl.dims[0] <= wl.dims[1]))
    other = None
    if not args.no_alt_mode and len(wl.dims) > 2:
        # the other setting of the same switch, timed the same way
        B.gcn_set_tunable("cache_ax", 0 if default_cached else 2)
        try:
            m2 = B.gcn_model_create(g, wl.dims, dtype=dtype)
        finally:
            B.gcn_set_tunable("cache_ax", args.cache_ax)
        B.gcn_set_weights(m2, wl.weights)
        w2, e2 = timed_run(m2, wl.lr, args.steps, 0)
        other = {"layer1_from_cached_AX": not default_cached,
                 "epochs_per_s": round(args.steps / max(w2, e2 / 1e3), 3)}
        del m2
        if wl.name.startswith("c3"):
            # the same partition with its vertex ids scrambled: what a caller gets whose numbering does not keep
            # the vertices of a community together (no dense tiles, no L2 locality)
            wls = workloads.BY_NAME[args.workload](seed=args.seed, shuffle_ids=True)
            gs = gpu_graph(B, torch, np, wls, dtype)
            ms_ = B.gcn_model_create(gs, wls.dims, dtype=dtype)
            B.gcn_set_weights(ms_, wls.weights)
            w3, e3 = timed_run(ms_, wls.lr, max(10, args.steps // 4), 0)
            other["shuffled_ids_epochs_per_s"] = round(max(10, args.steps // 4) / max(w3, e3 / 1e3), 3)
            other["shuffled_ids_dense_tiles_in_use"] = B.gcn_graph_tile_info(gs)["in_use"]
            del ms_, gs, wls

    sage = None
    if args.sage and dtype == B.GCN_F32:
        sage = sage_leg(B, torch, np, g, wl, args, not args.no_cpu_baseline)

    cpu = None
    if not args.no_cpu_baseline:
        from oracle import gcn_oracle as O
        O.lib()
        og = O.canonicalise(wl.n, wl.rowptr, wl.col)
        ws = [w.astype(np.float64) for w in wl.weights]
        x64 = wl.x.astype(np.float64)
        del wl.x
        cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
        n_ep, dt = 0, 0.0
        t0 = time.perf_counter()
        while n_ep < 1 or (dt * cores < 15.0 and n_ep < 5):      # about 15-30 s of CPU work, at most 5 epochs
            ws, _ = O.train_epoch(og, x64, ws, wl.labels, wl.mask, wl.lr)
            n_ep += 1
            dt = time.perf_counter() - t0
        cpu = {"value": round(n_ep / dt, 4), "unit": "epochs/s", "cores": cores, "kind": "oracle",
               "sample": "%d full epoch(s) of %s (fp64 plain loops, OpenMP over rows) in %.1f s wall"
                         % (n_ep, wl.name, dt)}
        # one thread: the forward pass of the first layer's aggregation only, scaled by its share of the epoch's
        # arithmetic (a whole epoch on one thread takes minutes)
        if wl.name.startswith("c3") or wl.name.startswith("c2") or wl.name.startswith("c1"):
            import ctypes
            omp = ctypes.CDLL("libgomp.so.1")
            omp.omp_set_num_threads(1)
            sample_w = wl.dims[1]
            t_in = np.ascontiguousarray(x64[:, :sample_w] if x64.shape[1] >= sample_w else
                                        np.tile(x64, (1, sample_w // x64.shape[1] + 1))[:, :sample_w])
            t0 = time.perf_counter()
            O.aggregate(og, t_in)
            dt1 = time.perf_counter() - t0
            omp.omp_set_num_threads(cores)
            flops_epoch = sum(2.0 * 2 * E * d for d in wl.dims[1:]) + \
                sum(3 * 2.0 * n * a * b for a, b in zip(wl.dims[:-1], wl.dims[1:])) - 2.0 * n * wl.dims[0] * wl.dims[1]
            share = 2.0 * E * sample_w / flops_epoch
            cpu["one_thread"] = {"value": round(share / dt1, 4), "unit": "epochs/s (extrapolated)", "cores": 1,
                                 "sample": "one aggregation of width %d on one thread in %.1f s = %.1f %% of an epoch's "
                                           "flops" % (sample_w, dt1, 100 * share)}

    secs = max(wall, ev_ms / 1e3)
    out = {
        "metric": "GCN train epochs/sec (fwd+bwd) on one partition; SpMM HBM GB/s vs peak",
        "value": round(args.steps / secs, 3), "unit": "epochs/s", "n_gpus": 1, "steps": args.steps,
        "warmup": warmup, "ms_per_step": round(1e3 * secs / args.steps, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": wl.name, "n": n, "n_local": wl.n_local, "nnz_A_plus_I": E, "dims": wl.dims,
                   "lr": wl.lr, "optimizer": args.optimizer, "seed": args.seed, "layer1_from_cached_AX": default_cached,
                   "dense_tiles": tile_info, "entries_gathered": E_res,
                   "vertex_ids": "contiguous per community (what a partitioner's relabelling gives); "
                                 "other_mode.shuffled_ids_* is the same graph with ids scrambled"},
        "loss_readback": False,
        "regime": "the timed epochs follow %d untimed ones back to back (%.1f s in all): the rate at the clock the chip "
                  "settles to under this loop, which is what a training run of many epochs sees" % (warmup + 5, (warmup + 5 + args.steps) * secs / args.steps),
        "other_mode": other,
        "roofline": roofline, "ceilings": ceil, "kernels": kernels,
        "ms_per_step_with_events_around_every_launch": round(timed_ms, 4) if timed_ms else None,
        "cpu_baseline": cpu, "sage": sage,
        "final_loss": round(loss, 6), "final_acc": round(acc, 6),
        "event_ms_total": round(ev_ms, 3), "wall_s_total": round(wall, 4),
        "graph_create_s": round(t_create, 3), "generate_s": round(t_gen, 1),
        "workspace_bytes": int(g.ws.numel() + m.ws.numel()),
        "paper_context": "paper: about 1 s per epoch, Reddit (avg degree 100), 5 x GTX 1080 Ti (Section 1)",
    }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
