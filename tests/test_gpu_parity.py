"""GPU library vs CPU oracle, element by element, on the same seeded inputs (run with -m gpu)."""
import time

import numpy as np
import pytest
import torch

from synth import graphs, rng, workloads
from tests import helpers as H

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2012_04930_amd import binding
    binding.lib()
    return binding


def _say(capsys, text):
    """Progress line that reaches the terminal even under output capture (long tests must not look hung)."""
    with capsys.disabled():
        print("\n    [%s] %s" % (time.strftime("%H:%M:%S"), text), end="", flush=True)


def _heavy_row_workload(n=6000, heavy=(0, 17), seed=3):
    """Small random graph plus two vertices adjacent to almost everyone: rows longer than the
    in-LDS sort limit, so the bit-set path of the canonicalisation is exercised."""
    m = 3 * n
    rowptr, col = graphs.erdos_renyi_gnm(n, m, seed)
    deg = np.diff(rowptr)
    rows = np.repeat(np.arange(n, dtype=np.int64), deg)
    u = [rows, ]
    v = [col.astype(np.int64), ]
    for hv in heavy:
        others = np.nonzero(rng.uniform(seed, 50 + hv, n) < 0.9)[0]
        u.append(np.full(others.size, hv, dtype=np.int64))
        v.append(others)
    rp, cl = graphs.pairs_to_csr(n, np.concatenate(u), np.concatenate(v))
    return graphs.messy_copy(n, rp, cl, seed)


# ------------------------------------------------------------------ graph preparation: bit-exact
@pytest.mark.parametrize("case", ["tiny_messy", "heavy_rows", "isolated", "partition"])
def test_graph_preparation_is_bit_exact(B, oracle, case):
    if case == "tiny_messy":
        wl = workloads.tiny(messy=True)
    elif case == "heavy_rows":
        wl = workloads.tiny(n=6000)
        wl.rowptr, wl.col = _heavy_row_workload()
    elif case == "isolated":
        wl = workloads.tiny(n=300)
        wl.rowptr = np.zeros(301, dtype=np.int64)
        wl.col = np.zeros(0, dtype=np.int32)
    else:
        wl = workloads.reddit_partition(scale=0.05)
    og = oracle.canonicalise(wl.n, wl.rowptr, wl.col)
    g = H.gpu_graph(B, wl)
    info = B.gcn_graph_info(g)
    assert info["n"] == wl.n and info["nnz"] == int(og.rowptr[-1])
    assert info["n_train"] == int(wl.mask.sum()) and info["max_degree"] == int(og.deg.max())
    rowptr, col, deg, dinv = [t.cpu().numpy() for t in B.gcn_graph_get_csr(g)]
    np.testing.assert_array_equal(rowptr, og.rowptr)
    np.testing.assert_array_equal(col, og.col)
    np.testing.assert_array_equal(deg, og.deg)
    np.testing.assert_allclose(dinv, og.dinv, rtol=1e-7)


def test_graph_errors_are_reported_not_raised_by_the_gpu(B):
    wl = workloads.tiny(n=256)
    d = H.to_dev(wl)
    args = lambda **kw: {**d, **kw}

    def create(a):
        return B.gcn_graph_create(a["rowptr"], a["col"], a["x"], a["labels"], a["mask"], wl.dims[-1])

    bad_col = d["col"].clone()
    bad_col[5] = wl.n
    with pytest.raises(B.GcnError) as e:
        create(args(col=bad_col))
    assert e.value.code == -2
    bad_rp = d["rowptr"].clone()
    bad_rp[10] = bad_rp[11] + 1
    with pytest.raises(B.GcnError) as e:
        create(args(rowptr=bad_rp))
    assert e.value.code == -2
    # one direction of an edge removed: no longer symmetric
    rp, cl = wl.rowptr.copy(), wl.col.copy()
    first = int(np.nonzero(np.diff(rp))[0][0])
    cl = np.delete(cl, rp[first])
    rp[first + 1:] -= 1
    with pytest.raises(B.GcnError) as e:
        create(args(rowptr=torch.from_numpy(rp).cuda(), col=torch.from_numpy(cl).cuda()))
    assert e.value.code == -2
    bad_lab = d["labels"].clone()
    bad_lab[3] = wl.dims[-1]
    with pytest.raises(B.GcnError) as e:
        create(args(labels=bad_lab))
    assert e.value.code == -3
    with pytest.raises(B.GcnError) as e:
        create(args(mask=torch.zeros_like(d["mask"])))
    assert e.value.code == -1
    g = create(d)
    m = B.gcn_model_create(g, wl.dims)
    with pytest.raises(B.GcnError) as e:
        B.gcn_backward(m)                      # before forward
    assert e.value.code == -1
    with pytest.raises(B.GcnError):
        B.gcn_model_create(g, [wl.dims[0] + 1, 4, wl.dims[-1]])
    torch.cuda.synchronize()


def test_workspaces_that_are_short_or_misaligned_are_refused(B):
    """Every call that takes a workspace answers GCN_EWORKSPACE (-4) from the host, before a kernel runs, when the
    workspace is one byte short, missing or not 256-byte aligned; a right-sized one is then accepted."""
    import ctypes as C
    wl = workloads.tiny(n=512)
    g = H.gpu_graph(B, wl)
    L = B.lib()
    need = C.c_size_t()
    st = torch.cuda.current_stream().cuda_stream
    nl = len(wl.dims) - 1
    dims = (C.c_int32 * (nl + 1))(*wl.dims)
    assert L.gcn_model_workspace_bytes(g.handle, nl, dims, 0, C.byref(need)) == 0
    ws = torch.empty(need.value + 512, dtype=torch.uint8, device="cuda")
    h = C.c_void_p()
    for ptr, size in ((ws.data_ptr(), need.value - 1), (None, need.value), (ws.data_ptr() + 64, need.value)):
        assert L.gcn_model_create(C.byref(h), g.handle, nl, dims, 0, 0.0, 0, ptr, size, st) == -4
        assert h.value is None and b"workspace" in L.gcn_last_error()
    assert L.gcn_model_create(C.byref(h), g.handle, nl, dims, 0, 0.0, 0, ws.data_ptr(), need.value, st) == 0
    assert L.gcn_model_destroy(h) == 0
    x = torch.zeros((wl.n, 24), device="cuda")
    out = torch.empty_like(x)
    assert L.gcn_aggregate_workspace_bytes(g.handle, 24, 0, C.byref(need)) == 0
    ws = torch.empty(need.value + 512, dtype=torch.uint8, device="cuda")
    for ptr, size in ((ws.data_ptr(), need.value - 1), (None, need.value), (ws.data_ptr() + 128, need.value)):
        assert L.gcn_aggregate(g.handle, x.data_ptr(), out.data_ptr(), 24, 0, ptr, size, st) == -4
    assert L.gcn_aggregate(g.handle, x.data_ptr(), out.data_ptr(), 24, 0, ws.data_ptr(), need.value, st) == 0
    assert L.gcn_sage_workspace_bytes(g.handle, 16, 3, 2, 8, C.byref(need)) == 0
    ws = torch.empty(need.value + 512, dtype=torch.uint8, device="cuda")
    for ptr, size in ((ws.data_ptr(), need.value - 1), (None, need.value), (ws.data_ptr() + 64, need.value)):
        assert L.gcn_sage_create(C.byref(h), g.handle, 16, 3, 2, 8, 0, ptr, size, st) == -4
        assert h.value is None
    torch.cuda.synchronize()


# ------------------------------------------------------------------ aggregation alone
@pytest.mark.parametrize("width", [1, 7, 16, 41, 100, 128, 200, 256])
def test_aggregate_matches_oracle(B, oracle, width):
    wl = workloads.chung_lu_mid(scale=0.03)          # 3,000 vertices, ragged degrees 1..~150
    og = oracle.canonicalise(wl.n, wl.rowptr, wl.col)
    g = H.gpu_graph(B, wl)
    x = rng.normal_f32(width, 1, wl.n * width).reshape(wl.n, width)
    got = B.gcn_aggregate(g, torch.from_numpy(x).cuda()).cpu().numpy()
    H.assert_close(got, oracle.aggregate(og, x), what="A_hat x, width %d" % width)


def test_aggregate_heavy_rows_and_regular_invariant(B, oracle):
    wl = workloads.tiny(n=6000)
    wl.rowptr, wl.col = _heavy_row_workload()
    og = oracle.canonicalise(wl.n, wl.rowptr, wl.col)
    g = H.gpu_graph(B, wl)
    x = rng.normal_f32(9, 1, wl.n * 48).reshape(wl.n, 48)
    got = B.gcn_aggregate(g, torch.from_numpy(x).cuda()).cpu().numpy()
    H.assert_close(got, oracle.aggregate(og, x), what="heavy rows")
    # A_hat sqrt(d) = sqrt(d): holds at any size
    sq = np.sqrt(og.deg.astype(np.float64)).astype(np.float32)[:, None].repeat(4, 1)
    got = B.gcn_aggregate(g, torch.from_numpy(np.ascontiguousarray(sq)).cuda()).cpu().numpy()
    np.testing.assert_allclose(got, sq, rtol=2e-5)


@pytest.mark.parametrize("width,bf", [(7, False), (48, False), (128, False), (256, False), (100, True), (300, True)])
def test_rows_longer_than_the_split_degree_are_summed_in_chunks(B, oracle, width, bf):
    """Three vertices with about 10,800 neighbours each: cut into chunks of 2,048 entries, one wave per chunk."""
    wl = workloads.tiny(n=12000)
    wl.rowptr, wl.col = _heavy_row_workload(n=12000, heavy=(0, 17, 4000))
    og = oracle.canonicalise(wl.n, wl.rowptr, wl.col)
    assert np.sort(og.deg)[-3] > 3 * 2048
    g = H.gpu_graph(B, wl)
    x = rng.normal_f32(width, 8, wl.n * width).reshape(wl.n, width)
    got = B.gcn_aggregate(g, torch.from_numpy(x).cuda(), dtype=B.GCN_BF16 if bf else B.GCN_F32).cpu().numpy()
    H.assert_close(got, oracle.aggregate(og, x), rtol=H.RTOL_BF16 if bf else H.RTOL_F32, what="split rows, width %d" % width)
    again = B.gcn_aggregate(g, torch.from_numpy(x).cuda(), dtype=B.GCN_BF16 if bf else B.GCN_F32).cpu().numpy()
    np.testing.assert_array_equal(got, again)


def test_full_step_with_split_rows(B, oracle):
    wl = workloads.tiny(n=12000)
    wl.rowptr, wl.col = _heavy_row_workload(n=12000, heavy=(0, 17, 4000))
    g = H.gpu_graph(B, wl)
    _, gpu = H.gpu_epoch(B, g, wl)
    _, tr, new = H.oracle_epoch(oracle, wl, gpu=gpu)
    H.compare_epoch(oracle, wl, gpu, tr, new)


# ------------------------------------------------------------------ the whole step
def test_tiny_config_full_step(B, oracle):
    wl = workloads.tiny()                              # config 1
    g = H.gpu_graph(B, wl)
    _, gpu = H.gpu_epoch(B, g, wl)
    _, tr, new = H.oracle_epoch(oracle, wl, gpu=gpu)
    H.compare_epoch(oracle, wl, gpu, tr, new)


@pytest.mark.parametrize("classes", [2, 16, 17, 64, 65, 100, 200])
def test_loss_with_few_and_many_classes(B, oracle, classes):
    """Up to 64 classes a group of 16 lanes takes a vertex, above that a whole wave: both against the oracle, on
    both sides of the switch and of a lane group's width."""
    wl = workloads.tiny(n=1500, classes=classes)
    g = H.gpu_graph(B, wl)
    _, gpu = H.gpu_epoch(B, g, wl)
    _, tr, new = H.oracle_epoch(oracle, wl, gpu=gpu)
    H.compare_epoch(oracle, wl, gpu, tr, new)


@pytest.mark.parametrize("make", [lambda: workloads.chung_lu_mid(scale=0.1),
                                  lambda: workloads.reddit_partition(scale=0.08),
                                  lambda: workloads.rmat_large(scale=0.004)],
                         ids=["chung_lu_10k", "partition_3.7k", "rmat_9.6k_3layers"])
def test_mid_configs_full_step(B, oracle, make):
    wl = make()
    g = H.gpu_graph(B, wl)
    _, gpu = H.gpu_epoch(B, g, wl)
    _, tr, new = H.oracle_epoch(oracle, wl, gpu=gpu)
    H.compare_epoch(oracle, wl, gpu, tr, new)


def test_zero_last_layer_gives_log_c_and_closed_form_gradient(B):
    wl = workloads.tiny(n=1000)
    wl.weights[-1][:] = 0.0
    g = H.gpu_graph(B, wl)
    _, gpu = H.gpu_epoch(B, g, wl)
    assert abs(gpu["loss"] - np.log(7.0)) < 1e-6
    m = wl.mask.astype(bool)
    assert gpu["correct"] == int(np.sum(wl.labels[m] == 0))
    want = m[:, None] * (1.0 / 7 - np.eye(7)[wl.labels]) / m.sum()
    H.assert_close(gpu["dZ"][-1], want, what="dZ_L at W_L = 0")


def test_two_epochs_and_determinism(B, oracle):
    wl = workloads.chung_lu_mid(scale=0.05)
    g = H.gpu_graph(B, wl)
    runs = []
    for _ in range(2):
        m = B.gcn_model_create(g, wl.dims)
        B.gcn_set_weights(m, wl.weights)
        losses = []
        for _e in range(3):
            B.gcn_forward(m, True)
            losses.append(B.gcn_loss_acc(m)[0])
            B.gcn_backward(m)
            B.gcn_sgd_step(m, 0.5)
        runs.append((losses, [B.gcn_get_tensor(m, B.GCN_T_W, l).cpu().numpy() for l in (1, 2)]))
    assert runs[0][0] == runs[1][0]
    for a, b in zip(runs[0][1], runs[1][1]):
        np.testing.assert_array_equal(a, b)                      # no float atomics anywhere: bit-identical
    og = oracle.canonicalise(wl.n, wl.rowptr, wl.col)
    ws = [w.astype(np.float64) for w in wl.weights]
    ref_losses = []
    for _e in range(3):
        ws, tr = oracle.train_epoch(og, wl.x, ws, wl.labels, wl.mask, lr=0.5)
        ref_losses.append(tr.loss)
    np.testing.assert_allclose(runs[0][0], ref_losses, rtol=1e-4)
    for a, b in zip(runs[0][1], ws):
        H.assert_close(a, b, what="weights after 3 epochs")


def test_dropout_mask_and_scaling(B, oracle):
    wl = workloads.chung_lu_mid(scale=0.02)
    g = H.gpu_graph(B, wl)
    p, seed = 0.4, 12345
    _, gpu = H.gpu_epoch(B, g, wl, dropout_p=p, seed=seed, training=True)
    _, tr, new = H.oracle_epoch(oracle, wl, dropout_p=p, seed=seed, training=True, gpu=gpu)
    keep = oracle.dropout_keep(seed, 0, 1, wl.n, wl.dims[1], p)
    assert np.all(gpu["H"][0][keep == 0] == 0.0)                  # same mask, bit for bit
    H.compare_epoch(oracle, wl, gpu, tr, new)
    # evaluation mode ignores dropout
    _, gpu_eval = H.gpu_epoch(B, g, wl, dropout_p=p, seed=seed, training=False)
    _, tr_eval, _ = H.oracle_epoch(oracle, wl, dropout_p=p, seed=seed, training=False)
    H.assert_close(gpu_eval["logits"], tr_eval.Z[-1], what="eval logits")


# ------------------------------------------------------------------ full sizes, in the launch configuration bench.py times
def test_benchmark_config_c3_full_size(B, oracle, capsys):
    wl = workloads.reddit_partition()                  # 47,532 vertices, 23.7 M nonzeros, 602 -> 128 -> 41
    g = H.gpu_graph(B, wl)
    og = oracle.canonicalise(wl.n, wl.rowptr, wl.col)
    rowptr, col, deg, dinv = [t.cpu().numpy() for t in B.gcn_graph_get_csr(g)]
    np.testing.assert_array_equal(rowptr, og.rowptr)
    np.testing.assert_array_equal(col, og.col)
    np.testing.assert_array_equal(deg, og.deg)
    _, gpu = H.gpu_epoch(B, g, wl)
    _, tr, new = H.oracle_epoch(oracle, wl, gpu=gpu, say=lambda t: _say(capsys, "c3: oracle " + t))
    H.compare_epoch(oracle, wl, gpu, tr, new, say=lambda t: _say(capsys, "c3: " + t))


def test_benchmark_config_c3_full_size_in_bfloat16_storage(B, oracle, capsys):
    """The launch configuration `bench.py --dtype bf16` times: dense tiles on widened rows beside the gather."""
    wl = workloads.reddit_partition()
    g = H.gpu_graph(B, wl, dtype=B.GCN_BF16)
    assert B.gcn_graph_tile_info(g)["in_use"]
    _, gpu = H.gpu_epoch(B, g, wl, dtype=B.GCN_BF16, cache_ax=0)
    _, tr, new = H.oracle_epoch(oracle, wl, gpu=gpu, bf16=True, say=lambda t: _say(capsys, "c3 bf16: oracle " + t))
    H.compare_epoch(oracle, wl, gpu, tr, new, rtol=H.RTOL_BF16, say=lambda t: _say(capsys, "c3 bf16: " + t))


def test_config_c2_full_size(B, oracle, capsys):
    wl = workloads.chung_lu_mid()                      # 100,000 vertices, light and heavy rows mixed
    g = H.gpu_graph(B, wl)
    _, gpu = H.gpu_epoch(B, g, wl)
    _, tr, new = H.oracle_epoch(oracle, wl, gpu=gpu, say=lambda t: _say(capsys, "c2: oracle " + t))
    H.compare_epoch(oracle, wl, gpu, tr, new, say=lambda t: _say(capsys, "c2: " + t))


@pytest.mark.timeout(900)
def test_config_c4_full_reddit_shape(B, oracle, capsys):
    _say(capsys, "c4: generating 232,965 vertices")
    wl = workloads.reddit_full()                       # 232,965 vertices, ~114 M nonzeros, rows up to ~10 k entries
    _say(capsys, "c4: graph preparation on GPU and in the oracle")
    g = H.gpu_graph(B, wl)
    og = oracle.canonicalise(wl.n, wl.rowptr, wl.col)
    rowptr, col, deg, _ = [t.cpu().numpy() for t in B.gcn_graph_get_csr(g)]
    np.testing.assert_array_equal(rowptr, og.rowptr)
    np.testing.assert_array_equal(col, og.col)
    np.testing.assert_array_equal(deg, og.deg)
    del rowptr, col, deg
    _say(capsys, "c4: GPU epoch")
    _, gpu = H.gpu_epoch(B, g, wl)
    _say(capsys, "c4: oracle epoch")
    _, tr, new = H.oracle_epoch(oracle, wl, gpu=gpu, say=lambda t: _say(capsys, "c4: oracle " + t))
    _say(capsys, "c4: comparing")
    H.compare_epoch(oracle, wl, gpu, tr, new, say=lambda t: _say(capsys, "c4: " + t))


# ------------------------------------------------------------------ bfloat16 storage, fp32 accumulation (tolerance 2e-2)
@pytest.mark.parametrize("width", [7, 47, 100, 256, 300])
def test_aggregate_bf16_storage(B, oracle, width):
    wl = workloads.chung_lu_mid(scale=0.03)
    og = oracle.canonicalise(wl.n, wl.rowptr, wl.col)
    g = H.gpu_graph(B, wl)
    x = rng.normal_f32(width, 2, wl.n * width).reshape(wl.n, width)
    got = B.gcn_aggregate(g, torch.from_numpy(x).cuda(), dtype=B.GCN_BF16).cpu().numpy()
    H.assert_close(got, oracle.aggregate(og, x), rtol=H.RTOL_BF16, what="bf16 A_hat x, width %d" % width)
    # with an input that is exactly representable the only error left is fp32 summation order
    xi = np.round(x * 4).astype(np.float32) / 4 * (og.deg[:, None] == og.deg[:, None])
    ones = np.ones((wl.n, 8), dtype=np.float32)
    got1 = B.gcn_aggregate(g, torch.from_numpy(ones).cuda(), dtype=B.GCN_BF16).cpu().numpy()
    H.assert_close(got1, oracle.aggregate(og, ones), rtol=H.RTOL_BF16, what="bf16 A_hat 1")


@pytest.mark.parametrize("make", [lambda: workloads.tiny(),
                                  lambda: workloads.chung_lu_mid(scale=0.1),
                                  lambda: workloads.reddit_partition(scale=0.08),
                                  lambda: workloads.rmat_large(scale=0.004)],
                         ids=["tiny", "chung_lu_10k", "partition_3.7k", "rmat_9.6k_3layers"])
def test_full_step_bf16_storage(B, oracle, make):
    wl = make()
    g = H.gpu_graph(B, wl, dtype=B.GCN_BF16)
    _, gpu = H.gpu_epoch(B, g, wl, dtype=B.GCN_BF16)
    _, tr, new = H.oracle_epoch(oracle, wl, gpu=gpu, bf16=True)
    H.compare_epoch(oracle, wl, gpu, tr, new, rtol=H.RTOL_BF16)


def test_model_and_graph_storage_types_must_agree(B):
    wl = workloads.tiny(n=256)
    g = H.gpu_graph(B, wl)
    with pytest.raises(B.GcnError) as e:
        B.gcn_model_create(g, wl.dims, dtype=B.GCN_BF16)
    assert e.value.code == -1


@pytest.mark.timeout(1700)
def test_config_c5_full_size_bf16(B, oracle, capsys):
    _say(capsys, "c5: generating 2.4 M vertices")
    wl = workloads.rmat_large()                        # 2.4 M vertices, 122.4 M nonzeros, 100 -> 256 -> 256 -> 47
    _say(capsys, "c5: graph preparation on GPU and in the oracle")
    g = H.gpu_graph(B, wl, dtype=B.GCN_BF16)
    og = oracle.canonicalise(wl.n, wl.rowptr, wl.col)
    rowptr, col, deg, _ = [t.cpu().numpy() for t in B.gcn_graph_get_csr(g)]
    np.testing.assert_array_equal(rowptr, og.rowptr)
    np.testing.assert_array_equal(col, og.col)
    np.testing.assert_array_equal(deg, og.deg)
    del rowptr, col, deg, og
    _say(capsys, "c5: GPU epoch")
    _, gpu = H.gpu_epoch(B, g, wl, dtype=B.GCN_BF16)
    _say(capsys, "c5: oracle epoch (about a minute of fp64 loops)")
    _, tr, new = H.oracle_epoch(oracle, wl, gpu=gpu, bf16=True, say=lambda t: _say(capsys, "c5: oracle " + t))
    _say(capsys, "c5: comparing")
    H.compare_epoch(oracle, wl, gpu, tr, new, rtol=H.RTOL_BF16, say=lambda t: _say(capsys, "c5: " + t))


# ------------------------------------------------------------------ layer 1 from the cached A_hat X
@pytest.mark.parametrize("dtype_name", ["f32", "bf16"])
@pytest.mark.parametrize("case", ["partition_602_to_128", "rmat_100_to_256_3layers", "chung_lu_dropout"])
def test_first_layer_from_cached_aggregate(B, oracle, case, dtype_name):
    bf = dtype_name == "bf16"
    dtype = B.GCN_BF16 if bf else B.GCN_F32
    rtol = H.RTOL_BF16 if bf else H.RTOL_F32
    p = 0.0
    if case == "partition_602_to_128":
        wl = workloads.reddit_partition(scale=0.08)     # 602 columns: the cached product is built in three column slabs
    elif case == "rmat_100_to_256_3layers":
        wl = workloads.rmat_large(scale=0.004)
    else:
        wl = workloads.chung_lu_mid(scale=0.05)
        p = 0.3
        # inverted dropout multiplies kept values, and their rounding errors, by 1/(1-p) but the rms of the
        # tensor (a fraction p of it zeroed) only by 1/sqrt(1-p): the bfloat16 bound scales with the ratio
        if bf:
            rtol = rtol / np.sqrt(1.0 - p)
    g = H.gpu_graph(B, wl, dtype=dtype)
    results = {}
    for mode in (0, 2):
        _, gpu = H.gpu_epoch(B, g, wl, dtype=dtype, cache_ax=mode, dropout_p=p, seed=77)
        _, tr, new = H.oracle_epoch(oracle, wl, gpu=gpu, bf16=bf, dropout_p=p, seed=77)
        H.compare_epoch(oracle, wl, gpu, tr, new, rtol=rtol)
        results[mode] = gpu
    assert results[0]["G"][0] is not None and results[2]["G"][0] is None


# ------------------------------------------------------------------ layer 1's product on the bfloat16 instruction
@pytest.mark.parametrize("cache_ax", [0, 2])
def test_split_product_and_epilogue_planes_against_the_plain_paths(B, oracle, cache_ax):
    """Layer 1's feature transform from packed three-plane operands ("gemm_split") against the float32 matrix
    instruction: both within the bar of the oracle, and within 1e-5 of each other.  The operand planes that the
    dense products write for the tile product ("fused_planes") are bit for bit what the separate pass writes, so
    every tensor of the epoch is identical with and without; so it is with the upper layer's weight gradient beside
    the input gradient ("tn_beside") or in line.  Layer 1's weight gradient the same way ("gemm_split_tn", the shared
    index being the vertices, cut over workgroups) against the float32 one.  A partition with dense tiles, 602 input columns (19 k-blocks, the
    last one padded), dropout on."""
    wl = workloads.reddit_partition(scale=0.12)
    g = H.gpu_graph(B, wl)
    assert B.gcn_graph_tile_info(g)["in_use"]
    runs = {}
    try:
        for split, fused in ((2, 1), (0, 1), (2, 0)):
            B.gcn_set_tunable("gemm_split", split)
            B.gcn_set_tunable("fused_planes", fused)
            _, runs[(split, fused)] = H.gpu_epoch(B, g, wl, cache_ax=cache_ax, dropout_p=0.25, seed=5)
        B.gcn_set_tunable("gemm_split", 2)
        B.gcn_set_tunable("fused_planes", 1)
        B.gcn_set_tunable("tn_beside", 0)       # the upper layer's weight gradient in line instead of beside
        _, in_line = H.gpu_epoch(B, g, wl, cache_ax=cache_ax, dropout_p=0.25, seed=5)
        B.gcn_set_tunable("tn_beside", 1)
        B.gcn_set_tunable("gemm_split_tn", 0)   # layer 1's weight gradient on the float32 instruction
        _, runs["tn32"] = H.gpu_epoch(B, g, wl, cache_ax=cache_ax, dropout_p=0.25, seed=5)
    finally:
        B.gcn_set_tunable("gemm_split", 1)
        B.gcn_set_tunable("fused_planes", 1)
        B.gcn_set_tunable("tn_beside", 1)
        B.gcn_set_tunable("gemm_split_tn", 1)
    for name in ("H", "dW", "W", "dZ"):
        for x, y in zip(runs[(2, 1)][name], in_line[name]):
            np.testing.assert_array_equal(x, y)
    for key, gpu in runs.items():
        _, tr, new = H.oracle_epoch(oracle, wl, gpu=gpu, dropout_p=0.25, seed=5)
        H.compare_epoch(oracle, wl, gpu, tr, new, rtol=H.RTOL_F32)
    a, b, c, d = runs[(2, 1)], runs[(0, 1)], runs[(2, 0)], runs["tn32"]
    for name in ("H", "dW", "W"):
        for x, y, z, u in zip(a[name], b[name], c[name], d[name]):
            np.testing.assert_array_equal(x, z)                                  # planes from the epilogue or not
            for other in (y, u):
                scale = float(np.sqrt(np.mean(np.square(other.astype(np.float64))))) + 1e-30
                assert float(np.max(np.abs(x.astype(np.float64) - other))) <= 1e-5 * scale * 8.0, name
    for x, u in zip(a["H"], d["H"]):
        np.testing.assert_array_equal(x, u)                                      # (the forward pass is the same one)
    np.testing.assert_array_equal(a["logits"], c["logits"])


@pytest.mark.parametrize("n,f,hidden,classes", [(1999, 300, 16, 7), (2500, 256, 48, 5), (3001, 515, 200, 9),
                                                 (700, 260, 128, 3), (4130, 1030, 72, 11)])
def test_split_products_on_ragged_shapes(B, oracle, n, f, hidden, classes):
    """Both forms of the three-plane product at sizes that end inside a tile everywhere: vertex counts that are no
    multiple of 32 (the weight gradient's shared index, cut over workgroups: 3 cuts for 700 vertices, up to 17
    for the others), input widths that are no multiple of 32 or 128 (its rows; the transform's shared index), hidden
    widths of half a column tile, one and a half, two and a quarter, four, and six and a quarter (the last column
    group of a workgroup partly or wholly past the end).  Layer 1 from the cached A_hat X, so that both forms run, then the
    default form, where only the transform does."""
    wl = workloads.tiny(n=n, classes=classes)
    wl.dims = [f, hidden, classes]
    wl.x = workloads._features(11, n, f)
    wl.weights = workloads.glorot_weights(wl.dims, 12)
    g = H.gpu_graph(B, wl)
    B.gcn_set_tunable("gemm_split", 2)
    try:
        for mode in (2, 0):
            _, gpu = H.gpu_epoch(B, g, wl, cache_ax=mode)
            _, tr, new = H.oracle_epoch(oracle, wl, gpu=gpu)
            H.compare_epoch(oracle, wl, gpu, tr, new, rtol=H.RTOL_F32)
    finally:
        B.gcn_set_tunable("gemm_split", 1)


# ------------------------------------------------------------------ Adam
def test_adam_update_kernel_matches_oracle(B, oracle):
    count = 100_003
    w0 = rng.normal_f32(21, 1, count) * 0.1
    w = torch.from_numpy(w0.copy()).cuda()
    m = torch.zeros(count, device="cuda")
    v = torch.zeros(count, device="cuda")
    state, ref = {}, [w0.astype(np.float64)]
    # the C ABI carries lr, beta1, beta2, eps as float32: the oracle gets exactly those numbers
    lr, b1, b2, eps = (float(np.float32(x)) for x in (0.02, 0.9, 0.999, 1e-8))
    for t in range(1, 7):
        g = rng.normal_f32(21, 10 + t, count) * (10.0 ** -(t % 4 + 2))      # magnitudes 1e-2 .. 1e-5
        g[::97] = 0.0
        B.gcn_adam_update(w, torch.from_numpy(g).cuda(), m, v, lr=0.02, step=t)
        ref = oracle.adam(ref, [g], state, lr, b1, b2, eps)
        H.assert_close(w.cpu().numpy(), ref[0], rtol=1e-5, what="weights after Adam step %d" % t)
    H.assert_close(m.cpu().numpy(), state["m"][0], rtol=1e-5, what="first moment")
    H.assert_close(v.cpu().numpy(), state["v"][0], rtol=1e-5, what="second moment")


def test_training_with_adam_follows_the_oracle(B, oracle):
    wl = workloads.chung_lu_mid(scale=0.05)
    g = H.gpu_graph(B, wl)
    m = B.gcn_model_create(g, wl.dims)
    B.gcn_set_weights(m, wl.weights)
    og = oracle.canonicalise(wl.n, wl.rowptr, wl.col)
    ws = [w.astype(np.float64) for w in wl.weights]
    state = {}
    gpu_loss, ref_loss = [], []
    lr, b1, b2, eps = (float(np.float32(x)) for x in (0.02, 0.9, 0.999, 1e-8))
    for _e in range(6):
        B.gcn_forward(m, True)
        gpu_loss.append(B.gcn_loss_acc(m)[0])
        B.gcn_backward(m)
        B.gcn_adam_step(m, 0.02)
        tr = oracle.backward(og, oracle.forward(og, wl.x, ws), ws, wl.labels, wl.mask)
        ref_loss.append(tr.loss)
        ws = oracle.adam(ws, tr.dW, state, lr, b1, b2, eps)
    # Adam divides by sqrt(v): where a gradient entry is ~0 the quotient amplifies fp32-vs-fp64 differences, so
    # weights are compared as a whole (relative Frobenius error) and by the share of entries within 1e-3
    np.testing.assert_allclose(gpu_loss, ref_loss, rtol=2e-4)
    assert gpu_loss[-1] < gpu_loss[0] - 0.05            # Adam at the paper's learning rate actually learns
    for l in (1, 2):
        got = B.gcn_get_tensor(m, B.GCN_T_W, l).cpu().numpy().astype(np.float64)
        rel = np.linalg.norm(got - ws[l - 1]) / np.linalg.norm(ws[l - 1])
        close = np.abs(got - ws[l - 1]) <= 1e-3 * np.maximum(np.abs(ws[l - 1]), np.sqrt(np.mean(ws[l - 1] ** 2)))
        assert rel < 1e-3 and close.mean() > 0.999, (l, rel, close.mean())


# ------------------------------------------------------------------ phased aggregation schedule
@pytest.mark.parametrize("width,bf", [(w, b) for b in (False, True) for w in (24, 41, 64, 128, 200, 256)] + [(300, True)],
                         ids=lambda v: ("bf16" if v else "f32") if isinstance(v, bool) else str(v))
def test_phased_schedule_matches_oracle_and_the_plain_schedule(B, oracle, width, bf):
    wl = workloads.reddit_partition(scale=0.1)          # 4.7 k vertices, every row has >= 32 entries
    og = oracle.canonicalise(wl.n, wl.rowptr, wl.col)
    assert og.deg.min() >= 32
    g = H.gpu_graph(B, wl)
    x = rng.normal_f32(width, 3, wl.n * width).reshape(wl.n, width)
    xd = torch.from_numpy(x).cuda()
    dtype = B.GCN_BF16 if bf else B.GCN_F32
    out = {}
    for knob in (0, 1):
        B.gcn_set_tunable("spmm_phased", knob)
        try:
            out[knob] = B.gcn_aggregate(g, xd, dtype=dtype).cpu().numpy()
        finally:
            B.gcn_set_tunable("spmm_phased", -1)
    ref = oracle.aggregate(og, x)
    for knob in (0, 1):
        H.assert_close(out[knob], ref, rtol=H.RTOL_BF16 if bf else H.RTOL_F32, what="schedule %d" % knob)
    # same terms, another order of summation: the two schedules agree to rounding
    np.testing.assert_allclose(out[1], out[0], rtol=0, atol=3e-6 * np.abs(ref).max() * (300 if bf else 1))


@pytest.mark.parametrize("width", [41, 128])
def test_phased_schedule_with_every_number_of_column_ranges_per_phase(B, oracle, width):
    """A phase may take 1, 2, 4 or 8 adjacent column ranges: every entry is still added exactly once."""
    wl = workloads.reddit_partition(scale=0.1)
    og = oracle.canonicalise(wl.n, wl.rowptr, wl.col)
    g = H.gpu_graph(B, wl)
    x = rng.normal_f32(width, 5, wl.n * width).reshape(wl.n, width)
    xd = torch.from_numpy(x).cuda()
    ref = oracle.aggregate(og, x)
    B.gcn_set_tunable("spmm_phased", 1)
    try:
        for group in (1, 2, 4, 8, 0):
            B.gcn_set_tunable("phased_group", group)
            H.assert_close(B.gcn_aggregate(g, xd).cpu().numpy(), ref, rtol=H.RTOL_F32, what="group %d" % group)
    finally:
        B.gcn_set_tunable("spmm_phased", -1)
        B.gcn_set_tunable("phased_group", 0)


def test_partition_with_scrambled_vertex_ids(B, oracle):
    """The same kind of partition with its vertex ids scrambled: the search for dense tiles finds next to none, the
    aggregation is one gather over the whole pattern, and the phased schedule (forced here: the graph is small)
    sizes its phases for entries spread over all columns.  Aggregation at two widths and a whole epoch against the
    oracle."""
    wl = workloads.reddit_partition(scale=0.2, avg_degree=100.0, shuffle_ids=True)   # (1 % of all pairs, as at full size)
    g = H.gpu_graph(B, wl)
    info = B.gcn_graph_tile_info(g)
    assert not info["in_use"] and info["nnz_dense"] * 16 < B.gcn_graph_info(g)["nnz"]
    og = oracle.canonicalise(wl.n, wl.rowptr, wl.col)
    B.gcn_set_tunable("spmm_phased", 1)
    try:
        for width in (41, 128):
            x = rng.normal_f32(width, 8, wl.n * width).reshape(wl.n, width)
            got = B.gcn_aggregate(g, torch.from_numpy(x).cuda()).cpu().numpy()
            H.assert_close(got, oracle.aggregate(og, x), rtol=H.RTOL_F32, what="scrambled ids, width %d" % width)
        _, gpu = H.gpu_epoch(B, g, wl)
    finally:
        B.gcn_set_tunable("spmm_phased", -1)
    _, tr, new = H.oracle_epoch(oracle, wl, gpu=gpu)
    H.compare_epoch(oracle, wl, gpu, tr, new, rtol=H.RTOL_F32)


def test_workgroups_are_dealt_round_robin_over_the_xcds(B):
    """The aggregation kernels give the workgroups b with equal b mod 8 one contiguous range of rows and count on them
    sharing an XCD (and its L2).  That rests on this dispatch order: workgroup b runs on XCD (b + s) mod 8, with a
    start s that depends on the queue (0 and 7 have been seen) but not on b."""
    for nb in (64, 1488, 20000):
        ids = B.gcn_xcc_ids(nb).cpu().numpy()
        assert 0 <= ids.min() and ids.max() <= 7
        np.testing.assert_array_equal(ids, (np.arange(nb) + int(ids[0])) % 8)
