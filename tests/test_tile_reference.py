"""The numpy restatement of the dense-tile split (tiles of 128 rows x 32 columns) that the GPU tests compare against (tests/helpers.tile_split) is
itself checked here, without a GPU: tiles plus residual give back the pattern, and the split obeys its definition."""
import numpy as np
import pytest

from synth import workloads
from tests import helpers as H


@pytest.mark.parametrize("thr", [64, 200])
def test_tiles_plus_residual_are_the_pattern(oracle, thr):
    wl = workloads.reddit_partition(scale=0.05)
    og = oracle.canonicalise(wl.n, wl.rowptr, wl.col)
    n = wl.n
    tile_ptr, tile_col, bits, res_rowptr, res_col, n_dense = H.tile_split(n, og.rowptr, og.col, thr)
    R = H.TILE_ROWS
    n_rt, n_ct = (n + R - 1) // R, (n + 31) // 32
    assert len(tile_ptr) == n_rt + 1 and tile_ptr[-1] == len(tile_col) == len(bits) and bits.shape[1] == R
    # entries of the dense tiles, from the bit words
    rt_of_tile = np.repeat(np.arange(n_rt), np.diff(tile_ptr))
    k, r, c = np.nonzero((bits[:, :, None] >> np.arange(32, dtype=np.uint32)[None, None, :]) & 1)
    rows_d = rt_of_tile[k] * R + r
    assert rows_d.max() < n
    cols_d = tile_col[k].astype(np.int64) * 32 + c
    assert len(rows_d) == n_dense
    per_tile = np.bincount(k, minlength=len(tile_col))
    assert per_tile.min() >= thr                                   # every dense tile holds at least thr entries
    for t in range(n_rt):                                          # ascending column tiles inside a row block
        seg = tile_col[tile_ptr[t]:tile_ptr[t + 1]]
        assert np.all(np.diff(seg) > 0)
    rows_r = np.repeat(np.arange(n), np.diff(res_rowptr))
    # no residual entry lies in a dense tile, and no tile outside the list reaches thr
    dense_keys = set((rt_of_tile * n_ct + tile_col).tolist())
    res_keys, res_cnt = np.unique((rows_r // R) * n_ct + res_col // 32, return_counts=True)
    assert not dense_keys.intersection(res_keys.tolist())
    assert res_cnt.max() < thr
    # together they are exactly the canonical pattern, rows still sorted
    all_rows = np.concatenate([rows_d, rows_r])
    all_cols = np.concatenate([cols_d, res_col.astype(np.int64)])
    order = np.lexsort((all_cols, all_rows))
    want_rows = np.repeat(np.arange(n), np.diff(og.rowptr))
    np.testing.assert_array_equal(all_rows[order], want_rows)
    np.testing.assert_array_equal(all_cols[order], og.col)
    for i in range(0, n, 97):
        seg = res_col[res_rowptr[i]:res_rowptr[i + 1]]
        assert np.all(np.diff(seg) > 0)
