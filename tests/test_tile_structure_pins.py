"""Pins for the oracle's integer side (oracle/tw_ref.py: tile_structure): the only numbers the
paper prints for the format (Fig. 4 worked example), the degenerate granularities of Sec. I
(G = whole matrix is global structured pruning, G = 1 is element-wise), and brute-force
reconstruction of the mask from the index lists."""
import os

import numpy as np
import pytest

from oracle import tw_ref
from paper_2008_13006_amd import workloads as W

GOLD = os.path.join(os.path.dirname(__file__), "golden", "fig4_worked_example.txt")


def _gold():
    out = {}
    with open(GOLD) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            key, *vals = line.split()
            out[key] = [int(v) for v in vals]
    return out


def fig4_mask(G: int, K: int):
    """A K x 4G mask built from the paper's words: the four original tiles lose 4, 3, 2, 1 columns,
    the re-grouped tiles then lose 2, 4, 8, 1 rows."""
    g = _gold()
    N = 4 * G
    pruned = []
    for t, c in enumerate(g["cols_pruned_per_original_tile"]):
        pruned += [t * G + G - 1 - 2 * i for i in range(c)]      # towards the end of each original tile
    kept = np.setdiff1d(np.arange(N), pruned)
    mask = np.zeros((K, N), np.uint8)
    for t in range(4):
        cols = kept[t * G:(t + 1) * G]
        rows_gone = [(5 * t + 3 * i) % K for i in range(-g["height_minus_K"][t])]
        rows = np.setdiff1d(np.arange(K), rows_gone)
        mask[np.ix_(rows, cols)] = 1
    return mask, g


@pytest.mark.parametrize("G,K", [(16, 40), (32, 64), (128, 96)])
def test_fig4_worked_example(G, K):
    mask, g = fig4_mask(G, K)
    s = tw_ref.tile_structure(mask, G)
    assert s["T"] == 4
    widths = np.diff(s["tile_col_ptr"])
    spans = np.diff(s["tile_span"])
    heights = np.diff(s["tile_row_ptr"])
    assert (widths - G).tolist() == g["width_minus_G"]
    assert (spans - G).tolist() == g["span_minus_G"]
    assert (heights - K).tolist() == g["height_minus_K"]


def _rebuild(s):
    m = np.zeros((s["K"], s["N"]), np.uint8)
    for t in range(s["T"]):
        cols = s["col_idx"][s["tile_col_ptr"][t]:s["tile_col_ptr"][t + 1]]
        rows = s["row_idx"][s["tile_row_ptr"][t]:s["tile_row_ptr"][t + 1]]
        for r in rows:
            for c in cols:
                m[r, c] = 1
    return m


@pytest.mark.parametrize("seed_offset,G,cp", [(9001, 8, 0.0), (9002, 16, 0.2), (9003, 32, 0.07)])
def test_index_lists_rebuild_the_mask(seed_offset, G, cp):
    spec = W.small_spec("pin_struct", M=1, K=48, N=100, G=G, col_prune=cp, seed_offset=seed_offset)
    w = W.generate(spec, with_A=False)
    s = tw_ref.tile_structure(w.mask, G)
    assert np.array_equal(_rebuild(s), w.mask)
    assert s["nnz"] == int(w.mask.sum())
    # canonical order and ownership
    assert np.all(np.diff(s["col_idx"]) > 0)
    for t in range(s["T"]):
        r = s["row_idx"][s["tile_row_ptr"][t]:s["tile_row_ptr"][t + 1]]
        assert np.all(np.diff(r) > 0)
        c = s["col_idx"][s["tile_col_ptr"][t]:s["tile_col_ptr"][t + 1]]
        assert 1 <= len(c) <= G
        assert s["tile_span"][t] <= c[0] and c[-1] < s["tile_span"][t + 1]
    assert s["tile_span"][0] == 0 and s["tile_span"][-1] == 100
    assert s["T"] == w.info["T"] and np.diff(s["tile_row_ptr"]).tolist() == w.info["k_t"]


def test_whole_matrix_granularity_is_global_row_and_column_pruning():
    """G = N: one tile; the kept rows and columns are global (Sec. I)."""
    K, N = 20, 30
    mask = np.zeros((K, N), np.uint8)
    rows, cols = [1, 4, 5, 19], [0, 2, 3, 29]
    mask[np.ix_(rows, cols)] = 1
    s = tw_ref.tile_structure(mask, N)
    assert s["T"] == 1 and s["row_idx"].tolist() == rows and s["col_idx"].tolist() == cols
    assert s["tile_span"].tolist() == [0, N]


def test_granularity_one_accepts_any_mask():
    """G = 1 is element-wise sparsity (Sec. I): every surviving column is its own tile."""
    rng = np.random.default_rng(0)
    mask = (rng.random((12, 9)) < 0.4).astype(np.uint8)
    mask[:, 3] = 0
    s = tw_ref.tile_structure(mask, 1)
    assert s["T"] == int(mask.any(axis=0).sum())
    assert np.array_equal(_rebuild(s), mask)


def test_unstructured_mask_is_rejected_for_wide_tiles():
    rng = np.random.default_rng(1)
    mask = (rng.random((64, 256)) < 0.5).astype(np.uint8)
    with pytest.raises(tw_ref.NotTileWise):
        tw_ref.tile_structure(mask, 32)


def test_fixed_grid_masks_are_accepted_too():
    """Tiles cut on the fixed N grid before column pruning (the other reading of Sec. IV-A):
    each grid tile's survivors share one row set, so the sweep finds them as they are."""
    K, N, G = 16, 64, 16
    rng = np.random.default_rng(2)
    mask = np.zeros((K, N), np.uint8)
    for t in range(N // G):
        rows = np.flatnonzero(rng.random(K) < 0.5)
        if len(rows) == 0:
            rows = np.array([0])
        cols = t * G + np.flatnonzero(rng.random(G) < 0.8)
        mask[np.ix_(rows, cols)] = 1
    s = tw_ref.tile_structure(mask, G)
    assert np.array_equal(_rebuild(s), mask)
    assert s["T"] <= 2 * (N // G)


def test_empty_mask_has_no_tiles():
    s = tw_ref.tile_structure(np.zeros((8, 40), np.uint8), 8)
    assert s["T"] == 0 and len(s["col_idx"]) == 0 and s["nnz"] == 0


def test_masked_weight_bits():
    B = np.array([[0x3C00, 0x8000], [0xBC00, 0x1234]], np.uint16)
    m = np.array([[1, 0], [0, 1]], np.uint8)
    assert tw_ref.masked_weight_bits(B, m).tolist() == [[0x3C00, 0], [0, 0x1234]]
