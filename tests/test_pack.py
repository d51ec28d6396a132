"""Host side of the C-ABI library (no GPU needed): the library loads and exports what include/tw.h
declares, tw_pack's integer arrays equal the oracle's tile structure bit for bit, pack -> unpack
gives back B*mask and the mask bit for bit, and bad input is refused with the documented codes."""
import ctypes
import os
import re

import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

from oracle import tw_ref
from paper_2008_13006_amd import binding as tw
from paper_2008_13006_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    text = open(os.path.join(ROOT, "include", "tw.h")).read()
    declared = set(re.findall(r"\b(tw_[a-z_]+)\s*\(", text))
    declared -= {"tw_info_t"}
    assert declared == set(tw.SYMBOLS)
    lib = ctypes.CDLL(tw.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name
    assert tw.tw_version() >= 1


def _check_against_oracle(mask, B, G, dtype):
    blob = tw.tw_pack(B, mask, G, dtype)
    inf = tw.tw_info(blob)
    s = tw_ref.tile_structure(mask, G)
    assert inf["T"] == s["T"] and inf["K"] == s["K"] and inf["N"] == s["N"] and inf["G"] == G
    assert inf["nnz"] == s["nnz"] and inf["n_kept_cols"] == len(s["col_idx"])
    for key in ("col_idx", "tile_col_ptr", "tile_row_ptr", "row_idx", "tile_span"):
        assert np.array_equal(inf[key], s[key]), key
    k_t = np.diff(s["tile_row_ptr"])
    assert np.array_equal(inf["sched_order"], np.argsort(-k_t, kind="stable").astype(np.int32))
    Bu, mu = tw.tw_unpack(blob)
    assert np.array_equal(mu, (mask != 0).astype(np.uint8))
    assert np.array_equal(Bu, tw_ref.masked_weight_bits(B, mask))
    assert inf["padded_macs_per_row"] >= inf["nnz"]
    return inf


@pytest.mark.parametrize("cfg", ["c1_single", "c2_bert_base_ffn_up", "c4_bert_large_skewed", "c5_conv_im2col"])
def test_pack_matches_oracle_on_the_paper_shaped_workloads(cfg):
    for spec in W.CONFIGS[cfg]:
        w = W.generate(spec, with_A=False)
        inf = _check_against_oracle(w.mask, w.B, spec.G, spec.dtype)
        assert inf["T"] == w.info["T"]


def test_pack_matches_oracle_on_the_fixed_grid_mask():
    """Tiles cut on a fixed grid of G original columns (the other description in Sec. IV-A): one tile per grid
    block, and every span starts at its block's first surviving column."""
    spec = W.C2_FIXED_GRID
    w = W.generate(spec, with_A=False)
    inf = _check_against_oracle(w.mask, w.B, spec.G, spec.dtype)
    assert inf["T"] == w.info["T"] == spec.N // spec.G
    ts = tw_ref.tile_structure(w.mask, spec.G)
    assert all(spec.G * t <= int(ts["tile_span"][t]) < spec.G * (t + 1) for t in range(1, ts["T"]))


def test_pack_matches_oracle_bert_base_layer():
    for spec in W.CONFIGS["c3_bert_base_layer"]:
        w = W.generate(spec, with_A=False)
        _check_against_oracle(w.mask, w.B, spec.G, spec.dtype)


def test_fig4_worked_example_through_the_library():
    from tests.test_tile_structure_pins import fig4_mask
    G, K = 32, 64
    mask, g = fig4_mask(G, K)
    B = np.arange(K * 4 * G, dtype=np.uint32).astype(np.uint16).reshape(K, 4 * G)
    inf = _check_against_oracle(mask, B, G, "f16")
    assert (np.diff(inf["tile_col_ptr"]) - G).tolist() == g["width_minus_G"]
    assert (np.diff(inf["tile_span"]) - G).tolist() == g["span_minus_G"]
    assert (np.diff(inf["tile_row_ptr"]) - K).tolist() == g["height_minus_K"]


def test_negative_zero_and_odd_strides_round_trip():
    K, N, G = 40, 70, 32
    rng = np.random.default_rng(0)
    Bbig = rng.integers(0, 65536, size=(K, N + 9)).astype(np.uint16)
    Bbig[3, 5] = 0x8000                                   # -0.0 at a kept position must survive
    mask = np.zeros((K, N), np.uint8)
    mask[np.ix_([1, 3, 8, 39], np.arange(0, 32))] = 1
    mask[np.ix_([0, 3], np.arange(33, 70))] = 1
    blob = tw.tw_pack(Bbig[:, :N], mask, G, "bf16")
    Bu, mu = tw.tw_unpack(blob)
    assert np.array_equal(mu, mask)
    assert np.array_equal(Bu, tw_ref.masked_weight_bits(Bbig[:, :N], mask))
    assert Bu[3, 5] == 0x8000


def test_streamed_k_layout_round_trips():
    """K above the LDS-resident limit switches the blob to chunked K; the integer arrays do not change."""
    spec = W.small_spec("bigk", M=1, K=2304, N=200, G=64, col_prune=0.1, keep=("upow", 0.05, 0.5), seed_offset=9100)
    w = W.generate(spec, with_A=False)
    inf = _check_against_oracle(w.mask, w.B, 64, "f16")
    assert inf["k_chunk"] < 2304


def test_empty_and_full_masks():
    K, N, G = 24, 64, 32
    B = np.full((K, N), 0x3C00, np.uint16)
    inf = _check_against_oracle(np.zeros((K, N), np.uint8), B, G, "f16")
    assert inf["T"] == 0 and inf["nnz"] == 0
    inf = _check_against_oracle(np.ones((K, N), np.uint8), B, G, "f16")
    assert inf["T"] == 2 and inf["nnz"] == K * N and inf["row_idx"].tolist() == list(range(K)) * 2


def test_error_codes():
    K, N = 16, 64
    B = np.zeros((K, N), np.uint16)
    rng = np.random.default_rng(3)
    unstructured = (rng.random((K, N)) < 0.5).astype(np.uint8)
    with pytest.raises(tw.TwError) as e:
        tw.tw_pack(B, unstructured, 32, "f16")
    assert e.value.status == -2                            # TW_ERR_NOT_TILEWISE
    with pytest.raises(tw.TwError) as e:
        tw.tw_pack(B, np.ones((K, N), np.uint8), 48, "f16")
    assert e.value.status == -6                            # TW_ERR_UNSUPPORTED granularity
    with pytest.raises(tw.TwError) as e:
        tw.tw_info(np.zeros(512, np.uint8))
    assert e.value.status == -3                            # TW_ERR_BUF: not a blob
    lib = ctypes.CDLL(tw.LIB_PATH)
    n = ctypes.c_size_t(0)
    assert lib.tw_pack_size(None, 4, 4, 32, 0, ctypes.byref(n)) == -1
    m = np.ones((K, N), np.uint8)
    assert lib.tw_pack_size(ctypes.c_void_p(m.ctypes.data), K, N, 32, 7, ctypes.byref(n)) == -1
    blob = tw.tw_pack(B, m, 32, "f16")
    small = np.zeros(64, np.uint8)
    assert lib.tw_pack(ctypes.c_void_p(B.ctypes.data), N, ctypes.c_void_p(m.ctypes.data), K, N, 32, 0,
                       ctypes.c_void_p(blob.ctypes.data), ctypes.c_size_t(64)) == -3
    assert small.sum() == 0
    assert tw._strerror(-2).startswith("mask is not tile-wise")


@st.composite
def tw_masks(draw):
    G = draw(st.sampled_from([32, 64, 128]))
    K = draw(st.integers(1, 70))
    T = draw(st.integers(1, 4))
    N = draw(st.integers(max(1, (T - 1) * G + 1), T * G + 20))
    seed = draw(st.integers(0, 2 ** 31 - 1))
    rng = np.random.default_rng(seed)
    n_prune = draw(st.integers(0, min(N - 1, 25)))
    pruned = rng.choice(N, size=n_prune, replace=False)
    kept = np.setdiff1d(np.arange(N), pruned)
    mask = np.zeros((K, N), np.uint8)
    for t in range(0, len(kept), G):
        cols = kept[t:t + G]
        kt = int(rng.integers(1, K + 1))
        rows = rng.choice(K, size=kt, replace=False)
        mask[np.ix_(rows, cols)] = 1
    return G, mask, seed


@settings(max_examples=60, deadline=None)
@given(tw_masks())
def test_random_tile_wise_masks_round_trip(arg):
    G, mask, seed = arg
    rng = np.random.default_rng(seed + 1)
    B = rng.integers(0, 65536, size=mask.shape).astype(np.uint16)
    _check_against_oracle(mask, B, G, "f16" if seed % 2 else "bf16")


# ------------------------------------------------------------------ tw_prune (one-shot magnitude pruning)
@pytest.mark.parametrize("K,N,G,dtype,cp,sp", [
    (64, 96, 32, "f16", 0.1, 0.5),
    (96, 200, 64, "f16", 0.05, 0.75),
    (128, 300, 128, "bf16", 0.2, 0.875),
    (40, 70, 32, "bf16", 0.0, 0.3),
    (33, 129, 128, "f16", 0.5, 0.9),
])
def test_tw_prune_matches_oracle_bit_exact(K, N, G, dtype, cp, sp):
    """Library mask == the oracle's plain-loop version of Alg. 1 (magnitude score), bit for bit."""
    rng = np.random.default_rng(4242 + K + N)
    B = W.f32_to_bits((rng.standard_normal((K, N)) * 0.02).astype(np.float32), dtype)
    got = tw.tw_prune(B, G, dtype, cp, sp)
    ref = tw_ref.prune_one_shot(B, G, dtype, cp, sp)
    assert np.array_equal(got, ref)


def test_tw_prune_properties():
    """What Alg. 1 promises: whole columns first, then whole row segments of G regrouped columns; the target
    sparsity is met with at most one segment to spare; the mask packs as TW with ceil(kept/G) tiles."""
    rng = np.random.default_rng(777)
    K, N, G = 96, 260, 64
    B = W.f32_to_bits((rng.standard_normal((K, N)) * 0.05).astype(np.float32), "f16")
    mask = tw.tw_prune(B, G, "f16", 0.1, 0.75)
    kept_cols = np.flatnonzero(mask.any(axis=0))
    assert N - len(kept_cols) == int(np.floor(0.1 * N + 0.5))
    # pruned columns are the least important ones
    cs = np.abs(tw_ref.decode(B, "f16")).sum(axis=0)
    assert cs[kept_cols].min() >= np.delete(cs, kept_cols).max()
    zeros = mask.size - int(mask.sum())
    assert zeros >= 0.75 * mask.size and zeros - G < 0.75 * mask.size
    # row segments: inside a tile of regrouped columns every row is all-kept or all-pruned
    for i in range(0, len(kept_cols), G):
        seg = mask[:, kept_cols[i:i + G]]
        assert np.all((seg.sum(axis=1) == 0) | (seg.sum(axis=1) == seg.shape[1]))
        assert seg.any()
    blob = tw.tw_pack(B, mask, G, "f16")
    assert tw.tw_info(blob)["T"] <= -(-len(kept_cols) // G) + 1
    # tiles differ in kept rows (global ranking across tiles), and sparsity 0 keeps everything
    assert np.array_equal(tw.tw_prune(B, G, "f16", 0.0, 0.0), np.ones((K, N), dtype=np.uint8))


def test_tw_prune_refuses_bad_arguments():
    B = np.zeros((8, 8), dtype=np.uint16)
    for cp, sp in ((-0.1, 0.5), (1.0, 0.5), (0.1, 1.0), (0.1, -0.2)):
        with pytest.raises(tw.TwError):
            tw.tw_prune(B, 32, "f16", cp, sp)


def test_header_is_plain_c(tmp_path):
    """include/tw.h is the boundary: it must compile as C (no C++ or torch types in the signatures)."""
    import subprocess
    src = tmp_path / "use_tw.c"
    src.write_text('#include "tw.h"\nint f(void) { tw_info_t i; (void)i; return (int)sizeof(tw_info_t) + TW_OK; }\n')
    inc = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include")
    r = subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-pedantic", "-I", inc, "-c", str(src), "-o",
                        str(tmp_path / "use_tw.o")], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr


# ------------------------------------------------------------------ TEW hybrid: tile-wise pattern + element-wise residual
@pytest.mark.parametrize("K,N,G,dtype,delta", [(64, 96, 32, "f16", 0.02), (200, 300, 128, "bf16", 0.01),
                                               (96, 128, 64, "f16", 0.0), (40, 70, 32, "f16", 0.2)])
def test_tw_restore_ew_matches_oracle_bit_exact(K, N, G, dtype, delta):
    spec = W.small_spec("tew", M=4, K=K, N=N, G=G, dtype=dtype, col_prune=0.1, keep=("upow", 0.1, 0.6), seed_offset=4242 + K)
    w = W.generate(spec)
    got = tw.tw_restore_ew(w.B, w.mask, delta, dtype)
    ref = tw_ref.restore_ew(w.B, w.mask, delta, dtype)
    assert np.array_equal(got, ref)
    # properties the paper states: only pruned weights come back, exactly delta*K*N of them (if that many are
    # there), none weaker than one that stays pruned - wherever they lie, also in columns pruned altogether
    assert not np.any(got & w.mask)
    n_cand = int((w.mask == 0).sum())
    assert int(got.sum()) == min(n_cand, int(np.floor(delta * K * N + 0.5)))
    if got.any() and n_cand > got.sum():
        mag = np.abs(tw_ref.decode(w.B, dtype))
        left = (w.mask == 0) & (got == 0)
        assert mag[got == 1].min() >= mag[left].max()


def test_tw_restore_ew_matches_the_hand_worked_case():
    """The library on the oracle's hand-worked case (tests/test_oracle_pins.py): the three strongest pruned weights
    lie in the column that the tile-wise pattern removed."""
    B = W.f32_to_bits(np.array([[1, -9, 2, 7, 3, 1], [5, 2, -8, 7, 1, 2], [-3, 4, 6, -7, 2, 3], [2, 1, 5, 1, 8, 4]],
                               np.float32), "f16")
    mask = np.array([[1, 1, 1, 0, 0, 0], [1, 1, 1, 0, 0, 0], [0, 0, 0, 0, 1, 1], [0, 0, 0, 0, 1, 1]], np.uint8)
    got = tw.tw_restore_ew(B, mask, 4 / 24.0, "f16")
    want = np.zeros((4, 6), np.uint8)
    for k, n in [(0, 3), (1, 3), (2, 3), (2, 2)]:
        want[k, n] = 1
    assert np.array_equal(got, want)


def test_tew_pack_round_trip_and_errors():
    spec = W.small_spec("tew_rt", M=4, K=160, N=260, G=64, dtype="f16", col_prune=0.1, keep=("upow", 0.1, 0.5), seed_offset=4300)
    w = W.generate(spec)
    ew = tw_ref.restore_ew(w.B, w.mask, 0.03, "f16")
    blob = tw.tw_pack_tew(w.B, w.mask, ew, spec.G, "f16")
    inf = tw.tw_info(blob)
    assert inf["ew_nnz"] == int(ew.sum()) and inf["nnz"] == int(w.mask.sum())
    # the tile structure is that of the tile-wise pattern alone
    s = tw_ref.tile_structure(w.mask, spec.G)
    for key in ("col_idx", "tile_col_ptr", "tile_row_ptr", "row_idx", "tile_span"):
        assert np.array_equal(inf[key], s[key]), key
    Bu, mu = tw.tw_unpack(blob)
    union = (w.mask | ew).astype(np.uint8)
    assert np.array_equal(mu, union)
    assert np.array_equal(Bu, tw_ref.masked_weight_bits(w.B, union))
    # a restored weight whose value is zero is still part of the mask (the residual is stored as blocks of
    # weights for the matrix cores, most of them zero: which of them are weights is recorded apart)
    Bz = w.B.copy()
    kz, nz = np.argwhere((ew != 0) & w.mask.any(axis=0)[None, :])[5]
    Bz[kz, nz] = 0
    Buz, muz = tw.tw_unpack(tw.tw_pack_tew(Bz, w.mask, ew, spec.G, "f16"))
    assert np.array_equal(muz, union) and np.array_equal(Buz, tw_ref.masked_weight_bits(Bz, union))
    # entries that the tile-wise pattern keeps anyway are ignored
    blob2 = tw.tw_pack_tew(w.B, w.mask, (ew | w.mask).astype(np.uint8), spec.G, "f16")
    assert tw.tw_info(blob2)["ew_nnz"] == int(ew.sum())
    # residual weights in columns without tile-wise weights are part of the blob too (stored by column)
    pruned_cols = np.flatnonzero(~w.mask.any(axis=0))
    assert ew[:, pruned_cols].any()                     # the restored set reaches into pruned columns by itself
    only = np.zeros_like(ew)
    only[3, pruned_cols[0]] = 1
    only[7, pruned_cols[-1]] = 1
    only[150, pruned_cols[-1]] = 1
    blob3 = tw.tw_pack_tew(w.B, w.mask, only, spec.G, "f16")
    assert tw.tw_info(blob3)["ew_nnz"] == 3
    Bu3, mu3 = tw.tw_unpack(blob3)
    assert np.array_equal(mu3, (w.mask | only).astype(np.uint8))
    assert np.array_equal(Bu3, tw_ref.masked_weight_bits(w.B, w.mask | only))
    # a weight without any tile-wise weight at all: every column is of that kind
    none = np.zeros_like(w.mask)
    blob4 = tw.tw_pack_tew(w.B, none, ew, spec.G, "f16")
    inf4 = tw.tw_info(blob4)
    assert inf4["T"] == 0 and inf4["ew_nnz"] == int(ew.sum())
    Bu4, mu4 = tw.tw_unpack(blob4)
    assert np.array_equal(mu4, ew) and np.array_equal(Bu4, tw_ref.masked_weight_bits(w.B, ew))
    # streamed K (several chunks of 384 rows, the last one ragged): the residual is stored per tile and chunk
    big = W.generate(W.small_spec("tew_big", M=4, K=1600, N=200, G=32, dtype="bf16", col_prune=0.1, keep=("upow", 0.05, 0.4),
                                  seed_offset=4301))
    ewb = tw_ref.restore_ew(big.B, big.mask, 0.01, "bf16")
    blob = tw.tw_pack_tew(big.B, big.mask, ewb, 32, "bf16")
    inf = tw.tw_info(blob)
    assert inf["k_chunk"] == 384 and inf["ew_nnz"] == int(ewb.sum()) > 0
    Bu, mu = tw.tw_unpack(blob)
    union = (big.mask | ewb).astype(np.uint8)
    assert np.array_equal(mu, union)
    assert np.array_equal(Bu, tw_ref.masked_weight_bits(big.B, union))


# ------------------------------------------------------------------ the launch plan (host logic, no GPU call)
def _plan(cfg, idx, **kw):
    spec = W.CONFIGS[cfg][idx]
    w = W.generate(spec, with_A=False)
    blob = tw.tw_pack(w.B, w.mask, spec.G, spec.dtype)
    return spec, tw.tw_info(blob), tw.tw_gemm_plan(blob, spec.M, **kw)


def test_plan_of_the_paper_shaped_workloads():
    """What the host decides for the five workloads on 256 compute units."""
    spec, inf, pl = _plan("c2_bert_base_ffn_up", 0)
    assert (pl["mode"], pl["rows_per_block"], pl["n_items"], pl["grid"]) == (0, 64, 256, 256)       # K = 768 resident
    spec, inf, pl = _plan("c1_single", 0)
    # 256 rows are 4 blocks of 64: too few, so 8 blocks of 32 whose 6 tiles are shared out over workgroups
    assert pl["mode"] == 0 and pl["rows_per_block"] == 32 and pl["n_row_blocks"] == 8 and pl["n_sets"] == inf["T"]
    assert pl["n_items"] == 8 * inf["T"] and pl["grid"] == pl["n_items"]
    spec, inf, pl = _plan("c3_bert_base_layer", 3)            # FFN-down, K = 3072 streamed, 6 tiles, 256 row blocks
    assert (pl["mode"], pl["rows_per_block"], pl["tiles_per_set"], pl["n_sets"], pl["n_items"]) == (1, 64, 8, 1, 256)
    spec, inf, pl = _plan("c4_bert_large_skewed", 1)          # K = 4096, 8 tiles, only 128 blocks of 64 rows
    assert inf["T"] == 8
    assert (pl["mode"], pl["rows_per_block"], pl["tiles_per_set"], pl["n_sets"], pl["n_items"]) == (2, 64, 4, 2, 256)
    spec, inf, pl = _plan("c5_conv_im2col", 0)                # K = 2304, 4 tiles
    assert (pl["mode"], pl["rows_per_block"], pl["tiles_per_set"], pl["n_sets"]) == (2, 64, 4, 1)
    assert pl["n_items"] == (spec.M + 63) // 64 and pl["grid"] == 256 and pl["row_lists"] == 0
    spec, inf, plt = _plan("c5_conv_im2col", 0, transposed=True)       # whole 128-byte lines of tokens: 64 stay
    assert plt["mode"] == 2 and plt["rows_per_block"] == 64 and plt["n_items"] == (spec.M + 63) // 64
    assert plt["row_lists"] == 1 and plt["lds_bytes"] > pl["lds_bytes"]
    spec, inf, plt = _plan("c4_bert_large_skewed", 1, transposed=True)
    assert plt["mode"] == 2 and plt["n_sets"] == 2 and plt["row_lists"] == 0     # the lists are per set of eight tiles
    # the hybrid on the same shape, with residual weights in pruned columns: the row lists keep their place in LDS
    # (the per-wave areas for those columns come after them, if there is room), and nothing outgrows the LDS
    spec = W.CONFIGS["c5_conv_im2col"][0]
    w = W.generate(spec, with_A=False)
    mask = w.mask.copy()
    mask[:, -8:] = 0                                          # the last tile loses eight columns: T stays 4
    ew = tw.tw_restore_ew(w.B, mask, 0.01, spec.dtype)
    assert ew[:, -8:].any() and tw.tw_info(tw.tw_pack(w.B, mask, spec.G, spec.dtype))["T"] == 4
    blob = tw.tw_pack_tew(w.B, mask, ew, spec.G, spec.dtype)
    ple, plet = tw.tw_gemm_plan(blob, spec.M), tw.tw_gemm_plan(blob, spec.M, transposed=True)
    assert plet["row_lists"] == 1 and plet["mode"] == 2 and ple["mode"] == 2
    assert max(ple["lds_bytes"], plet["lds_bytes"]) <= 160 * 1024 and ple["lds_bytes"] > pl["lds_bytes"]


def test_plan_fills_the_last_round_on_the_row_major_boundary():
    """Two to four rounds of 64-row blocks with a partly empty last one: lower row blocks (a multiple of 8 rows)
    that fill it; the transposed boundary keeps 64 tokens."""
    spec = W.CONFIGS["c2_bert_base_ffn_up"][0]
    w = W.generate(spec, with_A=False)
    blob = tw.tw_pack(w.B, w.mask, spec.G, spec.dtype)
    for M, rows in ((16384, 64), (17000, 40), (20001, 40), (24576, 48), (32768, 64), (33000, 48), (100352, 64)):
        pl = tw.tw_gemm_plan(blob, M, n_cu=256)
        assert pl["rows_per_block"] == rows and pl["n_row_blocks"] == (M + rows - 1) // rows, (M, pl)
        rounds64 = ((M + 63) // 64 + 255) // 256
        assert (pl["n_items"] + 255) // 256 == rounds64, "no more rounds than 64-row blocks would make"
        assert tw.tw_gemm_plan(blob, M, n_cu=256, transposed=True)["rows_per_block"] == 64


def test_plan_limits_and_errors():
    rng = np.random.default_rng(3)
    for K, N, G in [(64, 256, 128), (1536, 128, 32), (1544, 128, 64), (3000, 300, 128)]:
        B = rng.integers(1, 1000, size=(K, N)).astype(np.uint16)
        mask = np.ones((K, N), dtype=np.uint8)
        blob = tw.tw_pack(B, mask, G, "f16")
        for M in (1, 31, 64, 65, 1000, 100000):
            for n_cu in (1, 8, 256, 304):
                for tr in (False, True):
                    pl = tw.tw_gemm_plan(blob, M, n_cu=n_cu, transposed=tr)
                    if tr and K > 1536:
                        assert pl["rows_per_block"] == 64      # the streamed transposed kernels take 64 tokens
                    assert pl["lds_bytes"] <= 160 * 1024
                    assert 32 <= pl["rows_per_block"] <= 64 and pl["rows_per_block"] % 8 == 0
                    assert pl["rows_per_block"] in (32, 64) or not tr
                    assert pl["n_row_blocks"] == (M + pl["rows_per_block"] - 1) // pl["rows_per_block"]
                    assert pl["n_items"] == pl["n_row_blocks"] * pl["n_sets"] * pl["k_parts"]
                    assert pl["grid"] == min(pl["n_items"], n_cu)
                    assert (pl["mode"] == 0) == (K <= 1536)
                    n_chunks = (K + 383) // 384
                    assert 1 <= pl["k_parts"] <= n_chunks and (pl["k_parts"] == 1 or pl["mode"] == 1)
                    if pl["k_parts"] > 1:                      # split K: only to fill idle compute units
                        assert pl["n_items"] <= n_cu and pl["rows_per_block"] == 64
                    if pl["mode"] != 0:
                        T = tw.tw_info(blob)["T"]
                        assert pl["n_sets"] == (T + pl["tiles_per_set"] - 1) // pl["tiles_per_set"]
    assert tw.tw_gemm_plan(blob, 0) == {k: 0 for k in tw.tw_gemm_plan(blob, 0)}
    with pytest.raises(tw.TwError) as e:
        tw.tw_gemm_plan(blob, -1)
    assert e.value.status == -1                            # TW_ERR_ARG
    with pytest.raises(tw.TwError) as e:
        tw.tw_gemm_plan(blob, 5, n_cu=0)
    assert e.value.status == -1
    bad = blob.copy()
    bad[:4] = 0
    with pytest.raises(tw.TwError) as e:
        tw.tw_gemm_plan(bad, 5)
    assert e.value.status == -3                            # TW_ERR_BUF: not a blob
