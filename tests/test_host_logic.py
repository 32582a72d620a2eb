"""CPU-only tests of the library's host logic: the shared object loads, exports what the header
declares, and its host mirrors agree with the paper's formulas and the oracle's sync model."""
import ctypes
import os
import re

import pytest

import paper_2305_13450_amd as ds
from oracle import sync_model as sm

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "depsync.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b([a-z_0-9]+)\s*\([^;{]*\)\s*;", text)))


def test_library_loads_and_exports_every_declared_symbol():
    lib = ctypes.CDLL(ds.LIB_PATH)
    names = _declared_functions()
    assert {"sync_policy_create", "dep_gemm_chain", "dep_conv_chain", "dep_chain_reset"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    assert set(ds.EXPORTS) == set(names)


def test_strerror_and_tile_shapes():
    assert ds._lib().depsync_strerror(0) == b"ok"
    assert b"invalid" in ds._lib().depsync_strerror(ds.EINVAL)
    assert ds.tile_shape(ds.TILE_256x256) == (256, 256)
    assert ds.tile_shape(ds.TILE_64x128) == (64, 128)
    assert ds.tile_shape(ds.TILE_128x192_DEEP) == (128, 192) and ds.tile_shape(ds.TILE_128x128_DEEP) == (128, 128)
    with pytest.raises(ds.DepsyncError):
        ds.tile_shape(0)
    with pytest.raises(ds.DepsyncError):
        ds.tile_shape(ds.TILE_128x128_DEEP + 1)      # one past the last shape
    # 65536 semaphores and 32768 arrival counters with a 128-byte line each, plus the rest
    assert (65536 + 32768) * 128 < ds.workspace_bytes() < 32 << 20


def test_policy_mirrors_match_oracle_model():
    for grid in ((3, 2), (24, 8), (5, 7)):
        for y in range(grid[1]):
            for x in range(grid[0]):
                assert ds.row_major(x, y, *grid) == sm.row_major((x, y), grid)
                assert ds.policy_sem(ds.TILESYNC, x, y, *grid) == sm.tilesync_sem((x, y), grid)
                assert ds.policy_sem(ds.ROWSYNC, x, y, *grid) == sm.rowsync_sem((x, y), grid)
        assert ds.policy_value(ds.TILESYNC, *grid) == 1
        assert ds.policy_value(ds.ROWSYNC, *grid) == grid[0]
    grid, s = (12, 5), 4
    for y in range(grid[1]):
        for x in range(grid[0]):
            assert ds.policy_sem(ds.STRIDEDSYNC, x, y, *grid, s) == sm.stridedsync_sem((x, y), grid, s)
    assert ds.policy_value(ds.STRIDEDSYNC, *grid, s) == 3


def test_wave_model_table1(golden):
    for batch, gemm, gx, gy, gz, occ, n_sm, w, util in golden("table1_waves.txt"):
        tbs = int(gx) * int(gy) * int(gz)
        waves, u = ds.wave_model(tbs, int(occ), int(n_sm))
        assert waves == -(-tbs // (int(occ) * int(n_sm)))
        assert 100 * u == pytest.approx(float(util))


def test_fig1_example_counts_and_schedule(golden):
    g = {k: int(v) for k, v in golden("fig1_example.txt")}
    grid = (g["col_tiles"], g["row_tiles"])
    assert ds.sync_count(ds.TILESYNC, grid, grid) == g["syncs_tilesync"]
    assert ds.sync_count(ds.ROWSYNC, grid, grid) == g["syncs_rowsync"]
    assert ds.simulate_chain(g["n_sm"], grid, 1.0, grid, 1.0, stream_sync=True) == g["total_waves_stream_sync"]
    assert ds.simulate_chain(g["n_sm"], grid, 1.0, grid, 1.0, stream_sync=False) == g["total_waves_fine_grained"]


def test_schedule_model_matches_oracle_simulator():
    for slots, pg, cg, d1, d2 in ((256, (24, 8), (48, 8), 2.0, 1.0), (7, (3, 5), (4, 5), 1.0, 1.5), (4, (2, 3), (2, 3), 1.0, 1.0)):
        tiles = sm.gemm_chain_tiles(pg, cg, d1, d2)
        for ss in (True, False):
            assert ds.simulate_chain(slots, pg, d1, cg, d2, stream_sync=ss) == pytest.approx(sm.simulate(slots, tiles, ss))


def _fake_gemm_desc(M, K1, N1, N2, mid=ds.MID_GELU, tile=0):
    d = ds.GemmChainDesc()
    d.M, d.K1, d.N1, d.N2, d.dtype, d.mid = M, K1, N1, N2, ds.BF16, mid
    d.X = d.W1t = d.H = d.W2t = d.Y = 0x1000          # never dereferenced by the planner
    d.ldx, d.ldw1, d.ldh, d.ldw2, d.ldy = K1, K1, N1, N1, N2
    d.tile_prod = d.tile_cons = tile
    return d


def test_planner_grids_flops_and_validation():
    d = _fake_gemm_desc(2048, 12288, 6144, 12288, tile=ds.TILE_256x256)
    info = ds.PlanInfo()
    assert ds._lib().depsync_gemm_chain_plan(ctypes.byref(d), None, 256, ctypes.byref(info)) == ds.OK
    assert (info.prod_grid_x, info.prod_grid_y, info.cons_grid_x, info.cons_grid_y) == (24, 8, 48, 8)
    assert (info.n_prod, info.n_cons, info.slots) == (192, 384, 256)
    assert (info.waves_streamsync, info.waves_fine) == (1 + 2, 3)
    assert info.flops == pytest.approx(2 * 2048 * 12288 * 6144 * 2)
    assert info.bytes == pytest.approx(2 * (2048 * 12288 + 2 * 12288 * 6144 + 2 * 2048 * 6144 + 2048 * 12288))
    # gate/up fusion halves the producer's output tile width
    d = _fake_gemm_desc(256, 8192, 2752, 8192, mid=ds.MID_SWIGLU, tile=ds.TILE_128x128)
    assert ds._lib().depsync_gemm_chain_plan(ctypes.byref(d), None, 256, ctypes.byref(info)) == ds.OK
    assert (info.prod_grid_x, info.cons_grid_x) == (43, 64)
    # rejections
    bad = _fake_gemm_desc(256, 1000, 4096, 1024)
    assert ds._lib().depsync_gemm_chain_plan(ctypes.byref(bad), None, 256, ctypes.byref(info)) == ds.EINVAL
    bad = _fake_gemm_desc(256, 1024, 4096, 1024); bad.X = 0x1004
    assert ds._lib().depsync_gemm_chain_plan(ctypes.byref(bad), None, 256, ctypes.byref(info)) == ds.EINVAL
    bad = _fake_gemm_desc(256, 1024, 4096, 1024); bad.ldh = 4100
    assert ds._lib().depsync_gemm_chain_plan(ctypes.byref(bad), None, 256, ctypes.byref(info)) == ds.EINVAL
    bad = _fake_gemm_desc(0, 1024, 4096, 1024)
    assert ds._lib().depsync_gemm_chain_plan(ctypes.byref(bad), None, 256, ctypes.byref(info)) == ds.EINVAL
    assert ds._lib().depsync_gemm_chain_plan(None, None, 256, ctypes.byref(info)) == ds.EINVAL


def test_planner_auto_tile_prefers_more_tiles_for_small_m():
    info = ds.PlanInfo()
    d = _fake_gemm_desc(2048, 12288, 6144, 12288)
    assert ds._lib().depsync_gemm_chain_plan(ctypes.byref(d), None, 256, ctypes.byref(info)) == ds.OK
    big = info.tile_prod
    d = _fake_gemm_desc(64, 12288, 6144, 12288)
    assert ds._lib().depsync_gemm_chain_plan(ctypes.byref(d), None, 256, ctypes.byref(info)) == ds.OK
    r_big, c_big = ds.tile_shape(big)
    r_small, c_small = ds.tile_shape(info.tile_prod)
    assert r_small * c_small <= r_big * c_big and r_small <= 128


@pytest.mark.parametrize("K1,N1,N2,mid,M,tile", [
    (12288, 6144, 12288, ds.MID_GELU, 64, ds.TILE_64x192),
    (12288, 6144, 12288, ds.MID_GELU, 256, ds.TILE_128x192_DEEP),
    (12288, 6144, 12288, ds.MID_GELU, 512, ds.TILE_128x192_DEEP),
    (12288, 6144, 12288, ds.MID_GELU, 1024, ds.TILE_256x192),
    (12288, 6144, 12288, ds.MID_GELU, 2048, ds.TILE_256x192),
    (8192, 2752, 8192, ds.MID_SWIGLU, 1, ds.TILE_64x128),
    (8192, 2752, 8192, ds.MID_SWIGLU, 256, ds.TILE_128x128_DEEP),
    (8192, 2752, 8192, ds.MID_SWIGLU, 1024, ds.TILE_256x128),
    (8192, 2752, 8192, ds.MID_SWIGLU, 2048, ds.TILE_256x128),
])
def test_planner_auto_tile_matches_the_measured_choice(K1, N1, N2, mid, M, tile):
    # the schedule model (split along K included) on a 256-CU chip picks the macro-tile that was
    # measured fastest on these MLP chains; asked twice, it answers the same (the choice is remembered)
    d = _fake_gemm_desc(M, K1, N1, N2, mid=mid)
    info = ds.PlanInfo()
    for _ in range(2):
        assert ds._lib().depsync_gemm_chain_plan(ctypes.byref(d), None, 256, ctypes.byref(info)) == ds.OK
        assert info.tile_prod == tile and info.tile_cons == tile


def test_conv_planner():
    d = ds.ConvChainDesc()
    d.B, d.H, d.W, d.C, d.K1, d.K2, d.dtype = 4, 56, 56, 256, 256, 256, ds.BF16
    d.inp = d.w1 = d.mid = d.w2 = d.out = 0x1000
    d.tile_prod = d.tile_cons = ds.TILE_128x128
    info = ds.PlanInfo()
    assert ds._lib().depsync_conv_chain_plan(ctypes.byref(d), None, 256, ctypes.byref(info)) == ds.OK
    assert (info.prod_grid_x, info.prod_grid_y) == (2, 98)
    assert info.flops == pytest.approx(2 * 2.0 * 4 * 56 * 56 * 256 * 9 * 256)
    d.C = 96
    assert ds._lib().depsync_conv_chain_plan(ctypes.byref(d), None, 256, ctypes.byref(info)) == ds.EINVAL


def test_planner_splits_small_stages_along_k_on_segment_boundaries():
    info = ds.PlanInfo()
    # 32 producer tiles on 512 slots, 192 K steps: eight parts of 24 steps; the consumer (64 tiles,
    # 96 steps, RowSync) takes six parts of 16 steps (eight would be shorter than 16 steps)
    d = _fake_gemm_desc(64, 12288, 6144, 12288, tile=ds.TILE_128x192)
    assert ds._lib().depsync_gemm_chain_plan(ctypes.byref(d), None, 256, ctypes.byref(info)) == ds.OK
    assert (info.prod_grid_x * info.prod_grid_y, info.n_prod) == (32, 32 * 8)
    assert (info.cons_grid_x * info.cons_grid_y, info.n_cons) == (64, 64 * 6)
    # a full-size stage is left alone
    d = _fake_gemm_desc(2048, 12288, 6144, 12288, tile=ds.TILE_128x192)
    assert ds._lib().depsync_gemm_chain_plan(ctypes.byref(d), None, 256, ctypes.byref(info)) == ds.OK
    assert (info.n_prod, info.n_cons) == (512, 1024)
    # conv, waits per filter row: parts must be whole filter rows (3 x 512 / 64 = 24 of the 72 steps)
    c = ds.ConvChainDesc()
    c.B, c.H, c.W, c.C, c.K1, c.K2, c.dtype = 1, 14, 14, 512, 512, 512, ds.BF16
    c.inp = c.w1 = c.mid = c.w2 = c.out = 0x1000
    c.tile_prod = c.tile_cons = ds.TILE_64x64
    assert ds._lib().depsync_conv_chain_plan(ctypes.byref(c), None, 256, ctypes.byref(info)) == ds.OK
    assert info.prod_grid_x * info.prod_grid_y == 32
    assert info.n_prod == 32 * 4 and info.n_cons == 32 * 3      # first conv: four parts of 18 steps; second: filter rows


def _fake_conv_n_desc(B, H, W, C, Ks, tile=0):
    d = ds.ConvChainNDesc()
    d.B, d.H, d.W, d.C, d.n, d.dtype = B, H, W, C, len(Ks), ds.BF16
    d.inp = 0x1000
    for i, k in enumerate(Ks):
        d.K[i], d.w[i], d.out[i] = k, 0x1000, 0x1000
    d.tile_prod = d.tile_cons = tile
    return d


ALL_TILES = list(range(1, ds.TILE_128x128_DEEP + 1))


@pytest.mark.parametrize("kind", [ds.ROWSYNC, ds.TILESYNC, ds.STRIDEDSYNC])
def test_every_slice_a_consumer_tile_loads_is_covered_by_a_wait(kind):
    # Section III-C: a consumer tile may read a producer tile's output only after waiting for it.
    # The library's own walk of every consumer K loop (same index functions as the kernel) finds
    # no K step whose slice of the intermediate lacks a wait at or before it, for every tile shape
    # it accepts, ragged M, split along K, the gated MLP (producer tiles half as wide) and attention.
    checked = 0
    for tile in ALL_TILES:
        for (M, K1, N1, N2, mid, extra) in (
                (300, 256, 768, 384, ds.MID_GELU, {}), (64, 12288, 6144, 12288, ds.MID_GELU, {}),
                (2048, 1024, 6144, 1536, ds.MID_GELU, {}), (200, 512, 1408, 512, ds.MID_SWIGLU, {}),
                (1, 8192, 2752, 8192, ds.MID_SWIGLU, {}),
                (512, 256, 3 * 256, 256, ds.MID_CAUSAL_ATTN, dict(batch=2, seq=256, heads=2, head_dim=128))):
            for ksplit in (0, 1, 2):
                d = _fake_gemm_desc(M, K1, N1, N2, mid=mid, tile=tile)
                if mid == ds.MID_CAUSAL_ATTN:
                    d.T, d.ldt, d.ldw2 = 0x1000, extra["heads"] * 128, extra["heads"] * 128
                    d.batch, d.seq, d.heads, d.head_dim = extra["batch"], extra["seq"], extra["heads"], 128
                try:
                    n = ds.gemm_chain_check_waits(d, kind, n_cu=256, ksplit=ksplit)
                except ds.DepsyncError as e:
                    assert e.status in (ds.EINVAL, ds.ENOTIMPL)      # shape the tile or policy cannot run
                    continue
                assert n == 0, (tile, M, K1, N1, N2, mid, ksplit)
                checked += 1
    assert checked > 100


def test_producer_and_consumer_may_use_different_tile_shapes():
    # Section III-C: the consumer maps its rows and K steps onto the PRODUCER's tiles, so the two
    # stages need not share a macro-tile shape.  Grids, slots and waves follow each stage's own shape.
    d = _fake_gemm_desc(2048, 12288, 6144, 12288)
    d.tile_prod, d.tile_cons = ds.TILE_256x192, ds.TILE_128x128
    info = ds.PlanInfo()
    assert ds._lib().depsync_gemm_chain_plan(ctypes.byref(d), None, 256, ctypes.byref(info)) == ds.OK
    assert (info.tile_prod, info.tile_cons) == (ds.TILE_256x192, ds.TILE_128x128)
    assert (info.prod_grid_x, info.prod_grid_y) == (32, 8)
    assert (info.cons_grid_x, info.cons_grid_y) == (96, 16)
    assert info.waves_streamsync == 1 + 3          # 256 tiles on 256 slots, 1536 tiles on 512 slots
    # every slice a consumer tile loads is covered by a wait, for every pair of shapes and policy
    checked = 0
    for tp in ALL_TILES:
        for tc in ALL_TILES:
            if tp == tc:
                continue
            for (M, K1, N1, N2, mid) in ((300, 192, 576, 328, ds.MID_GELU), (2048, 1024, 1536, 768, ds.MID_NONE),
                                         (150, 256, 192, 200, ds.MID_SWIGLU)):
                for kind in (ds.ROWSYNC, ds.TILESYNC, ds.STRIDEDSYNC):
                    d = _fake_gemm_desc(M, K1, N1, N2, mid=mid)
                    d.tile_prod, d.tile_cons = tp, tc
                    try:
                        n = ds.gemm_chain_check_waits(d, kind, n_cu=256)
                    except ds.DepsyncError as e:
                        assert e.status in (ds.EINVAL, ds.ENOTIMPL)
                        continue
                    assert n == 0, (tp, tc, M, K1, N1, N2, mid, kind)
                    checked += 1
    assert checked > 300
    # the attention chain's three stages share one shape
    d = _fake_gemm_desc(256, 512, 3 * 256, 512, mid=ds.MID_CAUSAL_ATTN)
    d.T, d.ldt, d.ldw2 = 0x1000, 256, 256
    d.batch, d.seq, d.heads, d.head_dim = 1, 256, 2, 128
    d.tile_prod, d.tile_cons = ds.TILE_128x128, ds.TILE_64x64
    assert ds._lib().depsync_gemm_chain_plan(ctypes.byref(d), None, 256, ctypes.byref(info)) == ds.ENOTIMPL
    # convolutions: pairs may differ, longer chains may not
    c = _fake_conv_n_desc(2, 28, 28, 128, (128, 64), tile=0)
    c.tile_prod, c.tile_cons = ds.TILE_128x128, ds.TILE_64x64
    for kind in (ds.ROWSYNC, ds.TILESYNC, ds.STRIDEDSYNC):
        assert ds.conv_chain_n_check_waits(c, kind, n_cu=256) == 0
    c = _fake_conv_n_desc(1, 56, 56, 64, (64, 64, 64), tile=0)
    c.tile_prod, c.tile_cons = ds.TILE_128x128, ds.TILE_64x64
    assert ds._lib().depsync_conv_chain_n_plan(ctypes.byref(c), None, 256, ctypes.byref(info)) == ds.ENOTIMPL


def test_gated_mlp_rejects_tiles_whose_producer_half_is_narrower_than_a_k_step():
    # 256x64 would leave 32-column producer tiles: a 64-wide K step of the consumer would then
    # read two producer tiles but wait for one (Section III-C's TileSync semantics broken)
    d = _fake_gemm_desc(256, 8192, 2752, 8192, mid=ds.MID_SWIGLU, tile=ds.TILE_256x64)
    info = ds.PlanInfo()
    assert ds._lib().depsync_gemm_chain_plan(ctypes.byref(d), None, 256, ctypes.byref(info)) == ds.EINVAL
    with pytest.raises(ds.DepsyncError):
        ds.gemm_chain_check_waits(d, ds.TILESYNC, n_cu=256)


@pytest.mark.parametrize("kind", [ds.ROWSYNC, ds.TILESYNC, ds.STRIDEDSYNC])
def test_conv_chain_waits_cover_the_halo(kind):
    # 3x3 convolution: a consumer row tile reads pixels up to W+1 rows beyond its own rows
    checked = 0
    for tile in ALL_TILES:
        for (B, H, W, C, Ks) in ((1, 14, 14, 512, (512, 512)), (2, 28, 28, 128, (128, 64)), (1, 56, 56, 64, (64, 64, 64)),
                                 (3, 9, 17, 64, (128, 64, 64, 8)), (16, 14, 14, 64, (64, 64))):
            for ksplit in (0, 1, 3):
                d = _fake_conv_n_desc(B, H, W, C, Ks, tile=tile)
                try:
                    n = ds.conv_chain_n_check_waits(d, kind, n_cu=256, ksplit=ksplit)
                except ds.DepsyncError as e:
                    assert e.status in (ds.EINVAL, ds.ENOTIMPL)
                    continue
                assert n == 0, (tile, B, H, W, C, Ks, ksplit)
                checked += 1
    assert checked > 100


def test_k_blocked_layout_is_validated():
    info = ds.PlanInfo()
    d = _fake_gemm_desc(256, 1024, 4096, 1024)
    d.w_layout = ds.W_KBLOCKED
    d.ldw1 = d.ldw2 = 0                                        # ignored for packed weights
    assert ds._lib().depsync_gemm_chain_plan(ctypes.byref(d), None, 256, ctypes.byref(info)) == ds.OK
    d.w_layout = 7
    assert ds._lib().depsync_gemm_chain_plan(ctypes.byref(d), None, 256, ctypes.byref(info)) == ds.EINVAL


def test_bench_refuses_more_than_one_gpu():
    # the build is single-GPU: bench.py says so and exits before it touches a device
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""
