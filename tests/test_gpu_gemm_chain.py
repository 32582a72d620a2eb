"""GPU parity tests of dep_gemm_chain against the fp64 oracle, element by element, plus the
bit-exactness of fine-grained synchronisation against the same kernels under stream sync."""
import numpy as np
import pytest
import torch

import inputs
import oracle
import paper_2305_13450_amd as ds
from gpu_util import TOL_BF16, TOL_FP16, TOL_MID, mid_err, rel_err, run_gemm_chain

pytestmark = pytest.mark.gpu

ALL_TILES = [ds.TILE_256x256, ds.TILE_256x128, ds.TILE_128x256, ds.TILE_128x128, ds.TILE_64x128, ds.TILE_64x64,
             ds.TILE_256x192, ds.TILE_128x192, ds.TILE_256x64, ds.TILE_64x64_DEEP, ds.TILE_64x192,
             ds.TILE_128x192_DEEP, ds.TILE_128x128_DEEP]
MODES = [ds.MODE_FINE, ds.MODE_STREAMSYNC, ds.MODE_PLAIN, ds.MODE_FUSED]


@pytest.fixture(scope="module")
def cfg1():
    t = inputs.mlp(**inputs.CFG1)
    H, Y = oracle.gemm_chain(inputs.to_f64(t["X"]), inputs.to_f64(t["W1"]), inputs.to_f64(t["W2"]), oracle.ACT_GELU)
    return t, H, Y


def test_cfg1_rowsync_matches_oracle_and_is_bit_exact(cfg1):
    t, Href, Yref = cfg1
    pol = ds.SyncPolicy(ds.ROWSYNC)
    outs = {}
    for mode in MODES:
        print(f"cfg1 mode={mode}", flush=True)
        H, Y = run_gemm_chain(t["X"], t["W1"], t["W2"], pol, mode)
        assert mid_err(H, Href) <= TOL_MID
        assert rel_err(Y, Yref) <= TOL_BF16
        outs[mode] = (H, Y)
    for mode in (ds.MODE_STREAMSYNC, ds.MODE_PLAIN, ds.MODE_FUSED):
        assert torch.equal(outs[ds.MODE_FINE][0], outs[mode][0])
        assert torch.equal(outs[ds.MODE_FINE][1], outs[mode][1])
    pol.destroy()


@pytest.mark.parametrize("tile", ALL_TILES)
@pytest.mark.parametrize("kind", [ds.ROWSYNC, ds.TILESYNC])
def test_every_tile_shape_ragged(tile, kind):
    # several tiles in both directions and ragged tails in M and N for every macro-tile shape
    M, K1, N1, N2 = 300, 192, 576, 328
    print(f"ragged tile={tile} kind={kind}", flush=True)
    t = inputs.mlp(M, K1, N1, N2, seed=3)
    Href, Yref = oracle.gemm_chain(inputs.to_f64(t["X"]), inputs.to_f64(t["W1"]), inputs.to_f64(t["W2"]), oracle.ACT_GELU)
    pol = ds.SyncPolicy(kind)
    res = [run_gemm_chain(t["X"], t["W1"], t["W2"], pol, mode, tile=tile) for mode in MODES]
    for H, Y in res:
        assert mid_err(H, Href) <= TOL_MID
        assert rel_err(Y, Yref) <= TOL_BF16
    for H, Y in res[1:]:
        assert torch.equal(res[0][0], H) and torch.equal(res[0][1], Y)
    pol.destroy()
    # one dispatch names its tiles by the block index unless told otherwise: the dispatch queues
    # (persistent workgroups) must give the same bits
    pol = ds.SyncPolicy(kind, flags=ds.FLAG_QUEUE_ORDER)
    H, Y = run_gemm_chain(t["X"], t["W1"], t["W2"], pol, ds.MODE_FUSED, tile=tile)
    assert torch.equal(res[0][0], H) and torch.equal(res[0][1], Y)
    assert pol.status().timed_out == 0
    pol.destroy()


@pytest.mark.parametrize("mid,act", [(ds.MID_NONE, oracle.ACT_NONE), (ds.MID_RELU, oracle.ACT_RELU)])
def test_other_pointwise_ops(mid, act):
    t = inputs.mlp(130, 128, 256, 136, seed=5)
    Href, Yref = oracle.gemm_chain(inputs.to_f64(t["X"]), inputs.to_f64(t["W1"]), inputs.to_f64(t["W2"]), act)
    pol = ds.SyncPolicy(ds.TILESYNC)
    H, Y = run_gemm_chain(t["X"], t["W1"], t["W2"], pol, ds.MODE_FINE, mid=mid, tile=ds.TILE_64x64)
    assert mid_err(H, Href) <= TOL_MID and rel_err(Y, Yref) <= TOL_BF16
    pol.destroy()


def test_fp16_chain():
    t = inputs.mlp(200, 256, 384, 264, seed=7, dtype=torch.float16)
    Href, Yref = oracle.gemm_chain(inputs.to_f64(t["X"]), inputs.to_f64(t["W1"]), inputs.to_f64(t["W2"]), oracle.ACT_GELU)
    pol = ds.SyncPolicy(ds.ROWSYNC)
    a = run_gemm_chain(t["X"], t["W1"], t["W2"], pol, ds.MODE_FINE, tile=ds.TILE_128x128)
    b = run_gemm_chain(t["X"], t["W1"], t["W2"], pol, ds.MODE_STREAMSYNC, tile=ds.TILE_128x128)
    assert mid_err(a[0], Href, 2.0 ** -11) <= TOL_MID and rel_err(a[1], Yref) <= TOL_FP16
    assert torch.equal(a[1], b[1])
    pol.destroy()


@pytest.mark.parametrize("M", [1, 7, 64])
def test_skinny_m(M):
    t = inputs.mlp(M, 512, 1024, 512, seed=11)
    Href, Yref = oracle.gemm_chain(inputs.to_f64(t["X"]), inputs.to_f64(t["W1"]), inputs.to_f64(t["W2"]), oracle.ACT_GELU)
    pol = ds.SyncPolicy(ds.TILESYNC)
    for mode in MODES:
        H, Y = run_gemm_chain(t["X"], t["W1"], t["W2"], pol, mode)
        assert mid_err(H, Href) <= TOL_MID and rel_err(Y, Yref) <= TOL_BF16
    pol.destroy()


def test_swiglu_chain_matches_oracle():
    # Nh = 192 is not a multiple of the 128 gate/up columns a 256-wide tile owns: ragged tail
    M, K1, Nh, N2 = 150, 256, 192, 200
    t = inputs.swiglu(M, K1, Nh, N2, seed=13)
    Href, Yref = oracle.swiglu_chain(inputs.to_f64(t["X"]), inputs.to_f64(t["Wgu"]), inputs.to_f64(t["W2"]))
    for tile in (ds.TILE_256x256, ds.TILE_256x128, ds.TILE_128x256, ds.TILE_128x128, ds.TILE_64x128):
        print(f"swiglu tile={tile}", flush=True)
        pol = ds.SyncPolicy(ds.TILESYNC)
        res = [run_gemm_chain(t["X"], t["Wgu"], t["W2"], pol, mode, mid=ds.MID_SWIGLU, tile=tile) for mode in MODES]
        for H, Y in res:
            # silu(g)*u is heavy-tailed and K2 is small here, so the largest outputs sit more than five
            # RMS out, where one bf16 rounding alone exceeds 2e-2 of the RMS: bound the error beyond
            # the output's own rounding instead (stricter everywhere but in that extreme tail)
            assert mid_err(H, Href) <= TOL_MID and mid_err(Y, Yref) <= 1e-2
        assert all(torch.equal(res[0][1], r[1]) for r in res[1:])
        pol.destroy()


def test_stridedsync_on_gemm_chain():
    # 6 producer column tiles of 64; tiles x, x+2, x+4 share a semaphore (stride 2, count 3)
    t = inputs.mlp(192, 128, 384, 128, seed=17)
    Href, Yref = oracle.gemm_chain(inputs.to_f64(t["X"]), inputs.to_f64(t["W1"]), inputs.to_f64(t["W2"]), oracle.ACT_GELU)
    pol = ds.SyncPolicy(ds.STRIDEDSYNC, count=3, flags=ds.FLAG_COUNT, ksplit=1)   # counts per whole tile
    H, Y = run_gemm_chain(t["X"], t["W1"], t["W2"], pol, ds.MODE_FINE, tile=ds.TILE_64x64)
    assert rel_err(Y, Yref) <= TOL_BF16
    st = pol.status()
    assert st.posts == 6 * 3                   # every producer tile posts once
    assert st.waits == (3 * 2) * 2             # 6 consumer tiles, 2 shared semaphores each
    pol.destroy()


def test_sync_counts_of_the_fig1_shaped_chain(golden):
    # 3 row tiles x 2 column tiles per GeMM, as in Fig. 1: 12 waits under TileSync, 6 under RowSync
    g = {k: int(v) for k, v in golden("fig1_example.txt")}
    t = inputs.mlp(3 * 128, 128, 2 * 128, 2 * 128, seed=19)
    _, Yref = oracle.gemm_chain(inputs.to_f64(t["X"]), inputs.to_f64(t["W1"]), inputs.to_f64(t["W2"]), oracle.ACT_GELU)
    for kind, key in ((ds.TILESYNC, "syncs_tilesync"), (ds.ROWSYNC, "syncs_rowsync")):
        pol = ds.SyncPolicy(kind, flags=ds.FLAG_COUNT, ksplit=1)   # the figure has no split along K
        _, Y = run_gemm_chain(t["X"], t["W1"], t["W2"], pol, ds.MODE_FINE, tile=ds.TILE_128x128)
        st = pol.status()
        assert rel_err(Y, Yref) <= TOL_BF16
        assert st.posts == 6 and st.waits == g[key]
        pol.destroy()


def test_repeated_launches_reuse_the_workspace_without_reset():
    t = inputs.mlp(520, 256, 512, 384, seed=23)
    _, Yref = oracle.gemm_chain(inputs.to_f64(t["X"]), inputs.to_f64(t["W1"]), inputs.to_f64(t["W2"]), oracle.ACT_GELU)
    pol = ds.SyncPolicy(ds.TILESYNC)
    first = None
    for it in range(30):
        _, Y = run_gemm_chain(t["X"], t["W1"], t["W2"], pol, ds.MODE_FINE, tile=ds.TILE_64x128)
        if first is None:
            first = Y.clone()
            assert rel_err(Y, Yref) <= TOL_BF16
        assert torch.equal(Y, first), it
    # a different geometry on the same policy re-zeroes the workspace by itself
    _, Y = run_gemm_chain(t["X"], t["W1"], t["W2"], pol, ds.MODE_FINE, tile=ds.TILE_128x128)
    assert rel_err(Y, Yref) <= TOL_BF16
    pol.destroy()


def test_changing_inputs_on_reused_buffers_never_reads_stale_intermediate():
    # The same H and Y buffers are reused by back-to-back chains whose inputs alternate, so a consumer
    # that hit a cache line of H left over from the previous chain would produce the other answer.
    ta = inputs.mlp(1024, 512, 1024, 768, seed=41)
    tb = inputs.mlp(1024, 512, 1024, 768, seed=42)
    W1t = ta["W1"].t().contiguous().cuda(); W2t = ta["W2"].t().contiguous().cuda()
    Xs = [ta["X"].cuda(), tb["X"].cuda()]
    H = torch.empty((1024, 1024), dtype=torch.bfloat16, device="cuda"); Y = torch.empty((1024, 768), dtype=torch.bfloat16, device="cuda")
    pol = ds.SyncPolicy(ds.TILESYNC)
    want = []
    for X in Xs:
        ds.dep_gemm_chain(X, W1t, H, W2t, Y, pol, mode=ds.MODE_STREAMSYNC, tile=ds.TILE_128x128)
        torch.cuda.synchronize()
        want.append(Y.clone())
    assert not torch.equal(want[0], want[1])
    for kind in (ds.TILESYNC, ds.ROWSYNC):
        p2 = ds.SyncPolicy(kind)
        outs = []
        for it in range(24):                      # enqueue back to back, no host sync in between
            Yi = torch.empty_like(Y)
            ds.dep_gemm_chain(Xs[it & 1], W1t, H, W2t, Yi, p2, mode=ds.MODE_FUSED if it % 3 == 2 else ds.MODE_FINE,
                              tile=ds.TILE_128x128)
            outs.append(Yi)
        torch.cuda.synchronize()
        for it, Yi in enumerate(outs):
            assert torch.equal(Yi, want[it & 1]), (kind, it)
        p2.destroy()
    pol.destroy()


def test_delayed_and_reversed_producers_do_not_change_the_result():
    t = inputs.mlp(512, 256, 512, 256, seed=29)
    _, Yref = oracle.gemm_chain(inputs.to_f64(t["X"]), inputs.to_f64(t["W1"]), inputs.to_f64(t["W2"]), oracle.ACT_GELU)
    base = ds.SyncPolicy(ds.TILESYNC)
    _, Y0 = run_gemm_chain(t["X"], t["W1"], t["W2"], base, ds.MODE_STREAMSYNC, tile=ds.TILE_64x64)
    assert rel_err(Y0, Yref) <= TOL_BF16
    base.destroy()
    for kind in (ds.TILESYNC, ds.ROWSYNC):
        for kw in (dict(delay_tile=1, delay_iters=300), dict(delay_tile=37, delay_iters=300),
                   dict(flags=ds.FLAG_REVERSE_ORDER), dict(flags=ds.FLAG_NO_REORDER)):
            for mode in (ds.MODE_FINE, ds.MODE_FUSED):
                pol = ds.SyncPolicy(kind, **kw)
                _, Y = run_gemm_chain(t["X"], t["W1"], t["W2"], pol, mode, tile=ds.TILE_64x64)
                assert torch.equal(Y, Y0), (kind, kw, mode)
                pol.destroy()
        pol = ds.SyncPolicy(kind, flags=ds.FLAG_HW_ORDER, delay_tile=5, delay_iters=300)
        _, Y = run_gemm_chain(t["X"], t["W1"], t["W2"], pol, ds.MODE_FUSED, tile=ds.TILE_64x64)
        assert torch.equal(Y, Y0), (kind, "fused, hardware order")
        pol.destroy()


def test_bounded_wait_reports_timeout_and_reset_recovers():
    # The first producer tile's post is held back for a few milliseconds while consumers give up
    # after 8 polls: every kernel still exits, and the status reports the expired wait.
    t = inputs.mlp(128, 128, 128, 128, seed=31)
    _, Yref = oracle.gemm_chain(inputs.to_f64(t["X"]), inputs.to_f64(t["W1"]), inputs.to_f64(t["W2"]), oracle.ACT_GELU)
    pol = ds.SyncPolicy(ds.TILESYNC, spin_limit=8, delay_tile=1, delay_iters=2000)
    run_gemm_chain(t["X"], t["W1"], t["W2"], pol, ds.MODE_FINE, tile=ds.TILE_64x64)
    st = pol.status(raise_on_timeout=False)
    assert st.timed_out > 0 and st.first_timeout >= 4        # tickets 0..3 are producer tiles
    with pytest.raises(ds.DepsyncError):
        pol.status()
    pol.reset()
    pol2 = ds.SyncPolicy(ds.TILESYNC)
    _, Y = run_gemm_chain(t["X"], t["W1"], t["W2"], pol2, ds.MODE_FINE, tile=ds.TILE_64x64)
    assert rel_err(Y, Yref) <= TOL_BF16
    assert pol.status().timed_out == 0
    pol.destroy(); pol2.destroy()


def test_invalid_arguments_are_rejected_before_any_launch():
    t = inputs.mlp(64, 128, 128, 128, seed=1)
    X = t["X"].cuda(); W1t = t["W1"].t().contiguous().cuda(); W2t = t["W2"].t().contiguous().cuda()
    H = torch.empty((64, 128), dtype=torch.bfloat16, device="cuda"); Y = torch.empty_like(H)
    pol = ds.SyncPolicy(ds.ROWSYNC)
    with pytest.raises(ds.DepsyncError) as e:
        ds.dep_gemm_chain(X, W1t, H, W2t, Y, pol, mode=7)
    assert e.value.status == ds.EINVAL
    with pytest.raises(ds.DepsyncError) as e:     # misaligned base pointer
        ds.dep_gemm_chain(X.view(-1)[1:1 + 63 * 128].view(63, 128), W1t, H[:63], W2t, Y[:63], pol)
    assert e.value.status == ds.EINVAL
    pol.destroy()


def test_autotune_picks_a_tile_the_library_then_uses():
    M, K1, N1, N2 = 320, 256, 768, 384      # a shape no other test uses (the choice is kept per shape)
    t = inputs.mlp(M, K1, N1, N2, seed=23)
    Href, Yref = oracle.gemm_chain(inputs.to_f64(t["X"]), inputs.to_f64(t["W1"]), inputs.to_f64(t["W2"]), oracle.ACT_GELU)
    X, W1t, W2t = t["X"].cuda(), t["W1"].t().contiguous().cuda(), t["W2"].t().contiguous().cuda()
    H = torch.empty((M, N1), dtype=X.dtype, device="cuda")
    Y = torch.empty((M, N2), dtype=X.dtype, device="cuda")
    pol = ds.SyncPolicy(ds.TILESYNC)
    tile = ds.gemm_chain_autotune(X, W1t, H, W2t, Y, pol, reps=2)
    assert 1 <= tile <= ds.TILE_128x128_DEEP
    assert ds.gemm_chain_plan(X, W1t, H, W2t, Y, pol).tile_prod == tile
    res = [run_gemm_chain(t["X"], t["W1"], t["W2"], pol, mode) for mode in MODES]
    for Hm, Ym in res:
        assert mid_err(Hm, Href) <= TOL_MID and rel_err(Ym, Yref) <= TOL_BF16
        assert torch.equal(Hm, res[0][0]) and torch.equal(Ym, res[0][1])
    pol.destroy()


def test_remembered_hardware_order_alternates_with_the_dispatch_queues():
    # On a chain whose tiles are all resident at once, one-dispatch launches name tiles by the block
    # index (also with a remembered TUNED_HW_ORDER) while two-stream and stream-sync launches of the
    # same policy draw from the queues: the queue counters then advance on some chains only.
    # Several chains of each kind on one policy, same bits every time.
    M, K1, N1, N2 = 512, 256, 2048, 1024
    t = inputs.mlp(M, K1, N1, N2, seed=61)
    Href, Yref = oracle.gemm_chain(inputs.to_f64(t["X"]), inputs.to_f64(t["W1"]), inputs.to_f64(t["W2"]), oracle.ACT_GELU)
    X, W1t, W2t = t["X"].cuda(), t["W1"].t().contiguous().cuda(), t["W2"].t().contiguous().cuda()
    H = torch.empty((M, N1), dtype=X.dtype, device="cuda")
    Y = torch.empty((M, N2), dtype=X.dtype, device="cuda")
    pol = ds.SyncPolicy(ds.ROWSYNC)
    assert ds.gemm_chain_tuned(X, W1t, H, W2t, Y, pol) == (0, 0)
    ds.gemm_chain_set_tuned(X, W1t, H, W2t, Y, pol, ds.TILE_64x64, ds.TUNED_HW_ORDER | ds.TUNED_NO_SPLIT)
    assert ds.gemm_chain_tuned(X, W1t, H, W2t, Y, pol) == (ds.TILE_64x64, ds.TUNED_HW_ORDER | ds.TUNED_NO_SPLIT)
    plan = ds.gemm_chain_plan(X, W1t, H, W2t, Y, pol)
    assert plan.tile_prod == ds.TILE_64x64 and plan.n_prod + plan.n_cons <= plan.slots
    order = [ds.MODE_FUSED, ds.MODE_FINE, ds.MODE_FUSED, ds.MODE_STREAMSYNC, ds.MODE_FUSED, ds.MODE_FUSED,
             ds.MODE_FINE, ds.MODE_FINE, ds.MODE_FUSED]
    first = None
    for i, mode in enumerate(order):
        print(f"chain {i} mode={mode}", flush=True)
        Hm, Ym = run_gemm_chain(t["X"], t["W1"], t["W2"], pol, mode)
        if first is None:
            first = (Hm, Ym)
            assert mid_err(Hm, Href) <= TOL_MID and rel_err(Ym, Yref) <= TOL_BF16
        assert torch.equal(Hm, first[0]) and torch.equal(Ym, first[1]), (i, mode)
    assert pol.status().timed_out == 0
    ds.gemm_chain_set_tuned(X, W1t, H, W2t, Y, pol, 0)
    assert ds.gemm_chain_tuned(X, W1t, H, W2t, Y, pol) == (0, 0)
    with pytest.raises(ds.DepsyncError):
        ds.gemm_chain_set_tuned(X, W1t, H, W2t, Y, pol, 99)
    pol.destroy()


def test_autosync_policy_resolves_to_the_measured_kind():
    # Section IV-A: the policy is part of the search.  An AUTOSYNC policy runs under the rule of
    # thumb (per-tile waits up to 256 rows) until depsync_gemm_chain_autotune_policy has measured
    # the chain under every kind; then it runs under the remembered kind.  Either way its results
    # are those of a policy created with that kind, bit for bit.
    M, K1, N1, N2 = 192, 512, 1152, 640       # a shape no other test uses (choices are kept per shape)
    t = inputs.mlp(M, K1, N1, N2, seed=71)
    Href, Yref = oracle.gemm_chain(inputs.to_f64(t["X"]), inputs.to_f64(t["W1"]), inputs.to_f64(t["W2"]), oracle.ACT_GELU)
    X, W1t, W2t = t["X"].cuda(), t["W1"].t().contiguous().cuda(), t["W2"].t().contiguous().cuda()
    H = torch.empty((M, N1), dtype=X.dtype, device="cuda")
    Y = torch.empty((M, N2), dtype=X.dtype, device="cuda")
    auto = ds.SyncPolicy(ds.AUTOSYNC, flags=ds.FLAG_COUNT)
    assert ds.gemm_chain_policy(X, W1t, H, W2t, Y, auto) == ds.TILESYNC
    big = torch.empty((512, K1), dtype=X.dtype, device="cuda")
    assert ds.gemm_chain_policy(big, W1t, torch.empty((512, N1), dtype=X.dtype, device="cuda"), W2t,
                                torch.empty((512, N2), dtype=X.dtype, device="cuda"), auto) == ds.ROWSYNC
    kind, tile, us = ds.gemm_chain_autotune_policy(X, W1t, H, W2t, Y, auto, reps=2)
    print(f"autotune_policy: kind {kind} tile {tile} us {us}", flush=True)
    assert kind in (ds.ROWSYNC, ds.TILESYNC, ds.STRIDEDSYNC) and us[kind] > 0 and us[kind] == min(u for u in us if u > 0)
    assert ds.gemm_chain_policy(X, W1t, H, W2t, Y, auto) == kind
    auto.destroy()
    auto = ds.SyncPolicy(ds.AUTOSYNC, flags=ds.FLAG_COUNT)     # a fresh one: the tuning runs counted on the other
    explicit = ds.SyncPolicy(kind, flags=ds.FLAG_COUNT)
    assert ds.gemm_chain_plan(X, W1t, H, W2t, Y, auto).as_dict() == ds.gemm_chain_plan(X, W1t, H, W2t, Y, explicit).as_dict()
    assert ds.gemm_chain_plan(X, W1t, H, W2t, Y, auto).tile_prod == tile
    for mode in MODES:
        Ha, Ya = run_gemm_chain(t["X"], t["W1"], t["W2"], auto, mode)
        He, Ye = run_gemm_chain(t["X"], t["W1"], t["W2"], explicit, mode)
        assert torch.equal(Ha, He) and torch.equal(Ya, Ye)
        assert mid_err(Ha, Href) <= TOL_MID and rel_err(Ya, Yref) <= TOL_BF16
    sa, se = auto.status(), explicit.status()
    assert (sa.posts, sa.waits) == (se.posts, se.waits) and sa.timed_out == 0      # the same semaphore traffic: the same policy
    auto.destroy()
    explicit.destroy()


def test_trace_records_cover_every_tile_in_order():
    # DEPSYNC_FLAG_TRACE: one record per tile with enter <= start <= ready <= end, producers
    # finishing before the consumers that wait for their whole row start computing
    M, K1, N1, N2 = 512, 256, 1024, 512
    t = inputs.mlp(M, K1, N1, N2, seed=31)
    X, W1t, W2t = t["X"].cuda(), t["W1"].t().contiguous().cuda(), t["W2"].t().contiguous().cuda()
    H = torch.empty((M, N1), dtype=X.dtype, device="cuda")
    Y = torch.empty((M, N2), dtype=X.dtype, device="cuda")
    pol = ds.SyncPolicy(ds.ROWSYNC, flags=ds.FLAG_TRACE, ksplit=1)
    plan = ds.gemm_chain_plan(X, W1t, H, W2t, Y, pol, tile=ds.TILE_128x128)
    for mode in (ds.MODE_FINE, ds.MODE_FUSED, ds.MODE_STREAMSYNC):
        ds.dep_gemm_chain(X, W1t, H, W2t, Y, pol, mode=mode, tile=ds.TILE_128x128)
        torch.cuda.synchronize()
        recs = pol.read_trace(plan.n_prod + plan.n_cons)
        assert [r.rel for r in recs] == list(range(plan.n_prod + plan.n_cons))
        for r in recs:
            assert r.t_enter <= r.t_start <= r.t_ready <= r.t_end
            assert (r.where >> 8) & 0xff < 8           # XCD id
        prod, cons = recs[:plan.n_prod], recs[plan.n_prod:]
        assert {(r.tx, r.ty) for r in prod} == {(x, y) for x in range(plan.prod_grid_x) for y in range(plan.prod_grid_y)}
        for c in cons:   # RowSync: a consumer tile is ready only after every producer tile of its row has ended
            assert c.t_ready >= max(p.t_end for p in prod if p.ty == c.ty) - 100   # ticks of 10 ns
    pol.destroy()


@pytest.mark.parametrize("ksplit", [2, 3, 4, 8])
@pytest.mark.parametrize("kind", [ds.ROWSYNC, ds.TILESYNC])
def test_split_k_matches_oracle_and_does_not_depend_on_timing(ksplit, kind):
    # every output tile computed by `ksplit` workgroups over parts of K, the last to arrive adding
    # the fp32 partial tiles in K order: ragged M and N, K a multiple of 64 * 24
    M, K1, N1, N2 = 200, 1536, 1536, 328
    t = inputs.mlp(M, K1, N1, N2, seed=37)
    Href, Yref = oracle.gemm_chain(inputs.to_f64(t["X"]), inputs.to_f64(t["W1"]), inputs.to_f64(t["W2"]), oracle.ACT_GELU)
    for tile in (ds.TILE_64x64, ds.TILE_128x128, ds.TILE_128x192, ds.TILE_128x192_DEEP):
        print(f"split-K ksplit={ksplit} kind={kind} tile={tile}", flush=True)
        pol = ds.SyncPolicy(kind, ksplit=ksplit)
        plan = ds.gemm_chain_plan(t["X"].cuda(), t["W1"].t().contiguous().cuda(), torch.empty((M, N1), dtype=torch.bfloat16, device="cuda"),
                                  t["W2"].t().contiguous().cuda(), torch.empty((M, N2), dtype=torch.bfloat16, device="cuda"), pol, tile=tile)
        tm, tn = ds.tile_shape(tile)
        assert plan.n_prod == -(-M // tm) * -(-N1 // tn) * ksplit          # K1 / 64 = 24 divides by 2, 3, 4, 8
        res = [run_gemm_chain(t["X"], t["W1"], t["W2"], pol, mode, tile=tile) for mode in MODES]
        for H, Y in res:
            assert mid_err(H, Href) <= TOL_MID and rel_err(Y, Yref) <= TOL_BF16
            assert torch.equal(H, res[0][0]) and torch.equal(Y, res[0][1])
        pol.destroy()
        # a delayed part must not change the sum
        pol = ds.SyncPolicy(kind, ksplit=ksplit, flags=ds.FLAG_REVERSE_ORDER)
        H, Y = run_gemm_chain(t["X"], t["W1"], t["W2"], pol, ds.MODE_FINE, tile=tile)
        assert torch.equal(H, res[0][0]) and torch.equal(Y, res[0][1])
        pol.destroy()


def test_split_k_is_chosen_for_skinny_chains_and_swiglu():
    # few tiles on a big chip: the library splits on its own; the gated activation is applied
    # after the partial sums are added
    t = inputs.swiglu(48, 2048, 192, 256, seed=41)
    Href, Yref = oracle.swiglu_chain(inputs.to_f64(t["X"]), inputs.to_f64(t["Wgu"]), inputs.to_f64(t["W2"]))
    pol = ds.SyncPolicy(ds.TILESYNC)
    res = [run_gemm_chain(t["X"], t["Wgu"], t["W2"], pol, mode, mid=ds.MID_SWIGLU, tile=ds.TILE_64x128) for mode in MODES]
    X = t["X"].cuda()
    plan = ds.gemm_chain_plan(X, t["Wgu"].t().contiguous().cuda(), res[0][0], t["W2"].t().contiguous().cuda(), res[0][1], pol,
                              mid=ds.MID_SWIGLU, tile=ds.TILE_64x128)
    assert plan.n_prod > plan.prod_grid_x * plan.prod_grid_y               # split
    for H, Y in res:
        assert mid_err(H, Href) <= TOL_MID and mid_err(Y, Yref) <= 1e-2
        assert torch.equal(H, res[0][0]) and torch.equal(Y, res[0][1])
    pol.destroy()


def test_one_policy_reused_with_and_without_split_k():
    # the dispatch queues' lengths change with the split: the workspace must notice (regression)
    M, K1, N1, N2 = 128, 2048, 512, 256
    t = inputs.mlp(M, K1, N1, N2, seed=47)
    X, W1t, W2t = t["X"].cuda(), t["W1"].t().contiguous().cuda(), t["W2"].t().contiguous().cuda()
    H = torch.empty((M, N1), dtype=X.dtype, device="cuda")
    Y = torch.empty((M, N2), dtype=X.dtype, device="cuda")
    pol = ds.SyncPolicy(ds.TILESYNC, spin_limit=1 << 14)
    tile = ds.gemm_chain_autotune(X, W1t, H, W2t, Y, pol, reps=1)      # alternates split / no split on one policy
    assert pol.status().timed_out == 0
    Yref = oracle.gemm_chain(inputs.to_f64(t["X"]), inputs.to_f64(t["W1"]), inputs.to_f64(t["W2"]), oracle.ACT_GELU)[1]
    ds.dep_gemm_chain(X, W1t, H, W2t, Y, pol, mode=ds.MODE_FUSED)
    torch.cuda.synchronize()
    assert rel_err(Y, Yref) <= TOL_BF16 and pol.status().timed_out == 0 and tile >= 1
    pol.destroy()


@pytest.mark.parametrize("mid", [ds.MID_GELU, ds.MID_SWIGLU])
def test_k_blocked_weight_layout_gives_the_same_bits(mid):
    # weights re-arranged to [K/64][N][64] (each pipeline step of a tile reads one contiguous run):
    # a pure change of addressing, so the results equal the row-major ones bit for bit
    M, K1, N1, N2 = 200, 512, 384, 328
    if mid == ds.MID_SWIGLU:
        t = inputs.swiglu(M, K1, N1, N2, seed=59); W1 = t["Wgu"]
    else:
        t = inputs.mlp(M, K1, N1, N2, seed=59); W1 = t["W1"]
    X, W1t, W2t = t["X"].cuda(), W1.t().contiguous().cuda(), t["W2"].t().contiguous().cuda()
    W1b, W2b = ds.pack_weights_kblocked(W1t), ds.pack_weights_kblocked(W2t)
    assert W1b.shape == (K1 // 64, W1t.shape[0], 64)
    for tile in (ds.TILE_64x128, ds.TILE_128x128, ds.TILE_256x128):
        outs = []
        for a, b in ((W1t, W2t), (W1b, W2b)):
            pol = ds.SyncPolicy(ds.TILESYNC)
            H = torch.full((M, N1), float("nan"), dtype=X.dtype, device="cuda")
            Y = torch.full((M, N2), float("nan"), dtype=X.dtype, device="cuda")
            for mode in MODES:
                ds.dep_gemm_chain(X, a, H, b, Y, pol, mode=mode, mid=mid, tile=tile)
                torch.cuda.synchronize()
                outs.append((H.clone(), Y.clone()))
            pol.destroy()
        for H, Y in outs[1:]:
            assert torch.equal(H, outs[0][0]) and torch.equal(Y, outs[0][1])
    with pytest.raises(ValueError):      # both operands must use one layout
        ds.dep_gemm_chain(X, W1b, H, W2t, Y, ds.SyncPolicy(ds.ROWSYNC), mid=mid)


def test_mfma_calibration_reports_a_plausible_rate():
    # register-only MFMA loop: faster on zero operands than on random ones (power cap), both
    # below the 2516.6 TFLOP/s peak and far above anything a broken loop would report
    zero = ds.mfma_calibration(True, 30)
    rnd = ds.mfma_calibration(False, 30)
    assert 500.0 < rnd <= zero * 1.05 and zero < 2600.0, (zero, rnd)
    with pytest.raises(ds.DepsyncError):
        ds.mfma_calibration(False, 0)


MIXED_MODES = [ds.MODE_FINE, ds.MODE_STREAMSYNC, ds.MODE_PLAIN]


@pytest.mark.parametrize("kind", [ds.ROWSYNC, ds.TILESYNC])
@pytest.mark.parametrize("pair", [(ds.TILE_128x128, ds.TILE_64x64), (ds.TILE_64x128, ds.TILE_256x128),
                                  (ds.TILE_256x192, ds.TILE_128x256), (ds.TILE_64x64, ds.TILE_128x192)])
def test_producer_and_consumer_tiles_of_different_shapes(kind, pair):
    # Section III-C: a consumer tile waits by the rows and columns of the PRODUCER's tiles, whatever
    # its own shape.  Ragged sizes; two streams (behind the wait kernel of Section III-B), stream
    # sync and plain launches agree bit for bit; one dispatch cannot hold two kernels.
    M, K1, N1, N2 = 300, 192, 576, 328
    print(f"mixed tiles pair={pair} kind={kind}", flush=True)
    t = inputs.mlp(M, K1, N1, N2, seed=17)
    Href, Yref = oracle.gemm_chain(inputs.to_f64(t["X"]), inputs.to_f64(t["W1"]), inputs.to_f64(t["W2"]), oracle.ACT_GELU)
    pol = ds.SyncPolicy(kind)
    res = [run_gemm_chain(t["X"], t["W1"], t["W2"], pol, mode, tile=pair) for mode in MIXED_MODES + [ds.MODE_FINE]]
    for H, Y in res:
        assert mid_err(H, Href) <= TOL_MID
        assert rel_err(Y, Yref) <= TOL_BF16
    for H, Y in res[1:]:
        assert torch.equal(res[0][0], H) and torch.equal(res[0][1], Y)
    with pytest.raises(ds.DepsyncError) as e:
        run_gemm_chain(t["X"], t["W1"], t["W2"], pol, ds.MODE_FUSED, tile=pair)
    assert e.value.status == ds.ENOTIMPL
    assert pol.status().timed_out == 0
    pol.destroy()


def test_different_tile_shapes_with_more_producer_tiles_than_slots():
    # 1024 producer tiles of 64x64 on 512 slots, 128 consumer tiles of 128x128: on two streams the
    # consumer's workgroups start behind the wait kernel, next to the producer's persistent ones,
    # and wait for tiles those are still working through; launched back to back several times on
    # the same policy (the producer's launch of one chain may still be ending when the next begins)
    M, K1, N1, N2 = 4096, 256, 1024, 512
    t = inputs.mlp(M, K1, N1, N2, seed=19)
    Href, Yref = oracle.gemm_chain(inputs.to_f64(t["X"]), inputs.to_f64(t["W1"]), inputs.to_f64(t["W2"]), oracle.ACT_GELU)
    pair = (ds.TILE_64x64, ds.TILE_128x128)
    pol = ds.SyncPolicy(ds.ROWSYNC)
    ref = run_gemm_chain(t["X"], t["W1"], t["W2"], pol, ds.MODE_STREAMSYNC, tile=pair)
    assert mid_err(ref[0], Href) <= TOL_MID and rel_err(ref[1], Yref) <= TOL_BF16
    Xd, W1t, W2t = t["X"].cuda(), t["W1"].t().contiguous().cuda(), t["W2"].t().contiguous().cuda()
    H = torch.empty((M, N1), dtype=Xd.dtype, device="cuda")
    Y = torch.empty((M, N2), dtype=Xd.dtype, device="cuda")
    for rep in range(5):
        print(f"mixed tiles, two streams, launch {rep}", flush=True)
        H.fill_(float("nan")); Y.fill_(float("nan"))
        ds.dep_gemm_chain(Xd, W1t, H, W2t, Y, pol, mode=ds.MODE_FINE, tile=pair)
        ds.dep_gemm_chain(Xd, W1t, H, W2t, Y, pol, mode=ds.MODE_FINE, tile=pair)
        torch.cuda.synchronize()
        assert torch.equal(H, ref[0]) and torch.equal(Y, ref[1])
    assert pol.status().timed_out == 0
    pol.destroy()
