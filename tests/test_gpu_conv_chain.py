"""GPU parity tests of dep_conv_chain (implicit-GeMM 3x3 convolutions) against the fp64 oracle."""
import numpy as np
import pytest
import torch

import inputs
import oracle
import paper_2305_13450_amd as ds
from gpu_util import TOL_BF16, TOL_MID, mid_err, rel_err, run_conv_chain

pytestmark = pytest.mark.gpu

MODES = [ds.MODE_FINE, ds.MODE_STREAMSYNC, ds.MODE_PLAIN, ds.MODE_FUSED]
KINDS = [ds.STRIDEDSYNC, ds.ROWSYNC, ds.TILESYNC]


def _oracle(t):
    return oracle.conv_chain(inputs.to_f64(t["x"]), inputs.to_f64(t["w1"]), inputs.to_f64(t["w2"]))


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("tile", [ds.TILE_256x256, ds.TILE_128x128, ds.TILE_64x64, ds.TILE_256x192, ds.TILE_128x192, ds.TILE_256x64, ds.TILE_64x64_DEEP, ds.TILE_64x192,
                                  ds.TILE_128x192_DEEP, ds.TILE_128x128_DEEP])
def test_conv_chain_small_images_all_policies(kind, tile):
    # 3 images of 13x11 pixels (429 rows of the implicit GeMM: several row tiles, ragged tail, images
    # that straddle tile boundaries), 64 -> 128 -> 64 channels
    print(f"conv kind={kind} tile={tile}", flush=True)
    t = inputs.conv(3, 13, 11, 64, 128, 64, seed=2)
    mid_ref, out_ref = _oracle(t)
    pol = ds.SyncPolicy(kind)
    res = [run_conv_chain(t["x"], t["w1"], t["w2"], pol, mode, tile=tile) for mode in MODES]
    for mid, out in res:
        assert mid_err(mid, mid_ref) <= TOL_MID
        assert rel_err(out, out_ref) <= TOL_BF16
    for mid, out in res[1:]:
        assert torch.equal(res[0][0], mid) and torch.equal(res[0][1], out)
    pol.destroy()
    pol = ds.SyncPolicy(kind, flags=ds.FLAG_QUEUE_ORDER)      # one dispatch, tiles drawn from the queues
    mid, out = run_conv_chain(t["x"], t["w1"], t["w2"], pol, ds.MODE_FUSED, tile=tile)
    assert torch.equal(res[0][0], mid) and torch.equal(res[0][1], out)
    assert pol.status().timed_out == 0
    pol.destroy()


def test_conv_chain_one_pixel_wide_and_tiny_images():
    for (B, H, W) in ((2, 1, 9), (2, 7, 1), (5, 2, 2), (1, 1, 1)):
        t = inputs.conv(B, H, W, 64, 64, 64, seed=4)
        mid_ref, out_ref = _oracle(t)
        pol = ds.SyncPolicy(ds.STRIDEDSYNC)
        mid, out = run_conv_chain(t["x"], t["w1"], t["w2"], pol, ds.MODE_FINE, tile=ds.TILE_64x64)
        assert mid_err(mid, mid_ref) <= TOL_MID and rel_err(out, out_ref) <= TOL_BF16, (B, H, W)
        pol.destroy()


def test_conv_chain_delayed_halo_row_is_waited_for():
    # 28x28x128 image: a row tile of 64 pixels spans 2.3 image rows, so a consumer tile reads three or
    # four producer row tiles (its own and the halo above and below).  Delaying a halo producer must
    # not change the result under any policy.
    t = inputs.conv(1, 28, 28, 128, 128, 128, seed=6)
    mid_ref, out_ref = _oracle(t)
    for kind in KINDS:
        # the reference of each policy: the same kernels under stream sync (how a stage is split along
        # K depends on where the policy's dependency segments start, so policies may differ in rounding)
        base = ds.SyncPolicy(kind)
        _, out0 = run_conv_chain(t["x"], t["w1"], t["w2"], base, ds.MODE_STREAMSYNC, tile=ds.TILE_64x64)
        assert rel_err(out0, out_ref) <= TOL_BF16
        base.destroy()
        for delay_tile in (1, 6, 13, 26):      # producer tiles (2 channel tiles per row tile)
            pol = ds.SyncPolicy(kind, delay_tile=delay_tile, delay_iters=200)
            _, out = run_conv_chain(t["x"], t["w1"], t["w2"], pol, ds.MODE_FINE, tile=ds.TILE_64x64)
            assert torch.equal(out, out0), (kind, delay_tile)
            pol.destroy()
        pol = ds.SyncPolicy(kind, flags=ds.FLAG_REVERSE_ORDER)
        _, out = run_conv_chain(t["x"], t["w1"], t["w2"], pol, ds.MODE_FINE, tile=ds.TILE_64x64)
        assert torch.equal(out, out0), (kind, "reversed")
        pol.destroy()


def test_conv_chain_vgg_stage_sampled_pixels():
    # VGG-19 stage (56x56, 256 -> 256), batch 4: output checked at sampled pixels the oracle evaluates
    # one by one (corners, edges, image boundaries inside the batch, interior)
    B, H, W, C = 4, 56, 56, 256
    t = inputs.conv(B, H, W, C, C, C, seed=0)
    pol = ds.SyncPolicy(ds.STRIDEDSYNC)
    outs = [run_conv_chain(t["x"], t["w1"], t["w2"], pol, mode)[1] for mode in (ds.MODE_FINE, ds.MODE_STREAMSYNC)]
    assert torch.equal(outs[0], outs[1])
    rng = np.random.default_rng(0)
    pix = [(0, 0, 0), (0, 0, W - 1), (0, H - 1, 0), (B - 1, H - 1, W - 1), (1, 0, 0), (0, H - 1, W - 1), (2, 17, 0), (3, 0, 31)]
    pix += [(int(rng.integers(B)), int(rng.integers(H)), int(rng.integers(W))) for _ in range(40)]
    ref = oracle.conv_chain_pixels(inputs.to_f64(t["x"]), inputs.to_f64(t["w1"]), inputs.to_f64(t["w2"]), pix)
    got = torch.stack([outs[0][b, y, x] for (b, y, x) in pix]).cpu().double().numpy()
    rms = float(np.sqrt(np.mean(ref * ref)))
    assert float(np.max(np.abs(got - ref))) / rms <= TOL_BF16
    pol.destroy()


def test_conv_chain_rejects_bad_channels():
    x = torch.zeros((1, 4, 4, 32), dtype=torch.bfloat16, device="cuda")
    w1 = torch.zeros((64, 3, 3, 32), dtype=torch.bfloat16, device="cuda")
    mid = torch.zeros((1, 4, 4, 64), dtype=torch.bfloat16, device="cuda")
    w2 = torch.zeros((64, 3, 3, 64), dtype=torch.bfloat16, device="cuda")
    out = torch.zeros((1, 4, 4, 64), dtype=torch.bfloat16, device="cuda")
    pol = ds.SyncPolicy(ds.STRIDEDSYNC)
    with pytest.raises(ds.DepsyncError) as e:
        ds.dep_conv_chain(x, w1, mid, w2, out, pol)
    assert e.value.status == ds.EINVAL
    pol.destroy()


def test_posted_tiles_are_visible_on_every_xcd_repeated():
    # Regression: the post must wait for the L2 write-back of the tile before the semaphore moves,
    # or a consumer on another XCD occasionally reads the (NaN-poisoned) intermediate from memory
    # before the tile's data has arrived there.  Many short chains with fresh poisoned buffers.
    t = inputs.conv(1, 112, 112, 128, 128, 128, seed=0)
    x, w1, w2 = t["x"].cuda(), t["w1"].cuda(), t["w2"].cuda()
    for kind in (ds.TILESYNC, ds.STRIDEDSYNC):
        pol = ds.SyncPolicy(kind)
        ref_mid, ref_out = run_conv_chain(t["x"], t["w1"], t["w2"], pol, ds.MODE_STREAMSYNC)
        for mode in (ds.MODE_FINE, ds.MODE_FUSED):
            differ = 0
            for _ in range(250):
                mid = torch.full_like(ref_mid, float("nan"))
                out = torch.full_like(ref_out, float("nan"))
                torch.cuda.synchronize()
                ds.dep_conv_chain(x, w1, mid, w2, out, pol, mode=mode)
                torch.cuda.synchronize()
                differ += int(not (torch.equal(out, ref_out) and torch.equal(mid, ref_mid)))
            assert differ == 0, (kind, mode, differ)
        pol.destroy()


def test_conv_autotune_picks_a_tile_the_library_then_uses():
    t = inputs.conv(2, 20, 24, 64, 128, 64, seed=29)
    x, w1, w2 = t["x"].cuda(), t["w1"].cuda(), t["w2"].cuda()
    mid = torch.empty((2, 20, 24, 128), dtype=x.dtype, device="cuda")
    out = torch.empty((2, 20, 24, 64), dtype=x.dtype, device="cuda")
    pol = ds.SyncPolicy(ds.STRIDEDSYNC)
    tile = ds.conv_chain_autotune(x, w1, mid, w2, out, pol, reps=2)
    assert ds.conv_chain_plan(x, w1, mid, w2, out, pol).tile_prod == tile
    mref, oref = oracle.conv_chain(inputs.to_f64(t["x"]), inputs.to_f64(t["w1"]), inputs.to_f64(t["w2"]))
    a = run_conv_chain(t["x"], t["w1"], t["w2"], pol, ds.MODE_FINE)
    b = run_conv_chain(t["x"], t["w1"], t["w2"], pol, ds.MODE_STREAMSYNC)
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])
    assert rel_err(a[1], oref) <= TOL_BF16
    pol.destroy()


@pytest.mark.parametrize("kind", [ds.ROWSYNC, ds.TILESYNC, ds.STRIDEDSYNC])
def test_conv_chain_split_k(kind):
    # 9 * C / 64 = 18 K steps: three parts are one filter row each
    t = inputs.conv(1, 14, 14, 128, 128, 64, seed=43)
    mref, oref = oracle.conv_chain(inputs.to_f64(t["x"]), inputs.to_f64(t["w1"]), inputs.to_f64(t["w2"]))
    for ksplit in (3, 6):
        pol = ds.SyncPolicy(kind, ksplit=ksplit)
        res = [run_conv_chain(t["x"], t["w1"], t["w2"], pol, mode, tile=ds.TILE_64x64)
               for mode in (ds.MODE_FINE, ds.MODE_FUSED, ds.MODE_STREAMSYNC, ds.MODE_PLAIN)]
        for mid, out in res:
            assert rel_err(out, oref) <= TOL_BF16
            assert torch.equal(mid, res[0][0]) and torch.equal(out, res[0][1])
        pol.destroy()


def test_conv_chain_fp16():
    # the paper's precision: same kernels instantiated for fp16, tighter tolerance
    t = inputs.conv(2, 17, 19, 64, 128, 64, seed=53, dtype=torch.float16)
    mref, oref = oracle.conv_chain(inputs.to_f64(t["x"]), inputs.to_f64(t["w1"]), inputs.to_f64(t["w2"]))
    pol = ds.SyncPolicy(ds.STRIDEDSYNC)
    res = [run_conv_chain(t["x"], t["w1"], t["w2"], pol, mode)
           for mode in (ds.MODE_FINE, ds.MODE_FUSED, ds.MODE_STREAMSYNC, ds.MODE_PLAIN)]
    for mid, out in res:
        assert mid_err(mid, mref, ulp=2.0 ** -11) <= TOL_MID
        assert rel_err(out, oref) <= 4e-3
        assert torch.equal(mid, res[0][0]) and torch.equal(out, res[0][1])
    pol.destroy()


@pytest.mark.parametrize("hw,ch,batch", [(7, 512, 3), (14, 256, 2), (28, 128, 1)])
def test_conv_chain_resnet_pair_shapes(hw, ch, batch):
    # the paper's second conv workload: ResNet-38's pairs of 3x3 convolutions (images of 7x7 pixels are
    # smaller than a row tile, so one tile spans several images and its halo crosses image boundaries)
    print(f"resnet pair {hw}x{hw}x{ch} batch {batch}", flush=True)
    t = inputs.conv(batch, hw, hw, ch, ch, ch, seed=71)
    mid_ref, out_ref = _oracle(t)
    pol = ds.SyncPolicy(ds.STRIDEDSYNC)
    res = [run_conv_chain(t["x"], t["w1"], t["w2"], pol, mode) for mode in MODES]
    for mid, out in res:
        assert mid_err(mid, mid_ref) <= TOL_MID
        assert rel_err(out, out_ref) <= TOL_BF16
        assert torch.equal(mid, res[0][0]) and torch.equal(out, res[0][1])
    pol.destroy()


def _run_conv_n(x, ws, pol, mode, tile=ds.TILE_AUTO):
    xd = x.cuda()
    wd = [w.cuda() for w in ws]
    B, H, W, _ = x.shape
    outs = [torch.full((B, H, W, w.shape[0]), float("nan"), dtype=x.dtype, device="cuda") for w in ws]
    torch.cuda.synchronize()
    ds.dep_conv_chain_n(xd, wd, outs, pol, mode=mode, tile=tile)
    torch.cuda.synchronize()
    return outs


def _conv_n_inputs(B, H, W, chans, seed):
    # He-normal weights as in inputs.conv, one more layer at a time from the same recipe
    ws = []
    x = None
    for i in range(len(chans) - 1):
        t = inputs.conv(B, H, W, chans[i], chans[i + 1], 64, seed=seed + i)
        if x is None:
            x = t["x"]
        ws.append(t["w1"])
    return x, ws


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("chans,tile", [((64, 128, 64, 128), ds.TILE_64x64), ((64, 64, 128, 64, 64), ds.TILE_128x128),
                                        ((128, 64, 64, 192), ds.TILE_AUTO)])
def test_conv_chain_of_three_and_four_convolutions(kind, chans, tile):
    # VGG-style layers: every stage is checked against the oracle applied to the stage's OWN input as
    # the GPU produced it (one convolution's error: the 2e-2 bar), the whole chain against the
    # oracle end to end (n - 1 roundings of intermediates compound: 2e-2 * sqrt(n - 1)), and the
    # launch modes against each other bit for bit
    print(f"conv chain n={len(chans) - 1} kind={kind} tile={tile}", flush=True)
    x, ws = _conv_n_inputs(3, 13, 11, chans, seed=80)
    n = len(ws)
    ref = oracle.conv_chain_n(inputs.to_f64(x), [inputs.to_f64(w) for w in ws])
    pol = ds.SyncPolicy(kind)
    res = [_run_conv_n(x, ws, pol, mode, tile) for mode in MODES]
    outs = res[0]
    for other in res[1:]:
        for a, b in zip(outs, other):
            assert torch.equal(a, b)
    for i in range(n):
        prev = inputs.to_f64(x) if i == 0 else outs[i - 1].cpu().double().numpy()
        stage_ref = oracle.conv2d_nhwc(prev, inputs.to_f64(ws[i]), oracle.ACT_NONE if i == n - 1 else oracle.ACT_RELU)
        if i == n - 1:
            assert rel_err(outs[i], stage_ref) <= TOL_BF16, i
        else:
            assert mid_err(outs[i], stage_ref) <= TOL_MID, i
    assert rel_err(outs[-1], ref[-1]) <= TOL_BF16 * (n - 1) ** 0.5
    assert pol.status().timed_out == 0
    pol.destroy()


def test_conv_chain_n_delayed_middle_stage_and_bad_arguments():
    x, ws = _conv_n_inputs(1, 28, 28, (64, 64, 64, 64, 64), seed=90)
    base = ds.SyncPolicy(ds.STRIDEDSYNC)
    ref = _run_conv_n(x, ws, base, ds.MODE_STREAMSYNC, ds.TILE_64x64)
    base.destroy()
    for delay_tile in (1, 7, 13):
        pol = ds.SyncPolicy(ds.STRIDEDSYNC, delay_tile=delay_tile, delay_iters=200)
        for mode in (ds.MODE_FINE, ds.MODE_FUSED):
            outs = _run_conv_n(x, ws, pol, mode, ds.TILE_64x64)
            assert all(torch.equal(a, b) for a, b in zip(outs, ref)), (delay_tile, mode)
        pol.destroy()
    pol = ds.SyncPolicy(ds.STRIDEDSYNC)
    xd, wd = x.cuda(), [w.cuda() for w in ws]
    outs = [torch.empty((1, 28, 28, 64), dtype=x.dtype, device="cuda") for _ in ws]
    with pytest.raises(ValueError):
        ds.dep_conv_chain_n(xd, wd + wd[:1], outs + outs[:1], pol)        # five convolutions
    d = ds._conv_n_desc(xd, wd, outs, ds.TILE_AUTO)
    d.n = 5
    assert ds._lib().dep_conv_chain_n(d, pol.handle, ds.MODE_FINE, None, None) == ds.EINVAL
    d.n = 4
    d.K[1] = 72                                                          # an intermediate that is not a multiple of 64
    assert ds._lib().dep_conv_chain_n(d, pol.handle, ds.MODE_FINE, None, None) == ds.EINVAL
    pol.destroy()


@pytest.mark.parametrize("kind", KINDS)
def test_conv_pair_with_different_producer_and_consumer_tiles(kind):
    # the consumer's halo waits are computed from the producer's row tiles (Section III-C, Fig. 5c):
    # 128-row producer tiles under 64-row consumer tiles and the other way round
    t = inputs.conv(3, 13, 11, 64, 128, 64, seed=23)
    mid_ref, out_ref = _oracle(t)
    for pair in ((ds.TILE_128x128, ds.TILE_64x64), (ds.TILE_64x128, ds.TILE_256x64)):
        print(f"conv mixed tiles pair={pair} kind={kind}", flush=True)
        pol = ds.SyncPolicy(kind)
        res = [run_conv_chain(t["x"], t["w1"], t["w2"], pol, mode, tile=pair)
               for mode in (ds.MODE_FINE, ds.MODE_STREAMSYNC, ds.MODE_PLAIN, ds.MODE_FINE)]
        for mid, out in res:
            assert mid_err(mid, mid_ref) <= TOL_MID
            assert rel_err(out, out_ref) <= TOL_BF16
        for mid, out in res[1:]:
            assert torch.equal(res[0][0], mid) and torch.equal(res[0][1], out)
        assert pol.status().timed_out == 0
        pol.destroy()
