"""GPU parity tests of dep_copy_chain (the synchronisation-overhead chain: dst = mid = src as two
dependent tiled stages) against the oracle's definition, bit for bit, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
import paper_2305_13450_amd as ds

pytestmark = pytest.mark.gpu

MODES = [ds.MODE_FINE, ds.MODE_FUSED, ds.MODE_STREAMSYNC, ds.MODE_PLAIN]


def _src(nbytes, seed):
    g = torch.Generator().manual_seed(seed)
    return torch.randint(0, 256, (nbytes,), dtype=torch.uint8, generator=g)


def _run(src_host, pol, mode, tile_bytes):
    src = src_host.cuda()
    mid = torch.full_like(src, 0xA5)
    dst = torch.full_like(src, 0x5A)
    torch.cuda.synchronize()
    ds.dep_copy_chain(src, mid, dst, pol, mode=mode, tile_bytes=tile_bytes)
    torch.cuda.synchronize()
    return mid.cpu().numpy(), dst.cpu().numpy()


@pytest.mark.parametrize("kind", [ds.TILESYNC, ds.ROWSYNC])
@pytest.mark.parametrize("nbytes,tile_bytes", [
    (4096 * 5000 + 16 * 37, 4096),      # 5001 tiles on 2048 slots, ragged last tile
    (65536 * 300, 0),                   # default tile size
    (16, 4096),                         # one 16-byte unit
    (262144 * 17 + 4096, 262144),       # large tiles, short last one
])
def test_copy_chain_all_modes(kind, nbytes, tile_bytes):
    print(f"copy kind={kind} bytes={nbytes} tile={tile_bytes}", flush=True)
    h = _src(nbytes, seed=nbytes % 1000)
    mid_ref, dst_ref = oracle.copy_chain(h.numpy())
    pol = ds.SyncPolicy(kind)
    for mode in MODES:
        mid, dst = _run(h, pol, mode, tile_bytes)
        assert np.array_equal(mid, mid_ref) and np.array_equal(dst, dst_ref), mode
    assert pol.status().timed_out == 0
    pol.destroy()


def test_copy_chain_counts_one_post_and_one_wait_per_tile():
    h = _src(4096 * 700, seed=3)
    pol = ds.SyncPolicy(ds.TILESYNC, flags=ds.FLAG_COUNT)
    _run(h, pol, ds.MODE_FINE, 4096)
    st = pol.status()
    assert st.posts == 700 and st.waits == 700
    pol.destroy()
    pol = ds.SyncPolicy(ds.ROWSYNC, flags=ds.FLAG_COUNT)
    _run(h, pol, ds.MODE_FUSED, 4096)
    st = pol.status()
    assert st.posts == 700 and st.waits == 700
    pol.destroy()


def test_copy_chain_delayed_and_reversed_producers():
    # a producer tile that posts late, and producers drawn in reverse order: consumers wait for
    # their own tile and the bytes still arrive intact
    h = _src(4096 * 3000, seed=5)
    _, dst_ref = oracle.copy_chain(h.numpy())
    for kw in (dict(delay_tile=1, delay_iters=300), dict(delay_tile=2999, delay_iters=300),
               dict(flags=ds.FLAG_REVERSE_ORDER), dict(flags=ds.FLAG_HW_ORDER)):
        pol = ds.SyncPolicy(ds.TILESYNC, **kw)
        for mode in (ds.MODE_FINE, ds.MODE_FUSED):
            if kw.get("flags") == ds.FLAG_HW_ORDER and mode == ds.MODE_FINE:
                continue                     # more tiles than slots: refused in two-stream mode
            mid, dst = _run(h, pol, mode, 4096)
            assert np.array_equal(dst, dst_ref), (kw, mode)
        assert pol.status().timed_out == 0
        pol.destroy()


def test_copy_chain_reused_buffers_never_deliver_the_previous_contents():
    # the same three buffers and one policy over many chains with fresh contents each time: a
    # consumer that read the intermediate too early or from a stale cache line would hand on
    # the previous chain's bytes
    n = 65536 * 600
    src = torch.empty(n, dtype=torch.uint8, device="cuda")
    mid = torch.empty_like(src)
    dst = torch.empty_like(src)
    pol = ds.SyncPolicy(ds.TILESYNC)
    for it in range(12):
        src.random_(0, 256)
        torch.cuda.synchronize()
        mode = (ds.MODE_FUSED, ds.MODE_FINE, ds.MODE_STREAMSYNC)[it % 3]
        ds.dep_copy_chain(src, mid, dst, pol, mode=mode, tile_bytes=65536)
        torch.cuda.synchronize()
        assert torch.equal(dst, src) and torch.equal(mid, src), (it, mode)
    pol.destroy()


def test_copy_chain_rejects_bad_arguments():
    src = torch.zeros(8192, dtype=torch.uint8, device="cuda")
    mid = torch.zeros_like(src)
    dst = torch.zeros_like(src)
    pol = ds.SyncPolicy(ds.TILESYNC)
    with pytest.raises(ds.DepsyncError) as e:
        ds.dep_copy_chain(src, mid, dst, pol, tile_bytes=1000)          # not a multiple of 4096
    assert e.value.status == ds.EINVAL
    with pytest.raises(ds.DepsyncError) as e:
        ds.dep_copy_chain(src[8:8 + 4096], mid[:4096], dst[:4096], pol)  # source not 16-byte aligned
    assert e.value.status == ds.EINVAL
    with pytest.raises(ds.DepsyncError) as e:
        ds.dep_copy_chain(src[:4104], mid[:4104], dst[:4104], pol)       # size not a multiple of 16
    assert e.value.status == ds.EINVAL
    pol.destroy()
    pol = ds.SyncPolicy(ds.STRIDEDSYNC)
    with pytest.raises(ds.DepsyncError) as e:
        ds.dep_copy_chain(src, mid, dst, pol)
    assert e.value.status == ds.ENOTIMPL
    pol.destroy()
    big = torch.zeros(4096 * 70000, dtype=torch.uint8, device="cuda")
    pol = ds.SyncPolicy(ds.TILESYNC)
    with pytest.raises(ds.DepsyncError) as e:                           # 70000 tiles: more than the semaphores
        ds.dep_copy_chain(big, torch.empty_like(big), torch.empty_like(big), pol, tile_bytes=4096)
    assert e.value.status == ds.ENOMEM
    pol.destroy()
