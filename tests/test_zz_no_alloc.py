"""GPU test of the allocation-free entry point dep_gemm_chain_static: through the C ABI, its output
must be bit-identical to dep_gemm_chain's (one dispatch, same policy kind and parameters), on calls
in a row that share the library's static device workspace, the later ones smaller than the first."""
import ctypes

import pytest
import torch

import inputs
import paper_2305_13450_amd as ds
from gpu_util import same

pytestmark = pytest.mark.gpu


def _chain(t, mid):
    X = t["X"].cuda()
    W1 = t["Wgu" if mid == ds.MID_SWIGLU else "W1"]
    W1t, W2t = W1.t().contiguous().cuda(), t["W2"].t().contiguous().cuda()
    n1 = W1.shape[1] // 2 if mid == ds.MID_SWIGLU else W1.shape[1]
    return X, W1t, W2t, n1


def _outputs(M, n1, n2, dtype):
    return (torch.full((M, n1), float("nan"), dtype=dtype, device="cuda"),
            torch.full((M, n2), float("nan"), dtype=dtype, device="cuda"))


def _both(t, mid, kind, stream=None, **params):
    """(H, Y) of the static entry point and of dep_gemm_chain in one-dispatch mode."""
    X, W1t, W2t, n1 = _chain(t, mid)
    M, n2 = X.shape[0], W2t.shape[0]
    Hs, Ys = _outputs(M, n1, n2, X.dtype)
    torch.cuda.synchronize()
    ds.dep_gemm_chain_static(X, W1t, Hs, W2t, Ys, kind, mid=mid, stream=stream, **params)
    torch.cuda.synchronize()
    pol = ds.SyncPolicy(kind, **params)
    H, Y = _outputs(M, n1, n2, X.dtype)
    torch.cuda.synchronize()
    ds.dep_gemm_chain(X, W1t, H, W2t, Y, pol, mode=ds.MODE_FUSED, mid=mid, stream_producer=stream)
    torch.cuda.synchronize()
    assert pol.status().timed_out == 0
    pol.destroy()
    return (Hs, Ys), (H, Y)


def test_static_entry_matches_the_allocating_one_on_calls_in_a_row():
    print("static entry: 640 rows (split along K), then 200 rows, then 1 row, then 640 again", flush=True)
    # the first chain is split along K (few tiles on 256 CUs), so it uses semaphores, arrival
    # counters and partial tiles of the static array; the following, smaller ones find all of
    # that as the first left it
    big = inputs.mlp(640, 4096, 1536, 1024, seed=5)
    small = inputs.mlp(200, 512, 768, 320, seed=6)
    one = inputs.mlp(1, 4096, 1536, 1024, seed=7)
    for t, kind in ((big, ds.ROWSYNC), (small, ds.TILESYNC), (one, ds.ROWSYNC), (big, ds.TILESYNC), (small, ds.TILESYNC)):
        (Hs, Ys), (H, Y) = _both(t, ds.MID_GELU, kind)
        assert not torch.isnan(Ys).any()
        assert same(Hs, H, "H static/policy") and same(Ys, Y, "Y static/policy")


def test_static_entry_gated_mlp_and_side_stream():
    t = inputs.swiglu(300, 1024, 1408, 512, seed=8)
    s = torch.cuda.Stream()
    for kind in (ds.TILESYNC, ds.STRIDEDSYNC, ds.ROWSYNC):
        (Hs, Ys), (H, Y) = _both(t, ds.MID_SWIGLU, kind, stream=s, count=2 if kind == ds.STRIDEDSYNC else 0)
        assert same(Hs, H, "H static/policy") and same(Ys, Y, "Y static/policy")
    # repeated chains of one geometry back to back without a host synchronisation in between
    X, W1t, W2t, n1 = _chain(t, ds.MID_SWIGLU)
    outs = [_outputs(300, n1, 512, X.dtype) for _ in range(6)]
    torch.cuda.synchronize()
    for Hs, Ys in outs:
        ds.dep_gemm_chain_static(X, W1t, Hs, W2t, Ys, ds.TILESYNC, mid=ds.MID_SWIGLU, stream=s)
    torch.cuda.synchronize()
    for Hs, Ys in outs[1:]:
        assert same(Hs, outs[0][0]) and same(Ys, outs[0][1])


def test_static_entry_rejects_what_does_not_fit():
    # 32768 producer tiles under TileSync need more semaphores than the static workspace holds
    M, K1, N1, N2 = 8192, 64, 16384, 64
    X = torch.zeros((M, K1), dtype=torch.bfloat16, device="cuda")
    W1t = torch.zeros((N1, K1), dtype=torch.bfloat16, device="cuda")
    W2t = torch.zeros((N2, N1), dtype=torch.bfloat16, device="cuda")
    H = torch.zeros((M, N1), dtype=torch.bfloat16, device="cuda")
    Y = torch.full((M, N2), 7.0, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(ds.DepsyncError) as e:
        ds.dep_gemm_chain_static(X, W1t, H, W2t, Y, ds.TILESYNC, tile=ds.TILE_64x64)
    assert e.value.status == ds.ELIMIT
    with pytest.raises(ds.DepsyncError) as e:      # no trace area
        ds.dep_gemm_chain_static(X, W1t, H, W2t, Y, ds.ROWSYNC, flags=ds.FLAG_TRACE)
    assert e.value.status == ds.EINVAL
    d = ds._gemm_desc(X, W1t, H, W2t, Y, ds.MID_GELU, ds.TILE_AUTO)
    assert ds._lib().dep_gemm_chain_static(ctypes.byref(d), 9, None, None) == ds.EINVAL
    assert ds._lib().dep_gemm_chain_static(None, ds.ROWSYNC, None, None) == ds.EINVAL
    torch.cuda.synchronize()
    assert bool((Y == 7.0).all())                  # nothing was enqueued
