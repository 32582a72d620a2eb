"""GPU parity tests of the three-stage attention chain (QKV GeMM -> causal attention -> output
GeMM, Fig. 2b) against the fp64 oracle, and bit-exactness across the launch modes."""
import numpy as np
import pytest
import torch

import inputs
import oracle
import paper_2305_13450_amd as ds
from attn_floor import attention_floor, chain_tolerance
from gpu_util import TOL_BF16, TOL_MID, mid_err, rel_err, row_err, run_attn_chain, same

pytestmark = pytest.mark.gpu

ALL_TILES = [ds.TILE_256x256, ds.TILE_256x128, ds.TILE_128x256, ds.TILE_128x128, ds.TILE_64x128, ds.TILE_64x64,
             ds.TILE_256x192, ds.TILE_128x192, ds.TILE_256x64, ds.TILE_64x64_DEEP, ds.TILE_64x192,
             ds.TILE_128x192_DEEP, ds.TILE_128x128_DEEP]
MODES = [ds.MODE_FINE, ds.MODE_STREAMSYNC, ds.MODE_PLAIN, ds.MODE_FUSED]
KINDS = [ds.ROWSYNC, ds.TILESYNC, ds.STRIDEDSYNC]


# End to end over three stages the tolerance follows from the chain's rounding floor: the error
# that rounding QKV, T and Y to the storage type leaves when every stage is otherwise exact, computed
# on the CPU from the oracle alone (attn_floor.py; pinned by test_attention_floor.py).  Where that
# floor (with its margin) lies under the stated 2e-2 the stated tolerance is asserted.


def _case(batch, seq, heads, K1, N2, seed, dtype=torch.bfloat16):
    t = inputs.attention(batch * seq, K1, heads, 128, N2, seed=seed, dtype=dtype)
    ref = oracle.attn_chain(inputs.to_f64(t["X"]), inputs.to_f64(t["Wqkv"]), inputs.to_f64(t["Wo"]), batch, seq, heads, 128)
    t["dims"] = (batch, seq, heads)
    t["floor"] = attention_floor(t, ref, batch, seq, heads, dtype=dtype)
    return t, ref


def _f64(x):
    return x.detach().to("cpu").to(torch.float64).numpy()


def _check_end_to_end(T, Y, Tr, Yr, floor, what=""):
    """The chain against the unrounded oracle: max-abs error over the RMS of the whole tensor (the
    stated metric) and per row, each within the tolerance its rounding floor gives."""
    e = {"T": rel_err(T, Tr), "Y": rel_err(Y, Yr), "T_row": row_err(T, Tr), "Y_row": row_err(Y, Yr)}
    print(f"{what} max|err|/rms whole tensor: T {e['T']:.3e} (floor {floor['T']:.3e}) Y {e['Y']:.3e} (floor {floor['Y']:.3e}); "
          f"per row: T {e['T_row']:.3e} (floor {floor['T_row']:.3e}) Y {e['Y_row']:.3e} (floor {floor['Y_row']:.3e})", flush=True)
    for k, v in e.items():
        assert v <= chain_tolerance(floor[k]), (k, v, floor[k])


def _check(got, ref, t):
    """Every stage against the oracle applied to the input that stage really read (2e-2 per row),
    and the whole chain against the oracle end to end at the tolerance its rounding floor gives."""
    QKV, T, Y = got
    QKVr, Tr, Yr = ref
    batch, seq, heads = t["dims"]
    assert mid_err(QKV, QKVr) <= TOL_MID
    assert row_err(T, oracle.causal_attention(_f64(QKV), batch, seq, heads, 128)) <= TOL_BF16
    assert row_err(Y, oracle.gemm(_f64(T), inputs.to_f64(t["Wo"]))) <= TOL_BF16
    _check_end_to_end(T, Y, Tr, Yr, t["floor"])


@pytest.fixture(scope="module")
def two_sequences():
    return _case(batch=2, seq=256, heads=2, K1=256, N2=320, seed=11)


@pytest.fixture(scope="module")
def ragged_sequence():
    # one sequence whose length is a multiple of neither the query block (128) nor the key block (64)
    return _case(batch=1, seq=333, heads=3, K1=192, N2=200, seed=12)


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("tile", ALL_TILES)
def test_two_sequences_every_tile_and_policy(two_sequences, tile, kind):
    t, ref = two_sequences
    print(f"attn batch=2 seq=256 heads=2 tile={tile} kind={kind}", flush=True)
    pol = ds.SyncPolicy(kind)
    res = [run_attn_chain(t["X"], t["Wqkv"], t["Wo"], 2, 256, 2, pol, mode, tile=tile) for mode in MODES]
    for got in res:
        _check(got, ref, t)
    for got in res[1:]:
        for a, b in zip(res[0], got):
            assert torch.equal(a, b)
    pol.status()
    pol.destroy()
    pol = ds.SyncPolicy(kind, flags=ds.FLAG_QUEUE_ORDER)      # one dispatch, tiles drawn from the queues
    got = run_attn_chain(t["X"], t["Wqkv"], t["Wo"], 2, 256, 2, pol, ds.MODE_FUSED, tile=tile)
    for a, b in zip(res[0], got):
        assert torch.equal(a, b)
    assert pol.status().timed_out == 0
    pol.destroy()


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("tile", [ds.TILE_AUTO, ds.TILE_64x64, ds.TILE_256x128])
def test_ragged_sequence(ragged_sequence, tile, kind):
    t, ref = ragged_sequence
    print(f"attn batch=1 seq=333 heads=3 tile={tile} kind={kind}", flush=True)
    pol = ds.SyncPolicy(kind)
    res = [run_attn_chain(t["X"], t["Wqkv"], t["Wo"], 1, 333, 3, pol, mode, tile=tile) for mode in MODES]
    for got in res:
        _check(got, ref, t)
    for got in res[1:]:
        for a, b in zip(res[0], got):
            assert torch.equal(a, b)
    pol.destroy()


@pytest.fixture(scope="module")
def long_sequences():
    # two sequences of 1000 tokens: 16 key blocks for the last query block, ragged on both ends
    return _case(batch=1, seq=1000, heads=2, K1=128, N2=256, seed=13)


@pytest.mark.parametrize("ksplit", [0, 2, 3, 8])
@pytest.mark.parametrize("kind", KINDS)
def test_keys_of_long_causal_tiles_split_over_workgroups(long_sequences, ksplit, kind):
    # A causal tile's key blocks are one dependent chain, so the attention stage splits every tile's
    # keys over workgroups (0: the library's own choice); the last part to arrive combines the parts in
    # key order, so every launch mode and timing gives the same bits.
    t, ref = long_sequences
    print(f"attn seq=1000 heads=2 ksplit={ksplit} kind={kind}", flush=True)
    pol = ds.SyncPolicy(kind, ksplit=ksplit)
    res = [run_attn_chain(t["X"], t["Wqkv"], t["Wo"], 1, 1000, 2, pol, mode) for mode in MODES]
    _check(res[0], ref, t)
    for got in res[1:]:
        for a, b, name in zip(res[0], got, ("QKV", "T", "Y")):
            assert same(a, b, name)
    # a delayed producer tile and the reversed order: the parts arrive in another order, same bits
    slow = ds.SyncPolicy(kind, ksplit=ksplit, delay_tile=2, delay_iters=100000, flags=ds.FLAG_REVERSE_ORDER)
    got = run_attn_chain(t["X"], t["Wqkv"], t["Wo"], 1, 1000, 2, slow, ds.MODE_FINE)
    for a, b, name in zip(res[0], got, ("QKV", "T", "Y")):
        assert same(a, b, name)
    assert pol.status().timed_out == 0 and slow.status().timed_out == 0
    pol.destroy()
    slow.destroy()


def test_fp16_chain_meets_the_whole_tensor_tolerance():
    # in the paper's precision (fp16) the chain meets max-abs / RMS <= 2e-2 over the whole tensors
    t, (QKVr, Tr, Yr) = _case(batch=2, seq=256, heads=2, K1=256, N2=320, seed=11, dtype=torch.float16)
    pol = ds.SyncPolicy(ds.STRIDEDSYNC)
    res = [run_attn_chain(t["X"], t["Wqkv"], t["Wo"], 2, 256, 2, pol, mode) for mode in MODES]
    assert chain_tolerance(t["floor"]["T"]) == TOL_BF16 and chain_tolerance(t["floor"]["Y"]) == TOL_BF16
    for QKV, T, Y in res:
        assert mid_err(QKV, QKVr, ulp=2.0 ** -11) <= TOL_MID
        assert rel_err(T, Tr) <= TOL_BF16
        assert rel_err(Y, Yr) <= TOL_BF16
    for got in res[1:]:
        for a, b in zip(res[0], got):
            assert torch.equal(a, b)
    pol.destroy()


@pytest.mark.parametrize("M", inputs.CFG4["Ms"])
def test_gpt3_attention_shard_full_size(M):
    # config 4 at full size (12 of GPT-3's 96 heads, batch 1, seq = M) in the launch configuration
    # the benchmark times: library-chosen tile, Strided (QKV -> attention) + Tile (attention -> Wo)
    c = inputs.CFG4
    print(f"attn cfg4 M={M}", flush=True)
    t, ref = _case(batch=1, seq=M, heads=c["heads"], K1=c["K1"], N2=c["N2"], seed=0)
    pol = ds.SyncPolicy(ds.STRIDEDSYNC)
    polq = ds.SyncPolicy(ds.STRIDEDSYNC, flags=ds.FLAG_QUEUE_ORDER)
    # what bench.py does before it times: the library measures its tile, split and tile order
    E = c["heads"] * 128
    Xd, Wq, Wo = t["X"].cuda(), t["Wqkv"].t().contiguous().cuda(), t["Wo"].t().contiguous().cuda()
    bufs = [torch.empty((M, n), dtype=Xd.dtype, device="cuda") for n in (3 * E, E, c["N2"])]
    ds.gemm_chain_autotune(Xd, Wq, bufs[0], Wo, bufs[2], pol, mid=ds.MID_CAUSAL_ATTN, reps=2, T=bufs[1],
                           batch=1, seq=M, heads=c["heads"], head_dim=128)   # remembered per chain shape and policy kind
    torch.cuda.synchronize()
    del bufs
    fine = run_attn_chain(t["X"], t["Wqkv"], t["Wo"], 1, M, c["heads"], pol, ds.MODE_FINE)
    _check(fine, ref, t)
    for what, p, mode in (("streamsync", pol, ds.MODE_STREAMSYNC), ("fused", pol, ds.MODE_FUSED),
                          ("fused, dispatch queues", polq, ds.MODE_FUSED)):
        other = run_attn_chain(t["X"], t["Wqkv"], t["Wo"], 1, M, c["heads"], p, mode)
        for a, b, name in zip(fine, other, ("QKV", "T", "Y")):
            assert same(a, b, f"{name} fine/{what}")
    assert pol.status().timed_out == 0 and polq.status().timed_out == 0
    pol.destroy()
    polq.destroy()


def test_causality_on_the_device(two_sequences):
    # changing the LAST token of each sequence must leave every earlier row of T and Y unchanged
    t, _ = two_sequences
    pol = ds.SyncPolicy(ds.TILESYNC)
    base = run_attn_chain(t["X"], t["Wqkv"], t["Wo"], 2, 256, 2, pol, ds.MODE_FINE)
    X2 = t["X"].clone()
    X2[255] += 1.0
    X2[511] -= 1.0
    pert = run_attn_chain(X2, t["Wqkv"], t["Wo"], 2, 256, 2, pol, ds.MODE_FINE)
    keep = torch.ones(512, dtype=torch.bool)
    keep[255] = keep[511] = False
    for a, b in zip(base, pert):
        assert torch.equal(a[keep.cuda()], b[keep.cuda()])
        assert not torch.equal(a[~keep.cuda()], b[~keep.cuda()])
    pol.destroy()


def test_repeated_launches_and_delayed_producer(two_sequences):
    t, ref = two_sequences
    pol = ds.SyncPolicy(ds.TILESYNC, delay_tile=3, delay_iters=200000)
    first = run_attn_chain(t["X"], t["Wqkv"], t["Wo"], 2, 256, 2, pol, ds.MODE_STREAMSYNC)
    for i in range(4):
        got = run_attn_chain(t["X"], t["Wqkv"], t["Wo"], 2, 256, 2, pol, ds.MODE_FINE if i % 2 == 0 else ds.MODE_FUSED)
        for a, b in zip(first, got):
            assert torch.equal(a, b)
    _check(first, ref, t)
    pol.destroy()


def test_invalid_attention_arguments(two_sequences):
    t, _ = two_sequences
    pol = ds.SyncPolicy(ds.ROWSYNC)
    X = t["X"].cuda()
    Wq = t["Wqkv"].t().contiguous().cuda()
    Wo = t["Wo"].t().contiguous().cuda()
    QKV = torch.empty((512, 768), dtype=X.dtype, device="cuda")
    T = torch.empty((512, 256), dtype=X.dtype, device="cuda")
    Y = torch.empty((512, 320), dtype=X.dtype, device="cuda")
    kw = dict(mode=ds.MODE_FINE, mid=ds.MID_CAUSAL_ATTN)
    with pytest.raises(ds.DepsyncError):      # batch * seq != M
        ds.dep_gemm_chain(X, Wq, QKV, Wo, Y, pol, T=T, batch=2, seq=200, heads=2, head_dim=128, **kw)
    with pytest.raises(ds.DepsyncError):      # only head dimension 128 is built
        ds.dep_gemm_chain(X, Wq, QKV, Wo, Y, pol, T=T, batch=2, seq=256, heads=4, head_dim=64, **kw)
    with pytest.raises(ds.DepsyncError):      # T missing
        ds.dep_gemm_chain(X, Wq, QKV, Wo, Y, pol, batch=2, seq=256, heads=2, head_dim=128, **kw)
    torch.cuda.synchronize()
    pol.destroy()


# ---- token generation: cached keys and values (Fig. 2b, S' cached tokens) -------------------------

def _run_cached(t, kv, batch, seq, heads, pol, mode, tile=ds.TILE_AUTO):
    Xd = t["X"].cuda()
    Wqkv_t = t["Wqkv"].t().contiguous().cuda()
    Wo_t = t["Wo"].t().contiguous().cuda()
    M, E = Xd.shape[0], heads * 128
    QKV = torch.full((M, 3 * E), float("nan"), dtype=Xd.dtype, device="cuda")
    T = torch.full((M, E), float("nan"), dtype=Xd.dtype, device="cuda")
    Y = torch.full((M, t["Wo"].shape[1]), float("nan"), dtype=Xd.dtype, device="cuda")
    torch.cuda.synchronize()
    ds.dep_gemm_chain(Xd, Wqkv_t, QKV, Wo_t, Y, pol, mode=mode, mid=ds.MID_CAUSAL_ATTN, tile=tile, T=T,
                      batch=batch, seq=seq, heads=heads, head_dim=128, k_cache=kv["Kc"].cuda(), v_cache=kv["Vc"].cuda())
    torch.cuda.synchronize()
    return QKV, T, Y


@pytest.mark.parametrize("kind", [ds.ROWSYNC, ds.TILESYNC, ds.STRIDEDSYNC])
@pytest.mark.parametrize("batch,seq,cached", [
    (4, 1, 512),      # token generation: one new token per sequence
    (1, 1, 100),      # a cache that ends inside a key block
    (3, 1, 1),        # one cached token
    (1, 200, 77),     # a block of new tokens over a cache (chunked prompt): ragged on both sides
    (2, 128, 64),     # two sequences, whole query blocks
    (2, 16, 300),     # two sequences of fewer than 128 new tokens each
])
def test_attention_with_cached_keys_and_values(kind, batch, seq, cached):
    print(f"cached attention kind={kind} batch={batch} seq={seq} cached={cached}", flush=True)
    heads, K1, N2 = 2, 256, 192
    t = inputs.attention(batch * seq, K1, heads, 128, N2, seed=21 + cached)
    kv = inputs.kv_cache(batch, cached, heads, 128, seed=cached)
    Kc, Vc = inputs.to_f64(kv["Kc"]), inputs.to_f64(kv["Vc"])
    QKVr, Tr, Yr = oracle.attn_chain_cached(inputs.to_f64(t["X"]), inputs.to_f64(t["Wqkv"]), inputs.to_f64(t["Wo"]),
                                            Kc, Vc, batch, seq, heads, 128)
    pol = ds.SyncPolicy(kind)
    res = [_run_cached(t, kv, batch, seq, heads, pol, mode) for mode in (ds.MODE_FINE, ds.MODE_FUSED, ds.MODE_STREAMSYNC, ds.MODE_PLAIN)]
    QKV, T, Y = res[0]
    for other in res[1:]:
        assert all(same(a, b) for a, b in zip(res[0], other))
    # stage by stage against the oracle on the stage's own input (2e-2 per row), end to end at the
    # tolerance the chain's rounding floor gives
    assert mid_err(QKV, QKVr) <= TOL_MID
    assert row_err(T, oracle.cached_attention(_f64(QKV), Kc, Vc, batch, seq, heads, 128)) <= TOL_BF16
    assert row_err(Y, oracle.gemm(_f64(T), inputs.to_f64(t["Wo"]))) <= TOL_BF16
    _check_end_to_end(T, Y, Tr, Yr, attention_floor(t, (QKVr, Tr, Yr), batch, seq, heads, cache=(Kc, Vc)))
    assert pol.status().timed_out == 0
    pol.destroy()


def test_cached_attention_rejects_bad_caches():
    t = inputs.attention(2, 256, 2, 128, 192, seed=5)
    kv = inputs.kv_cache(2, 64, 2, 128, seed=5)
    X, Wq, Wo = t["X"].cuda(), t["Wqkv"].t().contiguous().cuda(), t["Wo"].t().contiguous().cuda()
    QKV = torch.empty((2, 768), dtype=X.dtype, device="cuda")
    T = torch.empty((2, 256), dtype=X.dtype, device="cuda")
    Y = torch.empty((2, 192), dtype=X.dtype, device="cuda")
    pol = ds.SyncPolicy(ds.ROWSYNC)
    kw = dict(mode=ds.MODE_FINE, mid=ds.MID_CAUSAL_ATTN, T=T, batch=2, seq=1, heads=2, head_dim=128)
    with pytest.raises(ValueError):           # values missing
        ds.dep_gemm_chain(X, Wq, QKV, Wo, Y, pol, k_cache=kv["Kc"].cuda(), **kw)
    with pytest.raises(ValueError):           # one cache block per sequence
        ds.dep_gemm_chain(X, Wq, QKV, Wo, Y, pol, k_cache=kv["Kc"][:1].cuda(), v_cache=kv["Vc"][:1].cuda(), **kw)
    d = ds._gemm_desc(X, Wq, QKV, Wo, Y, ds.MID_CAUSAL_ATTN, ds.TILE_AUTO, T, 2, 1, 2, 128, kv["Kc"].cuda(), kv["Vc"].cuda())
    d.ld_cache = 128                          # narrower than heads * head_dim
    assert ds._lib().dep_gemm_chain(d, pol.handle, ds.MODE_FINE, None, None) == ds.EINVAL
    d.ld_cache = 256
    d.v_cache = None
    assert ds._lib().dep_gemm_chain(d, pol.handle, ds.MODE_FINE, None, None) == ds.EINVAL
    torch.cuda.synchronize()
    pol.destroy()
