"""GPU parity at the full sizes of the paper's workloads (Section II-B, Table II, Section V), in the
launch configurations the benchmark times (the tile, split and tile order the autotuner picks for
the chain; two streams, one dispatch in block-index order and one dispatch drawing from the
dispatch queues): every fine-grained form must be bit-exact against stream synchronisation on the
whole tensors, and sampled
outputs the oracle can evaluate one by one (rows of an MLP are independent given their row of X; a
conv-chain pixel depends on a 5x5 window) must match the oracle."""
import numpy as np
import pytest
import torch

import inputs
import oracle
import paper_2305_13450_amd as ds
from attn_floor import attention_floor, chain_tolerance
from gpu_util import TOL_BF16, TOL_MID, dev, mid_err, rel_err, run_conv_chain, run_gemm_chain, same

pytestmark = pytest.mark.gpu


def _autotune_gemm(X, W1, W2, policies, mid):
    """Let the library measure its tile, split and tile order for this chain (what bench.py does
    before it times), for each policy object: the tests then run what the benchmark runs."""
    Xd, W1t, W2t = dev(X), dev(W1).t().contiguous(), dev(W2).t().contiguous()
    n1 = W1.shape[1] // 2 if mid == ds.MID_SWIGLU else W1.shape[1]
    H = torch.empty((X.shape[0], n1), dtype=X.dtype, device="cuda")
    Y = torch.empty((X.shape[0], W2.shape[1]), dtype=X.dtype, device="cuda")
    for pol in policies:
        ds.gemm_chain_autotune(Xd, W1t, H, W2t, Y, pol, mid=mid, reps=2)
    torch.cuda.synchronize()


def _sample_rows(M, n=24, seed=0):
    if M <= n:
        return list(range(M))
    rng = np.random.default_rng(seed)
    rows = {0, M - 1, M // 2, 127, 128, 255, 256} & set(range(M))
    while len(rows) < n:
        rows.add(int(rng.integers(M)))
    return sorted(rows)


@pytest.mark.parametrize("M", inputs.CFG2["Ms"])
def test_gpt3_mlp_shard(M):
    c = inputs.CFG2
    print(f"cfg2 M={M}", flush=True)
    t = inputs.mlp(M, c["K1"], c["N1"], c["N2"], seed=0)
    rows = _sample_rows(M)
    Href, Yref = oracle.gemm_chain(inputs.to_f64(t["X"][rows]), inputs.to_f64(t["W1"]), inputs.to_f64(t["W2"]), oracle.ACT_GELU)
    for kind in (ds.ROWSYNC, ds.TILESYNC):
        pol = ds.SyncPolicy(kind)
        polq = ds.SyncPolicy(kind, flags=ds.FLAG_QUEUE_ORDER)
        _autotune_gemm(t["X"], t["W1"], t["W2"], (pol,), ds.MID_GELU)
        H, Y = run_gemm_chain(t["X"], t["W1"], t["W2"], pol, ds.MODE_FINE)
        for what, p, mode in (("streamsync", pol, ds.MODE_STREAMSYNC), ("fused", pol, ds.MODE_FUSED),
                              ("fused, dispatch queues", polq, ds.MODE_FUSED)):
            Ho, Yo = run_gemm_chain(t["X"], t["W1"], t["W2"], p, mode)
            assert same(H, Ho, f"H fine/{what}") and same(Y, Yo, f"Y fine/{what}")
        assert mid_err(H[rows], Href) <= TOL_MID
        assert rel_err(Y[rows], Yref) <= TOL_BF16
        assert pol.status().timed_out == 0 and polq.status().timed_out == 0
        pol.destroy()
        polq.destroy()


@pytest.mark.parametrize("M", inputs.CFG3["Ms"])
def test_llama_swiglu_shard(M):
    c = inputs.CFG3
    print(f"cfg3 M={M}", flush=True)
    t = inputs.swiglu(M, c["K1"], c["Nh"], c["N2"], seed=0)
    rows = _sample_rows(M)
    Href, Yref = oracle.swiglu_chain(inputs.to_f64(t["X"][rows]), inputs.to_f64(t["Wgu"]), inputs.to_f64(t["W2"]))
    pol = ds.SyncPolicy(ds.TILESYNC)
    polq = ds.SyncPolicy(ds.TILESYNC, flags=ds.FLAG_QUEUE_ORDER)
    _autotune_gemm(t["X"], t["Wgu"], t["W2"], (pol,), ds.MID_SWIGLU)
    H, Y = run_gemm_chain(t["X"], t["Wgu"], t["W2"], pol, ds.MODE_FINE, mid=ds.MID_SWIGLU)
    for what, p, mode in (("streamsync", pol, ds.MODE_STREAMSYNC), ("fused", pol, ds.MODE_FUSED),
                          ("fused, dispatch queues", polq, ds.MODE_FUSED)):
        Ho, Yo = run_gemm_chain(t["X"], t["Wgu"], t["W2"], p, mode, mid=ds.MID_SWIGLU)
        assert same(H, Ho, f"H fine/{what}") and same(Y, Yo, f"Y fine/{what}")
    assert mid_err(H[rows], Href) <= TOL_MID
    assert rel_err(Y[rows], Yref) <= TOL_BF16
    assert pol.status().timed_out == 0 and polq.status().timed_out == 0
    pol.destroy()
    polq.destroy()


def _sample_pixels(B, H, W, n=32, seed=0):
    rng = np.random.default_rng(seed)
    pix = {(0, 0, 0), (0, 0, W - 1), (0, H - 1, 0), (B - 1, H - 1, W - 1), (B - 1, 0, 0), (0, H - 1, W - 1),
           (B // 2, H // 2, 0), (B // 2, 0, W // 2)}
    while len(pix) < n:
        pix.add((int(rng.integers(B)), int(rng.integers(H)), int(rng.integers(W))))
    return sorted(pix)


VGG_CASES = [(hw, ch, b) for (hw, ch) in inputs.CFG5["stages"] for b in inputs.CFG5["batches"]]


@pytest.mark.parametrize("hw,ch,batch", VGG_CASES)
def test_vgg_conv_pair(hw, ch, batch):
    print(f"cfg5 {hw}x{hw}x{ch} batch={batch}", flush=True)
    t = inputs.conv(batch, hw, hw, ch, ch, ch, seed=0)
    pol = ds.SyncPolicy(ds.STRIDEDSYNC)
    polq = ds.SyncPolicy(ds.STRIDEDSYNC, flags=ds.FLAG_QUEUE_ORDER)
    xd, w1d, w2d = dev(t["x"]), dev(t["w1"]), dev(t["w2"])
    mid, out = torch.empty((batch, hw, hw, ch), dtype=xd.dtype, device="cuda"), torch.empty((batch, hw, hw, ch), dtype=xd.dtype, device="cuda")
    ds.conv_chain_autotune(xd, w1d, mid, w2d, out, pol, reps=2)   # remembered per chain shape and policy kind
    torch.cuda.synchronize()
    del mid, out
    fine = run_conv_chain(t["x"], t["w1"], t["w2"], pol, ds.MODE_FINE)
    for what, p, mode in (("streamsync", pol, ds.MODE_STREAMSYNC), ("fused", pol, ds.MODE_FUSED),
                          ("fused, dispatch queues", polq, ds.MODE_FUSED)):
        other = run_conv_chain(t["x"], t["w1"], t["w2"], p, mode)
        assert same(fine[0], other[0], f"mid fine/{what}") and same(fine[1], other[1], f"out fine/{what}")
    assert pol.status().timed_out == 0 and polq.status().timed_out == 0
    pol.destroy()
    polq.destroy()
    pix = _sample_pixels(batch, hw, hw)
    ref = oracle.conv_chain_pixels(inputs.to_f64(t["x"]), inputs.to_f64(t["w1"]), inputs.to_f64(t["w2"]), pix)
    got = torch.stack([fine[1][b, y, x] for (b, y, x) in pix])
    assert rel_err(got, ref) <= TOL_BF16


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float16])
@pytest.mark.parametrize("batch,cached", [(4, 2048), (1, 512)])
def test_gpt3_attention_token_generation_full_size(batch, cached, dtype):
    # the generation phase at the shard's real widths, in the launch configuration bench.py times
    # (autotuned tile, keys of a (head, sequence) pair split over several workgroups): the oracle
    # computes the whole chain (a handful of rows), every stage is also checked on its own input
    from gpu_util import row_err
    print(f"generation batch={batch} cached={cached} {dtype}", flush=True)
    c = inputs.CFG4
    heads, d = c["heads"], c["d"]
    t = inputs.attention(batch, c["K1"], heads, d, c["N2"], seed=3, dtype=dtype)
    kv = inputs.kv_cache(batch, cached, heads, d, seed=3, dtype=dtype)
    Kc, Vc = inputs.to_f64(kv["Kc"]), inputs.to_f64(kv["Vc"])
    QKVr, Tr, Yr = oracle.attn_chain_cached(inputs.to_f64(t["X"]), inputs.to_f64(t["Wqkv"]), inputs.to_f64(t["Wo"]),
                                            Kc, Vc, batch, 1, heads, d)
    X, Wq, Wo = t["X"].cuda(), t["Wqkv"].t().contiguous().cuda(), t["Wo"].t().contiguous().cuda()
    kc, vc = kv["Kc"].cuda(), kv["Vc"].cuda()
    E = heads * d
    pol = ds.SyncPolicy(ds.ROWSYNC)
    kw = dict(mid=ds.MID_CAUSAL_ATTN, batch=batch, seq=1, heads=heads, head_dim=d, k_cache=kc, v_cache=vc)
    bufs = lambda: (torch.full((batch, 3 * E), float("nan"), dtype=dtype, device="cuda"),
                    torch.full((batch, E), float("nan"), dtype=dtype, device="cuda"),
                    torch.full((batch, c["N2"]), float("nan"), dtype=dtype, device="cuda"))
    QKV, T, Y = bufs()
    ds.gemm_chain_autotune(X, Wq, QKV, Wo, Y, pol, T=T, reps=2, **kw)
    res = []
    for mode in (ds.MODE_FUSED, ds.MODE_FINE, ds.MODE_STREAMSYNC):
        QKV, T, Y = bufs()
        torch.cuda.synchronize()
        ds.dep_gemm_chain(X, Wq, QKV, Wo, Y, pol, mode=mode, T=T, **kw)
        torch.cuda.synchronize()
        res.append((QKV, T, Y))
    for other in res[1:]:
        assert all(same(a, b) for a, b in zip(res[0], other))
    QKV, T, Y = res[0]
    f64 = lambda x: x.cpu().double().numpy()
    tol, ulp = (TOL_BF16, 2.0 ** -8) if dtype == torch.bfloat16 else (4e-3, 2.0 ** -11)
    assert mid_err(QKV, QKVr, ulp=ulp) <= TOL_MID
    assert row_err(T, oracle.cached_attention(f64(QKV), Kc, Vc, batch, 1, heads, d)) <= tol
    assert row_err(Y, oracle.gemm(f64(T), inputs.to_f64(t["Wo"]))) <= tol
    # end to end at the tolerance the chain's rounding floor gives (CPU, oracle only)
    floor = attention_floor(t, (QKVr, Tr, Yr), batch, 1, heads, d, dtype=dtype, cache=(Kc, Vc))
    for k, v in {"T": rel_err(T, Tr), "Y": rel_err(Y, Yr), "T_row": row_err(T, Tr), "Y_row": row_err(Y, Yr)}.items():
        print(f"generation {k}: {v:.3e} (floor {floor[k]:.3e})", flush=True)
        assert v <= chain_tolerance(floor[k], base=tol), (k, v, floor[k])
    assert pol.status().timed_out == 0
    pol.destroy()
