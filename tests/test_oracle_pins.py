"""Pins for the CPU oracle: closed forms, hand-computed cases, special cases that reduce to a
library routine, and values the paper prints.  None of these runs on a GPU."""
import math

import numpy as np
import pytest
import torch

import oracle
from oracle import sync_model as sm

rng = np.random.default_rng(1234)


# ---- pointwise ---------------------------------------------------------------

def test_pointwise_golden(golden):
    fn = {"gelu": oracle.gelu, "silu": oracle.silu}
    for op, x, v in golden("pointwise_values.txt"):
        assert fn[op](float(x)) == pytest.approx(float(v), abs=2e-10), (op, x)


def test_pointwise_limits_and_identities():
    assert oracle.gelu(40.0) == pytest.approx(40.0, rel=1e-15)
    assert oracle.gelu(-40.0) == pytest.approx(0.0, abs=1e-300)
    assert oracle.silu(50.0) == pytest.approx(50.0, rel=1e-15)
    assert abs(oracle.silu(-50.0)) < 1e-19
    for x in (0.3, 1.7, 4.0):
        # GeLU(x) - GeLU(-x) = x and silu(x) - silu(-x) = x  (Phi(x)+Phi(-x)=1, same for sigmoid)
        assert oracle.gelu(x) - oracle.gelu(-x) == pytest.approx(x, rel=1e-14)
        assert oracle.silu(x) - oracle.silu(-x) == pytest.approx(x, rel=1e-14)
        assert oracle.gelu(x) == pytest.approx(x * 0.5 * math.erfc(-x / math.sqrt(2)), rel=1e-14)
    assert oracle.relu(-3.0) == 0.0 and oracle.relu(2.5) == 2.5


# ---- GeMM --------------------------------------------------------------------

def test_gemm_hand_computed():
    A = [[1, 2, 3], [4, 5, 6]]
    B = [[7, 8], [9, 10], [11, 12]]
    # row 0: 1*7+2*9+3*11 = 58, 1*8+2*10+3*12 = 64; row 1: 139, 154
    assert oracle.gemm(A, B).tolist() == [[58.0, 64.0], [139.0, 154.0]]


def test_gemm_identity_and_ones():
    X = rng.standard_normal((7, 5))
    assert np.array_equal(oracle.gemm(X, np.eye(5)), X)
    assert np.array_equal(oracle.gemm(np.eye(7), X), X)
    assert np.array_equal(oracle.gemm(np.ones((4, 9)), np.ones((9, 6))), np.full((4, 6), 9.0))


def test_gemm_matches_library_on_rectangular():
    A = rng.standard_normal((13, 37))
    B = rng.standard_normal((37, 21))
    np.testing.assert_allclose(oracle.gemm(A, B), A @ B, rtol=1e-13, atol=1e-13)


def test_gemm_associativity():
    X = rng.standard_normal((6, 10))
    W1 = rng.standard_normal((10, 8))
    W2 = rng.standard_normal((8, 5))
    left = oracle.gemm(oracle.gemm(X, W1), W2)
    right = oracle.gemm(X, oracle.gemm(W1, W2))
    np.testing.assert_allclose(left, right, rtol=1e-12, atol=1e-12)


# ---- MLP chain ---------------------------------------------------------------

def test_chain_identity_weights_returns_gelu_of_input():
    X = rng.standard_normal((9, 16))
    H, Y = oracle.gemm_chain(X, np.eye(16), np.eye(16), oracle.ACT_GELU)
    want = np.vectorize(lambda v: 0.5 * v * math.erfc(-v / math.sqrt(2)))(X)
    np.testing.assert_allclose(Y, want, rtol=1e-14, atol=1e-16)
    assert np.array_equal(H, Y)


def test_chain_all_ones():
    M, K1, N1, N2 = 3, 4, 6, 5
    _, Y = oracle.gemm_chain(np.ones((M, K1)), np.ones((K1, N1)), np.ones((N1, N2)), oracle.ACT_GELU)
    g4 = 4 * 0.5 * math.erfc(-4 / math.sqrt(2))          # GeLU(K1)
    np.testing.assert_allclose(Y, np.full((M, N2), N1 * g4), rtol=1e-14)


def test_chain_act_none_is_plain_product_and_relu_clamps():
    X = rng.standard_normal((5, 8)); W1 = rng.standard_normal((8, 12)); W2 = rng.standard_normal((12, 4))
    _, Y = oracle.gemm_chain(X, W1, W2, oracle.ACT_NONE)
    np.testing.assert_allclose(Y, X @ W1 @ W2, rtol=1e-12, atol=1e-12)
    H, Y = oracle.gemm_chain(X, W1, W2, oracle.ACT_RELU)
    np.testing.assert_allclose(H, np.maximum(X @ W1, 0), rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(Y, np.maximum(X @ W1, 0) @ W2, rtol=1e-12, atol=1e-12)


def test_chain_output_rms_matches_gaussian_moment():
    # X ~ N(0,1), W ~ N(0,1/K): z = X W1 ~ N(0,1), Y has variance E[GeLU(z)^2] = 0.42522.
    M, K1, N1, N2 = 64, 256, 512, 64
    X = rng.standard_normal((M, K1)); W1 = rng.standard_normal((K1, N1)) / math.sqrt(K1)
    W2 = rng.standard_normal((N1, N2)) / math.sqrt(N1)
    _, Y = oracle.gemm_chain(X, W1, W2, oracle.ACT_GELU)
    assert math.sqrt(np.mean(Y * Y)) == pytest.approx(math.sqrt(0.42522), rel=0.08)


# ---- gated MLP chain -----------------------------------------------------------

def test_swiglu_up_equal_one_gives_silu():
    M, K, Nh = 4, 6, 6
    X = rng.standard_normal((M, K))
    Wg = np.eye(K)                                      # G = X
    Wu = np.zeros((K, Nh)); Xb = np.hstack([X, np.ones((M, 1))])
    Wgb = np.vstack([Wg, np.zeros((1, Nh))]); Wub = np.vstack([Wu, np.ones((1, Nh))])  # U = 1
    H, Y = oracle.swiglu_chain(Xb, np.hstack([Wgb, Wub]), np.eye(Nh))
    want = X / (1 + np.exp(-X))
    np.testing.assert_allclose(H, want, rtol=1e-14, atol=1e-16)
    np.testing.assert_allclose(Y, want, rtol=1e-14, atol=1e-16)


def test_swiglu_zero_gate_and_column_split():
    M, K, Nh, N2 = 3, 5, 4, 7
    X = rng.standard_normal((M, K)); Wu = rng.standard_normal((K, Nh)); W2 = rng.standard_normal((Nh, N2))
    _, Y = oracle.swiglu_chain(X, np.hstack([np.zeros((K, Nh)), Wu]), W2)
    assert np.array_equal(Y, np.zeros((M, N2)))
    Wg = rng.standard_normal((K, Nh))
    H, Y = oracle.swiglu_chain(X, np.hstack([Wg, Wu]), W2)
    G, U = X @ Wg, X @ Wu
    np.testing.assert_allclose(H, G / (1 + np.exp(-G)) * U, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(Y, (G / (1 + np.exp(-G)) * U) @ W2, rtol=1e-12, atol=1e-12)
    # swapping gate and up must change the answer (catches a swapped column split)
    H2, _ = oracle.swiglu_chain(X, np.hstack([Wu, Wg]), W2)
    assert not np.allclose(H, H2)


# ---- conv ----------------------------------------------------------------------

def test_conv_1x1_equals_gemm():
    B, H, W, C, K = 2, 5, 4, 6, 3
    x = rng.standard_normal((B, H, W, C)); w = rng.standard_normal((K, 1, 1, C))
    out = oracle.conv2d_nhwc(x, w)
    np.testing.assert_allclose(out.reshape(-1, K), x.reshape(-1, C) @ w.reshape(K, C).T, rtol=1e-13, atol=1e-13)
    w3 = np.zeros((K, 3, 3, C)); w3[:, 1, 1, :] = w[:, 0, 0, :]
    np.testing.assert_allclose(oracle.conv2d_nhwc(x, w3), out, rtol=1e-14, atol=1e-14)


def test_conv_delta_and_shift():
    B, H, W, C = 1, 4, 5, 3
    x = rng.standard_normal((B, H, W, C))
    w = np.zeros((C, 3, 3, C))
    for c in range(C):
        w[c, 1, 1, c] = 1.0
    assert np.array_equal(oracle.conv2d_nhwc(x, w), x)
    # one-hot tap at (r,s)=(0,2): out[y,x] = in[y-1, x+1] (cross-correlation, no flip), zero outside
    w = np.zeros((C, 3, 3, C))
    for c in range(C):
        w[c, 0, 2, c] = 1.0
    want = np.zeros_like(x)
    want[:, 1:, :-1, :] = x[:, :-1, 1:, :]
    assert np.array_equal(oracle.conv2d_nhwc(x, w), want)


def test_conv_all_ones_counts_valid_taps():
    C, K = 4, 2
    out = oracle.conv2d_nhwc(np.ones((1, 5, 6, C)), np.ones((K, 3, 3, C)))
    assert np.all(out[0, 1:-1, 1:-1] == 9 * C)
    assert np.all(out[0, 0, 1:-1] == 6 * C) and np.all(out[0, 1:-1, 0] == 6 * C)
    for (y, x) in ((0, 0), (0, 5), (4, 0), (4, 5)):
        assert np.all(out[0, y, x] == 4 * C)


def test_conv_matches_library():
    B, H, W, C, K = 2, 7, 6, 5, 4
    x = rng.standard_normal((B, H, W, C)); w = rng.standard_normal((K, 3, 3, C))
    ref = torch.nn.functional.conv2d(torch.from_numpy(x).permute(0, 3, 1, 2),
                                     torch.from_numpy(w).permute(0, 3, 1, 2), padding=1)
    np.testing.assert_allclose(oracle.conv2d_nhwc(x, w), ref.permute(0, 2, 3, 1).numpy(), rtol=1e-12, atol=1e-12)
    relu = oracle.conv2d_nhwc(x, w, oracle.ACT_RELU)
    np.testing.assert_allclose(relu, np.maximum(ref.permute(0, 2, 3, 1).numpy(), 0), rtol=1e-12, atol=1e-12)


def test_conv_chain_and_pixel_sampler_agree():
    B, H, W, C, K1, K2 = 2, 6, 5, 4, 6, 3
    x = rng.standard_normal((B, H, W, C)); w1 = rng.standard_normal((K1, 3, 3, C)); w2 = rng.standard_normal((K2, 3, 3, K1))
    mid, out = oracle.conv_chain(x, w1, w2)
    t = torch.nn.functional
    xm = t.relu(t.conv2d(torch.from_numpy(x).permute(0, 3, 1, 2), torch.from_numpy(w1).permute(0, 3, 1, 2), padding=1))
    ref = t.conv2d(xm, torch.from_numpy(w2).permute(0, 3, 1, 2), padding=1).permute(0, 2, 3, 1).numpy()
    np.testing.assert_allclose(out, ref, rtol=1e-12, atol=1e-12)
    assert mid.min() >= 0
    pix = [(b, y, xx) for b in range(B) for y in range(H) for xx in range(W)]
    samp = oracle.conv_chain_pixels(x, w1, w2, pix)
    np.testing.assert_allclose(samp, out.reshape(-1, K2), rtol=1e-12, atol=1e-12)


def test_conv_chain_interior_variance():
    # He-normal weights, unit-variance input: conv1 pre-activation has variance 2, relu halves the
    # second moment to 1, conv2 output has variance 2 in the interior.
    B, H, W, C = 1, 12, 12, 32
    x = rng.standard_normal((B, H, W, C))
    w1 = rng.standard_normal((C, 3, 3, C)) * math.sqrt(2 / (9 * C))
    w2 = rng.standard_normal((C, 3, 3, C)) * math.sqrt(2 / (9 * C))
    _, out = oracle.conv_chain(x, w1, w2)
    inner = out[:, 2:-2, 2:-2]
    assert math.sqrt(np.mean(inner * inner)) == pytest.approx(math.sqrt(2.0), rel=0.12)


# ---- attention -------------------------------------------------------------------

def _rand_qkv(batch, seq, heads, d):
    return rng.standard_normal((batch * seq, 3 * heads * d))


def test_attention_first_row_and_zero_query():
    batch, seq, heads, d = 2, 6, 3, 4
    qkv = _rand_qkv(batch, seq, heads, d)
    E = heads * d
    T = oracle.causal_attention(qkv, batch, seq, heads, d)
    for b in range(batch):
        np.testing.assert_allclose(T[b * seq], qkv[b * seq, 2 * E:], rtol=1e-14)   # row 0 sees only itself
    q0 = qkv.copy(); q0[:, :E] = 0.0
    T0 = oracle.causal_attention(q0, batch, seq, heads, d)
    V = qkv[:, 2 * E:].reshape(batch, seq, E)
    want = np.cumsum(V, axis=1) / np.arange(1, seq + 1)[None, :, None]
    np.testing.assert_allclose(T0.reshape(batch, seq, E), want, rtol=1e-13, atol=1e-14)


def test_attention_matches_library_and_head_layout():
    batch, seq, heads, d = 2, 9, 3, 8
    qkv = _rand_qkv(batch, seq, heads, d)
    E = heads * d
    T = oracle.causal_attention(qkv, batch, seq, heads, d)
    t = torch.from_numpy(qkv).reshape(batch, seq, 3, heads, d)
    q, k, v = (t[:, :, i].permute(0, 2, 1, 3) for i in range(3))
    ref = torch.nn.functional.scaled_dot_product_attention(q, k, v, is_causal=True)
    np.testing.assert_allclose(T, ref.permute(0, 2, 1, 3).reshape(batch * seq, E).numpy(), rtol=1e-12, atol=1e-13)
    # permuting heads in Q, K and V permutes the column blocks of T
    perm = [2, 0, 1]
    blocks = qkv.reshape(-1, 3, heads, d)[:, :, perm, :].reshape(-1, 3 * E)
    Tp = oracle.causal_attention(blocks, batch, seq, heads, d)
    np.testing.assert_allclose(Tp.reshape(-1, heads, d), T.reshape(-1, heads, d)[:, perm, :], rtol=1e-14)
    # a head subrange computes only those columns
    Ts = oracle.causal_attention(qkv, batch, seq, heads, d, head_range=(1, 2))
    np.testing.assert_allclose(Ts[:, d:2 * d], T[:, d:2 * d], rtol=1e-15)
    assert np.all(Ts[:, :d] == 0) and np.all(Ts[:, 2 * d:] == 0)


def test_attention_large_scores_do_not_overflow():
    batch, seq, heads, d = 1, 4, 1, 2
    qkv = np.zeros((4, 6)); qkv[:, 0] = 400.0; qkv[:, 2] = np.arange(4) * 10.0; qkv[:, 4] = np.arange(4)
    T = oracle.causal_attention(qkv, batch, seq, heads, d)
    assert np.all(np.isfinite(T))
    np.testing.assert_allclose(T[:, 0], np.arange(4), atol=1e-9)      # softmax saturates on the last key


def test_attn_chain_composition():
    batch, seq, heads, d, K1, N2 = 1, 5, 2, 4, 6, 3
    X = rng.standard_normal((batch * seq, K1)); Wqkv = rng.standard_normal((K1, 3 * heads * d))
    Wo = rng.standard_normal((heads * d, N2))
    QKV, T, Y = oracle.attn_chain(X, Wqkv, Wo, batch, seq, heads, d)
    np.testing.assert_allclose(QKV, X @ Wqkv, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(T, oracle.causal_attention(X @ Wqkv, batch, seq, heads, d), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(Y, T @ Wo, rtol=1e-12, atol=1e-12)


# ---- synchronisation model ---------------------------------------------------------

def test_policy_closed_forms():
    grid = (3, 2)
    assert [sm.row_major((x, y), grid) for y in range(2) for x in range(3)] == list(range(6))
    assert sm.tilesync_sem((2, 1), grid) == 2 * 2 + 1 and sm.tilesync_value((2, 1), grid) == 1
    assert len({sm.tilesync_sem((x, y), grid) for x in range(3) for y in range(2)}) == 6
    assert sm.rowsync_sem((2, 1), grid) == 1 and sm.rowsync_value((2, 1), grid) == 3
    # attention: Q, K, V column tiles at stride s share a semaphore, value 3
    s, g = 4, (12, 5)
    for y in range(5):
        for x in range(s):
            assert sm.stridedsync_sem((x, y), g, s) == sm.stridedsync_sem((x + s, y), g, s) == sm.stridedsync_sem((x + 2 * s, y), g, s)
    assert sm.stridedsync_value((0, 0), g, s) == 3
    assert len({sm.stridedsync_sem((x, y), g, s) for x in range(12) for y in range(5)}) == s * 5


def test_wave_model_table1(golden):
    for batch, gemm, gx, gy, gz, occ, n_sm, w, util in golden("table1_waves.txt"):
        tbs = int(gx) * int(gy) * int(gz)
        assert sm.waves(tbs, int(occ), int(n_sm)) == pytest.approx(float(w)), (batch, gemm)
        assert 100 * sm.utilization(tbs, int(occ), int(n_sm)) == pytest.approx(float(util)), (batch, gemm)


def test_fig1_example(golden):
    g = {k: int(v) for k, v in golden("fig1_example.txt")}
    grid = (g["col_tiles"], g["row_tiles"])
    n = grid[0] * grid[1]
    assert sm.wave_count(n, g["occupancy"], g["n_sm"]) == g["waves_per_kernel_stream_sync"]
    tiles = sm.gemm_chain_tiles(grid, grid)
    assert sm.simulate(g["n_sm"], tiles, stream_sync=True) == g["total_waves_stream_sync"]
    assert sm.simulate(g["n_sm"], tiles, stream_sync=False) == g["total_waves_fine_grained"]
    assert g["n_sm"] * g["waves_per_kernel_stream_sync"] - n == g["idle_sms_in_each_second_wave"]
    assert sm.sync_count("tile", grid, grid) == g["syncs_tilesync"]
    assert sm.sync_count("row", grid, grid) == g["syncs_rowsync"]


def test_copy_chain_is_the_identity_on_bytes():
    # hand-written bytes, a size that is not a multiple of the slice, and independence of the input
    src = np.array([0, 1, 2, 254, 255, 128, 127, 7], dtype=np.uint8)
    mid, dst = oracle.copy_chain(src)
    assert mid.tolist() == [0, 1, 2, 254, 255, 128, 127, 7] and dst.tolist() == mid.tolist()
    big = (np.arange((1 << 20) * 2 + 13, dtype=np.uint64) * 2654435761 >> 7).astype(np.uint8)
    mid, dst = oracle.copy_chain(big)
    assert mid.shape == big.shape and np.array_equal(dst, big) and np.array_equal(mid, big)
    big[5] ^= 0xFF
    assert dst[5] != big[5]                      # copies, not views
    f = np.array([1.5, -2.25], dtype=np.float32)
    mid, dst = oracle.copy_chain(f)
    assert dst.view(np.float32).tolist() == [1.5, -2.25]


def test_conv_chain_n_composes_the_pinned_convolution():
    # two convolutions: the same as the (separately pinned) conv_chain; three: hand-checkable
    # identity filters (centre tap 1 on the diagonal) pass a non-negative image through unchanged,
    # and a negating filter in the middle is clipped to zero by the ReLU that follows it
    rng = np.random.default_rng(5)
    x = rng.standard_normal((2, 5, 4, 3))
    w1, w2 = rng.standard_normal((4, 3, 3, 3)), rng.standard_normal((2, 3, 3, 4))
    mid, out = oracle.conv_chain(x, w1, w2)
    o = oracle.conv_chain_n(x, [w1, w2])
    assert np.array_equal(o[0], mid) and np.array_equal(o[1], out)
    ident = np.zeros((3, 3, 3, 3))
    for c in range(3):
        ident[c, 1, 1, c] = 1.0
    xp = np.abs(x)
    o = oracle.conv_chain_n(xp, [ident, ident, ident])
    assert all(np.array_equal(t, xp) for t in o)
    o = oracle.conv_chain_n(xp, [ident, -ident, ident])
    assert np.array_equal(o[0], xp) and not o[1].any() and not o[2].any()      # relu(-x) = 0 for x >= 0
    o = oracle.conv_chain_n(xp, [ident, ident, -ident])
    assert np.array_equal(o[2], -xp)                                            # no ReLU after the last


def test_cached_attention_agrees_with_the_prompt_phase():
    # (1) no cache: the separately pinned prompt-phase attention; (2) the last token of a prompt of
    # n+1 tokens is the same as one new token over a cache holding the first n tokens' keys and values
    # (and the same for a block of new tokens); (3) one cached token and one new one, by hand
    rng = np.random.default_rng(11)
    batch, heads, d, n, m = 2, 3, 4, 5, 3
    E = heads * d
    full = rng.standard_normal((batch * (n + m), 3 * E))
    T_full = oracle.causal_attention(full, batch, n + m, heads, d)
    none = np.zeros((batch, 0, E))
    assert np.allclose(oracle.cached_attention(full, none, none, batch, n + m, heads, d), T_full, rtol=0, atol=1e-12)
    seqs = full.reshape(batch, n + m, 3 * E)
    Kc, Vc = seqs[:, :n, E:2 * E].copy(), seqs[:, :n, 2 * E:].copy()
    new = seqs[:, n:, :].reshape(batch * m, 3 * E)
    T_new = oracle.cached_attention(new, Kc, Vc, batch, m, heads, d)
    want = T_full.reshape(batch, n + m, E)[:, n:, :].reshape(batch * m, E)
    assert np.allclose(T_new, want, rtol=0, atol=1e-12)
    # by hand: d = 1, one head; scores q*k = 0 for both keys -> weights 1/2, 1/2 -> mean of the values
    qkv = np.array([[0.0, 7.0, 4.0]])
    T = oracle.cached_attention(qkv, np.array([[[3.0]]]), np.array([[[10.0]]]), 1, 1, 1, 1)
    assert abs(T[0, 0] - 7.0) < 1e-12
    # and with q = ln 3: scores ln3 * (1, 0) -> weights 3/4, 1/4 (d = 1, no scaling beyond 1/sqrt(1))
    qkv = np.array([[np.log(3.0), 0.0, 4.0]])
    T = oracle.cached_attention(qkv, np.array([[[1.0]]]), np.array([[[8.0]]]), 1, 1, 1, 1)
    assert abs(T[0, 0] - (0.75 * 8.0 + 0.25 * 4.0)) < 1e-12


# ---- forward progress of the two tile orders (Section III-B) -----------------------------------

def test_block_index_order_progresses_when_workgroups_start_in_index_order():
    # tiles named by the block index: producers first in the index space, workgroups started in
    # index order (the assumption the one-dispatch block-index order rests on) -> same makespan as
    # the list schedule of Fig. 1c, nothing times out
    tiles = sm.gemm_chain_tiles((3, 2), (3, 2))
    order = list(range(len(tiles)))
    span, timeouts = sm.simulate_dispatch(4, tiles, order, by_ticket=False)
    assert span == sm.simulate(4, tiles, stream_sync=False) == 3.0 and timeouts == 0
    big = sm.gemm_chain_tiles((32, 8), (64, 8), 2.0, 1.0)
    span, timeouts = sm.simulate_dispatch(256, big, list(range(len(big))), by_ticket=False)
    assert span == sm.simulate(256, big, stream_sync=False) and timeouts == 0


def test_block_index_order_deadlocks_when_consumers_start_first_and_bounded_waits_turn_it_into_timeouts():
    # the same chain, workgroups started consumers first: six consumer workgroups on four slots
    # spin for producers that can never start (Section III-B's deadlock) ...
    tiles = sm.gemm_chain_tiles((3, 2), (3, 2))
    consumers_first = list(range(6, 12)) + list(range(6))
    span, timeouts = sm.simulate_dispatch(4, tiles, consumers_first, by_ticket=False)
    assert span is None
    # ... with bounded waits every workgroup ends, some of them timed out: the library's
    # DEPSYNC_ETIMEOUT instead of a hung GPU
    span, timeouts = sm.simulate_dispatch(4, tiles, consumers_first, by_ticket=False, spin_limit=10.0)
    assert span is not None and timeouts > 0
    # enough slots for every workgroup: any start order is safe (the library's rule for choosing the
    # block-index order on its own: all tiles of the chain resident at once)
    span, timeouts = sm.simulate_dispatch(12, tiles, consumers_first, by_ticket=False)
    assert span == 2.0 and timeouts == 0


def test_tiles_drawn_on_arrival_progress_under_any_start_order():
    # the dispatch queues: whichever workgroup starts next takes the next tile, producers before
    # consumers -> no start order can deadlock, with any number of slots
    import random
    tiles = sm.gemm_chain_tiles((5, 3), (7, 3), 1.5, 1.0)
    ref = sm.simulate(4, tiles, stream_sync=False)
    rng = random.Random(0)
    for slots in (1, 2, 4, 9):
        for _ in range(20):
            order = list(range(len(tiles)))
            rng.shuffle(order)
            span, timeouts = sm.simulate_dispatch(slots, tiles, order, by_ticket=True)
            assert span is not None and timeouts == 0
            if slots == 4:
                assert span == ref
