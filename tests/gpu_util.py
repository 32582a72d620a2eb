"""Helpers shared by the GPU parity tests (the tests call the library through its C ABI via the
thin binding; the oracle is only used to produce expected values)."""
import numpy as np
import torch

import inputs
import oracle
import paper_2305_13450_amd as ds

TOL_BF16 = 2e-2     # max-abs error normalised by the RMS of the oracle's output
TOL_FP16 = 4e-3


def rel_err(got: torch.Tensor, ref: np.ndarray) -> float:
    g = got.detach().to("cpu").to(torch.float64).numpy()
    rms = float(np.sqrt(np.mean(ref * ref)))
    return float(np.max(np.abs(g - ref))) / max(rms, 1e-30)


def mid_err(got: torch.Tensor, ref: np.ndarray, ulp: float = 2.0 ** -8) -> float:
    """Error of the 16-bit INTERMEDIATE beyond its own rounding.  One rounding to bf16 moves a value
    by up to 2^-9 of its magnitude, which for the largest of millions of GeLU outputs (about 5) is
    already 2.4e-2 of the tensor's RMS; so each element is allowed `ulp` * |ref| (one rounding plus as
    much again for the fp32 accumulation and activation) and only the excess is normalised by the RMS."""
    g = got.detach().to("cpu").to(torch.float64).numpy()
    rms = float(np.sqrt(np.mean(ref * ref)))
    return float(np.max(np.abs(g - ref) - ulp * np.abs(ref))) / max(rms, 1e-30)


TOL_MID = 2e-3


def row_err(got: torch.Tensor, ref: np.ndarray) -> float:
    """Largest error of any row, normalised by the RMS of THAT row of the oracle's output.  For the
    attention block the rows (tokens) differ in scale by the square root of their position (the
    first token's output is one row of V, a late token's an average of many), so one 16-bit
    rounding of a large early row already exceeds 2e-2 of the RMS of the whole tensor."""
    g = got.detach().to("cpu").to(torch.float64).numpy()
    rms = np.sqrt(np.mean(ref * ref, axis=1))
    return float(np.max(np.max(np.abs(g - ref), axis=1) / np.maximum(rms, 1e-30)))


def dev(t: torch.Tensor) -> torch.Tensor:
    return t.to("cuda")


def run_gemm_chain(X, W1, W2, policy, mode, mid=ds.MID_GELU, tile=ds.TILE_AUTO, poison=True, streams=None):
    """X[M,K1], W1/W2 in mathematical [K,N] shape (host or device).  Returns (H, Y) device tensors."""
    Xd = dev(X)
    W1t = dev(W1).t().contiguous()
    W2t = dev(W2).t().contiguous()
    M = X.shape[0]
    n1 = W1.shape[1] // 2 if mid == ds.MID_SWIGLU else W1.shape[1]
    H = torch.empty((M, n1), dtype=X.dtype, device="cuda")
    Y = torch.empty((M, W2.shape[1]), dtype=X.dtype, device="cuda")
    if poison:
        H.fill_(float("nan"))
        Y.fill_(float("nan"))
    sp, sc = streams if streams else (None, None)
    torch.cuda.synchronize()
    ds.dep_gemm_chain(Xd, W1t, H, W2t, Y, policy, mode=mode, mid=mid, tile=tile, stream_producer=sp, stream_consumer=sc)
    torch.cuda.synchronize()
    return H, Y


def run_conv_chain(x, w1, w2, policy, mode, tile=ds.TILE_AUTO, poison=True):
    xd, w1d, w2d = dev(x), dev(w1), dev(w2)
    B, H, W, C = x.shape
    mid = torch.empty((B, H, W, w1.shape[0]), dtype=x.dtype, device="cuda")
    out = torch.empty((B, H, W, w2.shape[0]), dtype=x.dtype, device="cuda")
    if poison:
        mid.fill_(float("nan"))
        out.fill_(float("nan"))
    torch.cuda.synchronize()
    ds.dep_conv_chain(xd, w1d, mid, w2d, out, policy, mode=mode, tile=tile)
    torch.cuda.synchronize()
    return mid, out


def run_attn_chain(X, Wqkv, Wo, batch, seq, heads, policy, mode, tile=ds.TILE_AUTO, poison=True, streams=None):
    """Attention block: X[M,K1], Wqkv[K1,3E], Wo[E,N2] with E = 128 * heads.  Returns (QKV, T, Y)."""
    Xd = dev(X)
    Wqkv_t = dev(Wqkv).t().contiguous()
    Wo_t = dev(Wo).t().contiguous()
    M, E = X.shape[0], heads * 128
    QKV = torch.empty((M, 3 * E), dtype=X.dtype, device="cuda")
    T = torch.empty((M, E), dtype=X.dtype, device="cuda")
    Y = torch.empty((M, Wo.shape[1]), dtype=X.dtype, device="cuda")
    if poison:
        for t in (QKV, T, Y):
            t.fill_(float("nan"))
    sp, sc = streams if streams else (None, None)
    torch.cuda.synchronize()
    ds.dep_gemm_chain(Xd, Wqkv_t, QKV, Wo_t, Y, policy, mode=mode, mid=ds.MID_CAUSAL_ATTN, tile=tile,
                      stream_producer=sp, stream_consumer=sc, T=T, batch=batch, seq=seq, heads=heads, head_dim=128)
    torch.cuda.synchronize()
    return QKV, T, Y


def same(a: torch.Tensor, b: torch.Tensor, what: str = "") -> bool:
    """torch.equal that says where two results differ (row / column ranges, NaN count, largest
    difference) before a bit-exactness assertion fails."""
    if torch.equal(a, b):
        return True
    bad = (a != b) | torch.isnan(a) | torch.isnan(b)
    flat = bad.reshape(-1, bad.shape[-1])
    rows = flat.any(dim=1).nonzero().flatten().tolist()
    cols = flat.any(dim=0).nonzero().flatten().tolist()
    d = (a.float() - b.float())[bad]
    print(f"MISMATCH {what}: {int(bad.sum())} elements, rows {rows[0]}..{rows[-1]} ({len(rows)}), "
          f"cols {cols[0]}..{cols[-1]} ({len(cols)}), NaN a/b {int(torch.isnan(a).sum())}/{int(torch.isnan(b).sum())}, "
          f"max |a-b| {float(d.abs().nan_to_num(0).max())}, first rows {rows[:8]}, first cols {cols[:8]}", flush=True)
    return False
