"""CPU oracle (test infrastructure only; the product never imports this package).

`chain_oracle.c` holds the naive fp64 definitions of the operator chains,
`sync_model.py` the paper's policy formulas, wave model and a small event-driven
schedule simulator.  This module compiles the C file with gcc and exposes it
through ctypes on numpy float64 arrays.  Only tests, the smoke check and the
benchmark's cpu_baseline leg may use it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "chain_oracle.c")
_SO = os.path.join(_HERE, "libchain_oracle.so")

ACT_NONE, ACT_GELU, ACT_RELU = 0, 1, 2

_lib = None


def build(force: bool = False) -> str:
    """Compile chain_oracle.c -> libchain_oracle.so (gcc, OpenMP)."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-o", _SO, _SRC, "-lm"]
        )
    return _SO


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_SO)
        d = ctypes.POINTER(ctypes.c_double)
        lg = ctypes.c_long
        L.oracle_num_threads.restype = ctypes.c_int
        for name in ("oracle_gelu", "oracle_silu", "oracle_relu"):
            getattr(L, name).restype = ctypes.c_double
            getattr(L, name).argtypes = [ctypes.c_double]
        L.oracle_gemm.argtypes = [lg, lg, lg, d, d, d]
        L.oracle_act_inplace.argtypes = [lg, ctypes.c_int, d]
        L.oracle_gemm_chain.argtypes = [lg, lg, lg, lg, d, d, d, ctypes.c_int, d, d]
        L.oracle_swiglu_chain.argtypes = [lg, lg, lg, lg, d, d, d, d, d, d]
        L.oracle_causal_attention.argtypes = [lg, lg, lg, lg, d, lg, lg, lg, lg, d, lg, lg, lg]
        L.oracle_attn_chain.argtypes = [lg, lg, lg, lg, lg, lg, d, d, d, d, d, d]
        L.oracle_conv2d_nhwc.argtypes = [lg, lg, lg, lg, lg, lg, lg, d, d, ctypes.c_int, d]
        L.oracle_conv_chain.argtypes = [lg, lg, lg, lg, lg, lg, d, d, d, d, d]
        L.oracle_conv_chain_pixels.argtypes = [lg, lg, lg, lg, lg, lg, d, d, d, lg,
                                               ctypes.POINTER(ctypes.c_long), d]
        _lib = L
    return _lib


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def gelu(x: float) -> float:
    return float(lib().oracle_gelu(float(x)))


def silu(x: float) -> float:
    return float(lib().oracle_silu(float(x)))


def relu(x: float) -> float:
    return float(lib().oracle_relu(float(x)))


def gemm(A, B) -> np.ndarray:
    """A[M x K] @ B[K x N] by the naive triple loop."""
    A, B = _f64(A), _f64(B)
    M, K = A.shape
    K2, N = B.shape
    assert K == K2
    C = np.empty((M, N), dtype=np.float64)
    lib().oracle_gemm(M, N, K, _p(A), _p(B), _p(C))
    return C


def gemm_chain(X, W1, W2, act: int = ACT_GELU):
    """Return (H, Y) with H = act(X W1), Y = H W2 (Fig. 2a)."""
    X, W1, W2 = _f64(X), _f64(W1), _f64(W2)
    M, K1 = X.shape
    _, N1 = W1.shape
    _, N2 = W2.shape
    assert W1.shape[0] == K1 and W2.shape[0] == N1
    H = np.empty((M, N1))
    Y = np.empty((M, N2))
    lib().oracle_gemm_chain(M, K1, N1, N2, _p(X), _p(W1), _p(W2), act, _p(H), _p(Y))
    return H, Y


def swiglu_chain(X, Wgu, W2):
    """Return (H, Y): H = silu(X Wgate) * (X Wup), Y = H W2; Wgu = [Wgate | Wup] (Fig. 3)."""
    X, Wgu, W2 = _f64(X), _f64(Wgu), _f64(W2)
    M, K1 = X.shape
    Nh = Wgu.shape[1] // 2
    N2 = W2.shape[1]
    assert Wgu.shape == (K1, 2 * Nh) and W2.shape[0] == Nh
    GU = np.empty((M, 2 * Nh))
    H = np.empty((M, Nh))
    Y = np.empty((M, N2))
    lib().oracle_swiglu_chain(M, K1, Nh, N2, _p(X), _p(Wgu), _p(W2), _p(GU), _p(H), _p(Y))
    return H, Y


def causal_attention(QKV, batch: int, seq: int, heads: int, d: int, head_range=None):
    """T[M x heads*d] from QKV[M x 3*heads*d] (Q | K | V column blocks), Fig. 2b prompt phase."""
    QKV = _f64(QKV)
    M, ld = QKV.shape
    E = heads * d
    assert M == batch * seq and ld == 3 * E
    h0, h1 = head_range if head_range is not None else (0, heads)
    T = np.zeros((M, E))
    lib().oracle_causal_attention(batch, seq, heads, d, _p(QKV), ld, 0, E, 2 * E, _p(T), E, h0, h1)
    return T


def attn_chain(X, Wqkv, Wo, batch: int, seq: int, heads: int, d: int):
    """Return (QKV, T, Y) for the attention block of Fig. 2b (prompt phase)."""
    X, Wqkv, Wo = _f64(X), _f64(Wqkv), _f64(Wo)
    M, K1 = X.shape
    E = heads * d
    N2 = Wo.shape[1]
    assert M == batch * seq and Wqkv.shape == (K1, 3 * E) and Wo.shape[0] == E
    QKV = np.empty((M, 3 * E))
    T = np.empty((M, E))
    Y = np.empty((M, N2))
    lib().oracle_attn_chain(batch, seq, heads, d, K1, N2, _p(X), _p(Wqkv), _p(Wo), _p(QKV), _p(T), _p(Y))
    return QKV, T, Y


def conv2d_nhwc(x, w, act: int = ACT_NONE):
    """x[B,H,W,C] (*) w[K,R,S,C], stride 1, zero pad (R-1)/2, cross-correlation."""
    x, w = _f64(x), _f64(w)
    B, H, W, C = x.shape
    K, R, S, C2 = w.shape
    assert C == C2
    out = np.empty((B, H, W, K))
    lib().oracle_conv2d_nhwc(B, H, W, C, K, R, S, _p(x), _p(w), act, _p(out))
    return out


def conv_chain(x, w1, w2):
    """Return (mid, out): mid = relu(conv3x3(x, w1)), out = conv3x3(mid, w2)."""
    x, w1, w2 = _f64(x), _f64(w1), _f64(w2)
    B, H, W, C = x.shape
    K1, K2 = w1.shape[0], w2.shape[0]
    assert w1.shape == (K1, 3, 3, C) and w2.shape == (K2, 3, 3, K1)
    mid = np.empty((B, H, W, K1))
    out = np.empty((B, H, W, K2))
    lib().oracle_conv_chain(B, H, W, C, K1, K2, _p(x), _p(w1), _p(w2), _p(mid), _p(out))
    return mid, out


def conv_chain_pixels(x, w1, w2, pixels):
    """The conv chain at sampled output pixels [(b,y,x), ...] -> [n, K2]."""
    x, w1, w2 = _f64(x), _f64(w1), _f64(w2)
    B, H, W, C = x.shape
    K1, K2 = w1.shape[0], w2.shape[0]
    pix = np.ascontiguousarray(np.asarray(pixels, dtype=np.int64).reshape(-1, 3))
    n = pix.shape[0]
    out = np.empty((n, K2))
    lib().oracle_conv_chain_pixels(B, H, W, C, K1, K2, _p(x), _p(w1), _p(w2), n,
                                   pix.ctypes.data_as(ctypes.POINTER(ctypes.c_long)), _p(out))
    return out


def copy_chain(src):
    """The copy -> copy chain of the synchronisation-overhead experiment (Section V): both the
    intermediate and the output are the input, byte for byte.  Returns (mid, dst) as new arrays."""
    a = np.ascontiguousarray(np.asarray(src)).view(np.uint8).reshape(-1)
    mid = np.empty_like(a)
    for i in range(0, a.size, 1 << 20):          # plain element-wise definition, in slices
        mid[i:i + (1 << 20)] = a[i:i + (1 << 20)]
    dst = np.empty_like(mid)
    for i in range(0, mid.size, 1 << 20):
        dst[i:i + (1 << 20)] = mid[i:i + (1 << 20)]
    return mid, dst


def conv_chain_n(x, ws):
    """Chain of len(ws) 3x3 convolutions (stride 1, zero padding 1), ReLU after every one but the
    last (the layers of VGG, Section V).  Returns the list of every convolution's output, the
    intermediates after their ReLU."""
    outs = []
    cur = _f64(x)
    for i, w in enumerate(ws):
        cur = conv2d_nhwc(cur, w, ACT_NONE if i == len(ws) - 1 else ACT_RELU)
        outs.append(cur)
    return outs


def cached_attention(QKV, Kc, Vc, batch: int, seq: int, heads: int, d: int):
    """Attention of `seq` new tokens per sequence over `cached` earlier tokens and themselves (Fig. 2b,
    token generation with cached keys and values): new token i of a sequence sees every cached token and
    new tokens 0..i.  QKV[batch*seq x 3*heads*d] (Q | K | V), Kc / Vc[batch x cached x heads*d].
    Written out from the definition, one (sequence, head, query) at a time."""
    QKV, Kc, Vc = _f64(QKV), _f64(Kc), _f64(Vc)
    E = heads * d
    cached = Kc.shape[1]
    assert QKV.shape == (batch * seq, 3 * E) and Kc.shape == (batch, cached, E) and Vc.shape == Kc.shape
    T = np.zeros((batch * seq, E))
    for b in range(batch):
        rows = slice(b * seq, (b + 1) * seq)
        for h in range(heads):
            cols = slice(h * d, (h + 1) * d)
            q = QKV[rows, h * d:(h + 1) * d]
            k = np.concatenate([Kc[b][:, cols], QKV[rows, E + h * d:E + (h + 1) * d]], axis=0)
            v = np.concatenate([Vc[b][:, cols], QKV[rows, 2 * E + h * d:2 * E + (h + 1) * d]], axis=0)
            for i in range(seq):
                n = cached + i + 1                       # keys this query sees
                sc = (k[:n] @ q[i]) / np.sqrt(float(d))
                sc = sc - sc.max()
                w = np.exp(sc)
                T[b * seq + i, cols] = (w / w.sum()) @ v[:n]
    return T


def attn_chain_cached(X, Wqkv, Wo, Kc, Vc, batch: int, seq: int, heads: int, d: int):
    """(QKV, T, Y) of the attention block with cached keys and values: QKV = X Wqkv, T as above, Y = T Wo."""
    QKV = gemm(X, Wqkv)
    T = cached_attention(QKV, Kc, Vc, batch, seq, heads, d)
    return QKV, T, gemm(T, Wo)
