"""The error a 16-bit attention chain (Fig. 2b) has by construction, computed on the CPU from the
oracle alone: QKV = X Wqkv rounded to the storage type, T = attention(rounded QKV) rounded, and
Y = (rounded T) Wo rounded, every stage evaluated by the fp64 oracle.  What is left against the
unrounded oracle chain is the rounding of the two intermediates and of the output and nothing
else (no fp32 accumulation, no kernel).  The GPU tests derive their end-to-end tolerances from
these floors; a CPU test pins the floors themselves."""
import numpy as np
import torch

import inputs
import oracle


def _round(a: np.ndarray, dtype) -> np.ndarray:
    return torch.from_numpy(np.ascontiguousarray(a)).to(dtype).to(torch.float64).numpy()


def tensor_err(got: np.ndarray, ref: np.ndarray) -> float:
    """max-abs error normalised by the RMS of the whole reference tensor."""
    return float(np.max(np.abs(got - ref)) / np.sqrt(np.mean(ref * ref)))


def row_err(got: np.ndarray, ref: np.ndarray) -> float:
    """largest error of any row normalised by the RMS of that row of the reference."""
    rms = np.sqrt(np.mean(ref * ref, axis=1))
    return float(np.max(np.max(np.abs(got - ref), axis=1) / np.maximum(rms, 1e-30)))


def attention_floor(t, ref, batch, seq, heads, d=128, dtype=torch.bfloat16, cache=None):
    """t: inputs.attention(...) tensors; ref = (QKV, T, Y) of the unrounded oracle chain;
    cache = (Kc, Vc) float64 arrays of cached keys and values or None.
    Returns {"T": whole-tensor floor of T, "Y": ..., "T_row": per-row floor of T, "Y_row": ...}."""
    QKVr, Tr, Yr = ref
    Q16 = _round(QKVr, dtype)
    if cache is None:
        T16 = _round(oracle.causal_attention(Q16, batch, seq, heads, d), dtype)
    else:
        T16 = _round(oracle.cached_attention(Q16, cache[0], cache[1], batch, seq, heads, d), dtype)
    Y16 = _round(oracle.gemm(T16, inputs.to_f64(t["Wo"])), dtype)
    return {"T": tensor_err(T16, Tr), "Y": tensor_err(Y16, Yr), "T_row": row_err(T16, Tr), "Y_row": row_err(Y16, Yr)}


def chain_tolerance(floor: float, base: float = 2e-2, margin: float = 1.5) -> float:
    """Tolerance of an end-to-end comparison whose rounding floor is `floor`: the stated tolerance
    where the floor lies under it, else the floor with a margin for what the kernel adds on top
    (fp32 accumulation, the 16-bit probabilities of the P V product, a maximum over more samples)."""
    return base if floor * margin <= base else margin * floor
