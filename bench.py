#!/usr/bin/env python3
"""Benchmark of the dependent-chain hot path on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input: the two
dependent GeMMs of the GPT-3 MLP shard (X[M,12288] W1[12288,6144] -> GeLU -> W2[6144,12288],
bf16, M = 2048) launched with fine-grained synchronisation (two streams, or all stages in one dispatch).
Inputs are resident in HBM before the timed region.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2516.6   # 256 CU x 4096 flop/clk/CU x 2.4 GHz, dense

# HBM-side bytes of one chain from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (each scaled by what the
# same counter reads for a 1 GiB copy), per workload and launch mode; see profiles/*.md for the runs.
MEASURED_TRAFFIC_BYTES = {
    ("gpt3_mlp", 2048, "fused"): (1160433 + 82393) * 1024,
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--rounds", type=int, default=3, help="interleaved timing blocks per variant (comparison table)")
    ap.add_argument("--m", type=int, default=2048, help="tokens (rows of X)")
    ap.add_argument("--workload", default="gpt3_mlp", choices=["gpt3_mlp", "llama_mlp", "gpt3_attn", "cfg1"])
    ap.add_argument("--policy", default="auto", choices=["auto", "row", "tile", "strided"])
    ap.add_argument("--tile", type=int, default=0, help="depsync_tile id, 0 = library's choice")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-autotune", action="store_true", help="use the library's model-based tile choice")
    ap.add_argument("--cpu-rows", type=int, default=384, help="rows of X the CPU oracle is timed on")
    ap.add_argument("--modes", default="fine,fused,streamsync,plain")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MiB",
                    help="also run a plain device-to-device copy of this many MiB three times, so that "
                         "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE readings can be scaled to bytes")
    return ap.parse_args()


def time_block(torch, call, sp, steps):
    """Mean latency (us) of `call` over `steps` back-to-back launches, by HIP events on stream sp
    (every launch mode returns to sp, so the events bracket whole chains)."""
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    e0.record(sp)
    for _ in range(steps):
        call()
    e1.record(sp)
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / steps


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); "
              "--gpus N with N > 1 is not supported.", file=sys.stderr)
        sys.exit(2)

    import torch
    import inputs
    import paper_2305_13450_amd as ds

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    n_cu, clock_khz = ds.device_info()

    M = args.m
    attn = None
    if args.workload == "gpt3_mlp":
        shape = dict(M=M, K1=12288, N1=6144, N2=12288); mid = ds.MID_GELU
        t = inputs.mlp(**shape)
        W1 = t["W1"]
        name = f"GPT-3 MLP shard X[{M}x12288] W1[12288x6144] GeLU W2[6144x12288] bf16"
    elif args.workload == "llama_mlp":
        shape = dict(M=M, K1=8192, Nh=2752, N2=8192); mid = ds.MID_SWIGLU
        t = inputs.swiglu(**shape)
        W1 = t["Wgu"]
        name = f"LLaMA-65B MLP shard X[{M}x8192] [Wg|Wu][8192x5504] SwiGLU W2[2752x8192] bf16"
    elif args.workload == "gpt3_attn":
        c = inputs.CFG4; mid = ds.MID_CAUSAL_ATTN
        t = inputs.attention(M, c["K1"], c["heads"], c["d"], c["N2"])
        W1 = t["Wqkv"]; t["W2"] = t["Wo"]
        attn = dict(batch=1, seq=M, heads=c["heads"], head_dim=c["d"])
        name = (f"GPT-3 attention shard X[{M}x12288] Wqkv[12288x4608] causal attention 12 heads x 128 "
                f"(batch 1, seq {M}) Wo[1536x12288] bf16")
    else:
        shape = dict(inputs.CFG1); M = shape["M"]; mid = ds.MID_GELU
        t = inputs.mlp(**shape)
        W1 = t["W1"]
        name = "cfg1 X[256x1024] W1[1024x4096] GeLU W2[4096x1024] bf16"
    X = t["X"].cuda()
    W1t = W1.t().contiguous().cuda()
    W2t = t["W2"].t().contiguous().cuda()
    n1 = W1t.shape[0] // 2 if mid == ds.MID_SWIGLU else W1t.shape[0]
    H = torch.empty((M, n1), dtype=X.dtype, device="cuda")
    Y = torch.empty((M, W2t.shape[0]), dtype=X.dtype, device="cuda")
    extra = {}
    if attn:
        extra = dict(attn, T=torch.empty((M, attn["heads"] * attn["head_dim"]), dtype=X.dtype, device="cuda"))

    if args.copy_calibration:
        src = torch.empty(args.copy_calibration << 20, dtype=torch.uint8, device="cuda").random_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    sp, sc = torch.cuda.Stream(), torch.cuda.Stream()
    kinds = {"row": ds.ROWSYNC, "tile": ds.TILESYNC, "strided": ds.STRIDEDSYNC}
    pol_names = (["row", "tile", "strided"] if attn else ["row", "tile"]) if args.policy == "auto" else [args.policy]
    modes = {"fine": ds.MODE_FINE, "fused": ds.MODE_FUSED, "streamsync": ds.MODE_STREAMSYNC, "plain": ds.MODE_PLAIN}
    want = [m for m in args.modes.split(",") if m]

    # Every (policy, launch mode) variant is warmed up, then timed in `rounds` interleaved blocks of
    # `steps` launches (the chip's clock follows its power and temperature history, so variants
    # timed one after the other are not comparable); a variant's latency is the median of its blocks.
    pols = {pn: ds.SyncPolicy(kinds[pn]) for pn in pol_names}
    if args.tile == 0 and not args.no_autotune:
        # outside the timed region: let the library time its macro-tile shapes on this chain once
        for pn in pol_names:
            ds.gemm_chain_autotune(X, W1t, H, W2t, Y, pols[pn], mid=mid, stream=sp, reps=3, **extra)
    plan = ds.gemm_chain_plan(X, W1t, H, W2t, Y, pols[pol_names[0]], mid=mid, tile=args.tile, **extra)
    variants = [(pn, mn) for pn in pol_names for mn in want
                if mn in ("fine", "fused") or pn == pol_names[0]]   # stream-sync / plain: first policy only

    def caller(pn, mn):
        pol, mode = pols[pn], modes[mn]
        def call():
            ds.dep_gemm_chain(X, W1t, H, W2t, Y, pol, mode=mode, mid=mid, tile=args.tile,
                              stream_producer=sp, stream_consumer=sc, **extra)
        return call
    calls = {v: caller(*v) for v in variants}
    for v in variants:
        for _ in range(args.warmup):
            calls[v]()
    blocks = {v: [] for v in variants}
    for _ in range(args.rounds):
        for v in variants:
            blocks[v].append(time_block(torch, calls[v], sp, args.steps))
    results = {v: sorted(b)[len(b) // 2] for v, b in blocks.items()}

    # the fine-grained variants: two streams (FINE) or one dispatch (FUSED), per policy
    fine = {v: results[v] for v in variants if v[1] in ("fine", "fused")}
    best = min(fine, key=fine.get) if fine else variants[0]
    best_pol, best_mode = best
    # the headline: W warm-up launches, then exactly K timed launches of the best variant
    for _ in range(args.warmup):
        calls[best]()
    lat = time_block(torch, calls[best], sp, args.steps)
    ss = results.get((pol_names[0], "streamsync"))
    plain = results.get((pol_names[0], "plain"))
    for pol in pols.values():
        pol.status()
        pol.destroy()
    flops, nbytes = plan.flops, plan.bytes
    tflops = flops / (lat * 1e-6) / 1e12
    hbm_bound = (nbytes / 8e12) > (flops / (PEAK_BF16_TFLOPS * 1e12))
    if hbm_bound:
        roof = {"bound": "hbm", "achieved": nbytes / (lat * 1e-6) / 1e9, "peak": 8000.0, "unit": "GB/s"}
    else:
        roof = {"bound": "mfma", "achieved": tflops, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s"}
    roof["frac"] = roof["achieved"] / roof["peak"]
    roof["traffic"] = MEASURED_TRAFFIC_BYTES.get((args.workload, M, best_mode)) if args.tile == 0 else None
    roof["kernel"] = "chain_kernel (producer + consumer dispatches of one chain, which overlap)"
    roof["per_launch"] = {"flops": flops, "bytes": nbytes, "duration_us": lat}

    out = {
        "metric": "dependent-chain latency, fine-grained sync, best of {two-stream, one-dispatch} x sync policies (mean of steps)",
        "value": lat, "unit": "us", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": lat / 1e3, "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": name, "M": M, "policy": best_pol, "launch": best_mode, "tile": ds.tile_shape(plan.tile_prod),
                   "tiles_producer": plan.n_prod, "tiles_consumer": plan.n_cons, "slots": plan.slots,
                   "waves_streamsync": plan.waves_streamsync, "waves_fine": plan.waves_fine},
        "latency_us": {f"{pn}/{mn}": round(v, 2) for (pn, mn), v in results.items()},
        "latency_blocks_us": {f"{pn}/{mn}": [round(x, 1) for x in b] for (pn, mn), b in blocks.items()},
        "speedup_vs_streamsync": (ss / lat) if ss else None,
        "speedup_vs_plain": (plain / lat) if plain else None,
        "tflops": tflops, "pct_bf16_mfma_peak": 100 * tflops / PEAK_BF16_TFLOPS,
        "device": {"cus": n_cu, "clock_mhz": clock_khz / 1e3},
        "roofline": roof,
    }

    if not args.no_cpu_baseline:
        import oracle
        rows = min(args.cpu_rows, M)
        Xs = inputs.to_f64(t["X"][:rows])
        W1f, W2f = inputs.to_f64(W1), inputs.to_f64(t["W2"])
        t0 = time.perf_counter()
        if attn:
            # causal: the first `rows` tokens of the sequence need nothing from later tokens
            oracle.attn_chain(Xs, W1f, W2f, 1, rows, attn["heads"], attn["head_dim"])
        elif mid == ds.MID_SWIGLU:
            oracle.swiglu_chain(Xs, W1f, W2f)
        else:
            oracle.gemm_chain(Xs, W1f, W2f, oracle.ACT_GELU)
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {
            "value": dt * 1e6 * (M / rows), "unit": "us", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"fp64 oracle timed on the first {rows} of {M} rows of X (rows are independent"
                      f"{', the attention of a prefix being a prefix of the attention' if attn else ''}); "
                      f"{dt:.2f} s measured, scaled by {M}/{rows} to the full chain",
            "measured_s": dt, "gflops": flops * (rows / M) / dt / 1e9,
        }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
