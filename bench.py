#!/usr/bin/env python3
"""Benchmark of the dependent-chain hot path on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input: by default the two
dependent GeMMs of the GPT-3 MLP shard (X[M,12288] W1[12288,6144] -> GeLU -> W2[6144,12288], bf16,
M = 2048) launched with fine-grained synchronisation (two streams, or all stages in one dispatch).
Inputs are resident in HBM before the timed region.  Prints ONE JSON line.

`--sweep FILE` instead runs every configuration of the workload set (GeMM chains at all M, the
attention chain, the VGG conv pairs) and writes a markdown table to FILE.
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
    ("gpt3_mlp", 2048, "fused"): (1035398 + 74933) * 1024,
    ("gpt3_attn", 2048, "fused"): (1278478 + 82272) * 1024,
    ("vgg_conv", 50176, "fused"): (327659 + 52046) * 1024,    # 56x56x256, batch 16 (the default conv shape)
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--rounds", type=int, default=3, help="interleaved timing blocks per variant (comparison table)")
    ap.add_argument("--m", type=int, default=2048, help="tokens (rows of X)")
    ap.add_argument("--workload", default="gpt3_mlp",
                    choices=["gpt3_mlp", "llama_mlp", "gpt3_attn", "gpt3_attn_gen", "cfg1", "vgg_conv", "vgg_layer", "resnet_conv"])
    ap.add_argument("--cached", type=int, default=2048, help="gpt3_attn_gen: cached tokens per sequence")
    ap.add_argument("--hw", type=int, default=56, help="vgg_conv: image height = width")
    ap.add_argument("--channels", type=int, default=256, help="vgg_conv: channels of all three tensors")
    ap.add_argument("--batch", type=int, default=16, help="vgg_conv: images")
    ap.add_argument("--policy", default="auto", choices=["auto", "row", "tile", "strided"])
    ap.add_argument("--tile", type=int, default=0, help="depsync_tile id, 0 = library's choice")
    ap.add_argument("--w-layout", default="rows", choices=["rows", "kblocked"],
                    help="GeMM chains: weights row-major [N x K] or packed [K/64][N][64]")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-autotune", action="store_true", help="use the library's model-based tile choice")
    ap.add_argument("--cpu-rows", type=int, default=2048, help="rows of X the CPU oracle is timed on")
    ap.add_argument("--modes", default="fine,fused,fused_hw,streamsync,plain",
                    help="fine: two streams; fused: one dispatch, the library's tile order (dispatch queues unless every tile is "
                         "resident at once); fused_hw: one dispatch, tiles named by the block index (DEPSYNC_FLAG_HW_ORDER, "
                         "reported, never the headline); streamsync; plain")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MiB",
                    help="also run a plain device-to-device copy of this many MiB three times, so that "
                         "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE readings can be scaled to bytes")
    ap.add_argument("--mfma-calibration", type=int, default=0, metavar="MS",
                    help="also run the library's register-only bf16 MFMA loop for this many milliseconds with zero "
                         "and with random operands (the practical MFMA ceiling under the chip's power cap) and "
                         "report both in the JSON line")
    ap.add_argument("--sync-overhead", default=None, metavar="FILE",
                    help="copy -> copy chain (consumer tile i waits for producer tile i; Section V, overhead of "
                         "synchronisation): one full wave of tiles at several tile sizes, every launch mode; writes a "
                         "markdown table and prints one JSON line for the 64 KiB tile")
    ap.add_argument("--sweep", default=None, metavar="FILE", help="run all configurations, write a markdown table")
    ap.add_argument("--sweep-set", default="paper", choices=["paper", "resnet", "vgg_layers", "generation"],
                    help="rows of --sweep: the five configurations of the headline table, ResNet-38's conv pairs, or "
                         "VGG-19's layer groups of four convolutions")
    ap.add_argument("--policy-table", default=None, metavar="FILE",
                    help="Row / Tile / Strided latency per chain size and the kind the library's policy search keeps "
                         "(Section IV-A's search, Section V-C's crossover), markdown table")
    ap.add_argument("--ablation", default=None, metavar="FILE",
                    help="time the chosen workload with the optimisations of Section IV-C switched off one at a time")
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


class Workload:
    """Device buffers of one chain plus closures to plan, tune and launch it."""

    def __init__(self, torch, ds, inputs, kind, M=2048, hw=56, channels=256, batch=16, w_layout="rows", cached=2048):
        self.kind, self.M = kind, M
        self.conv = kind in ("vgg_conv", "resnet_conv")
        self.convn = kind == "vgg_layer"
        if self.conv or self.convn:
            self.M = batch * hw * hw          # rows of the implicit GeMM
        self.attn = None
        self.ds = ds
        if self.convn:
            # one VGG-19 layer group: four 3x3 convolutions of equal width, ReLU between them (Section V)
            layers = [inputs.conv(batch, hw, hw, channels, channels, 64, seed=i) for i in range(4)]
            self.t = layers
            self.x = layers[0]["x"].cuda()
            self.ws = [l["w1"].cuda() for l in layers]
            self.outs = [torch.empty((batch, hw, hw, channels), dtype=self.x.dtype, device="cuda") for _ in range(4)]
            self.name = f"VGG layer of four convs {hw}x{hw}x{channels}, ReLU between, batch {batch}, 3x3 s1 p1, NHWC bf16"
            self.policies = ["strided", "row", "tile"]
            return
        if self.conv:
            t = inputs.conv(batch, hw, hw, channels, channels, channels)
            self.t = t
            self.x, self.w1, self.w2 = t["x"].cuda(), t["w1"].cuda(), t["w2"].cuda()
            self.mid_t = torch.empty((batch, hw, hw, channels), dtype=self.x.dtype, device="cuda")
            self.out = torch.empty_like(self.mid_t)
            net = "VGG" if kind == "vgg_conv" else "ResNet-38"
            self.name = f"{net} conv pair {hw}x{hw}x{channels} -> ReLU -> {channels}, batch {batch}, 3x3 s1 p1, NHWC bf16"
            self.policies = ["strided", "row", "tile"]
            return
        if kind == "gpt3_mlp":
            t = inputs.mlp(M=M, K1=12288, N1=6144, N2=12288); self.mid = ds.MID_GELU; W1 = t["W1"]
            self.name = f"GPT-3 MLP shard X[{M}x12288] W1[12288x6144] GeLU W2[6144x12288] bf16"
        elif kind == "llama_mlp":
            t = inputs.swiglu(M=M, K1=8192, Nh=2752, N2=8192); self.mid = ds.MID_SWIGLU; W1 = t["Wgu"]
            self.name = f"LLaMA-65B MLP shard X[{M}x8192] [Wg,Wu][8192x5504] SwiGLU W2[2752x8192] bf16"
        elif kind == "gpt3_attn_gen":
            # token generation (Fig. 2b): one new token per sequence over `cached` earlier ones
            c = inputs.CFG4; self.mid = ds.MID_CAUSAL_ATTN
            nb = batch if batch <= 8 else 4
            self.M = M = nb
            t = inputs.attention(M, c["K1"], c["heads"], c["d"], c["N2"])
            W1 = t["Wqkv"]; t["W2"] = t["Wo"]
            self.kv = inputs.kv_cache(nb, cached, c["heads"], c["d"])
            self.attn = dict(batch=nb, seq=1, heads=c["heads"], head_dim=c["d"])
            self.cache = dict(k_cache=self.kv["Kc"].cuda(), v_cache=self.kv["Vc"].cuda())
            self.name = (f"GPT-3 attention shard, token generation: X[{M}x12288] Wqkv[12288x4608] attention 12 heads x 128 "
                         f"over {cached} cached tokens (batch {nb}, 1 new token each) Wo[1536x12288] bf16")
        elif kind == "gpt3_attn":
            c = inputs.CFG4; self.mid = ds.MID_CAUSAL_ATTN
            t = inputs.attention(M, c["K1"], c["heads"], c["d"], c["N2"])
            W1 = t["Wqkv"]; t["W2"] = t["Wo"]
            self.attn = dict(batch=1, seq=M, heads=c["heads"], head_dim=c["d"])
            self.name = (f"GPT-3 attention shard X[{M}x12288] Wqkv[12288x4608] causal attention 12 heads x 128 "
                         f"(batch 1, seq {M}) Wo[1536x12288] bf16")
        else:
            shape = dict(inputs.CFG1); self.M = M = shape["M"]; self.mid = ds.MID_GELU
            t = inputs.mlp(**shape); W1 = t["W1"]
            self.name = "cfg1 X[256x1024] W1[1024x4096] GeLU W2[4096x1024] bf16"
        self.t, self.W1 = t, W1
        self.X = t["X"].cuda()
        self.W1t = W1.t().contiguous().cuda()
        self.W2t = t["W2"].t().contiguous().cuda()
        n1 = self.W1t.shape[0] // 2 if self.mid == ds.MID_SWIGLU else self.W1t.shape[0]
        self.H = torch.empty((M, n1), dtype=self.X.dtype, device="cuda")
        self.Y = torch.empty((M, self.W2t.shape[0]), dtype=self.X.dtype, device="cuda")
        if w_layout == "kblocked":      # weights are static: packed once, outside every timed region
            self.W1t, self.W2t = ds.pack_weights_kblocked(self.W1t), ds.pack_weights_kblocked(self.W2t)
            self.name += ", weights K-blocked"
        self.extra = {}
        if self.attn:
            self.extra = dict(self.attn, T=torch.empty((M, self.attn["heads"] * self.attn["head_dim"]),
                                                       dtype=self.X.dtype, device="cuda"))
            self.extra.update(getattr(self, "cache", {}))
        self.policies = ["row", "tile", "strided"] if self.attn else ["row", "tile"]

    def plan(self, pol, tile=0):
        ds = self.ds
        if self.convn:
            return ds.conv_chain_n_plan(self.x, self.ws, self.outs, pol, tile=tile)
        if self.conv:
            return ds.conv_chain_plan(self.x, self.w1, self.mid_t, self.w2, self.out, pol, tile=tile)
        return ds.gemm_chain_plan(self.X, self.W1t, self.H, self.W2t, self.Y, pol, mid=self.mid, tile=tile, **self.extra)

    def autotune(self, pol, sp):
        ds = self.ds
        if self.convn:
            return ds.conv_chain_n_autotune(self.x, self.ws, self.outs, pol, stream=sp, reps=3)
        if self.conv:
            return ds.conv_chain_autotune(self.x, self.w1, self.mid_t, self.w2, self.out, pol, stream=sp, reps=3)
        return ds.gemm_chain_autotune(self.X, self.W1t, self.H, self.W2t, self.Y, pol, mid=self.mid, stream=sp,
                                      reps=3, **self.extra)

    def caller(self, pol, mode, tile, sp, sc):
        ds = self.ds
        if self.convn:
            def call():
                ds.dep_conv_chain_n(self.x, self.ws, self.outs, pol, mode=mode, tile=tile,
                                    stream_producer=sp, stream_consumer=sc)
        elif self.conv:
            def call():
                ds.dep_conv_chain(self.x, self.w1, self.mid_t, self.w2, self.out, pol, mode=mode, tile=tile,
                                  stream_producer=sp, stream_consumer=sc)
        else:
            def call():
                ds.dep_gemm_chain(self.X, self.W1t, self.H, self.W2t, self.Y, pol, mode=mode, mid=self.mid, tile=tile,
                                  stream_producer=sp, stream_consumer=sc, **self.extra)
        return call

    def cpu_oracle(self, rows):
        """Run the fp64 oracle on a bounded sample; returns (seconds, fraction of the chain's flops, text)."""
        import inputs
        import oracle
        t = self.t
        if self.convn:
            B = t[0]["x"].shape[0]
            xs = inputs.to_f64(t[0]["x"][:1])
            wf = [inputs.to_f64(l["w1"]) for l in t]
            t0 = time.perf_counter()
            oracle.conv_chain_n(xs, wf)
            return time.perf_counter() - t0, 1.0 / B, f"fp64 oracle timed on the first of {B} images (images are independent)"
        if self.conv:
            B = t["x"].shape[0]
            xs = inputs.to_f64(t["x"][:1])
            w1, w2 = inputs.to_f64(t["w1"]), inputs.to_f64(t["w2"])
            t0 = time.perf_counter()
            oracle.conv_chain(xs, w1, w2)
            return time.perf_counter() - t0, 1.0 / B, f"fp64 oracle timed on the first of {B} images (images are independent)"
        rows = min(rows, self.M)
        Xs = inputs.to_f64(t["X"][:rows])
        W1f, W2f = inputs.to_f64(self.W1), inputs.to_f64(t["W2"])
        t0 = time.perf_counter()
        if self.attn and hasattr(self, "kv"):
            rows = self.M
            oracle.attn_chain_cached(inputs.to_f64(t["X"]), W1f, W2f, inputs.to_f64(self.kv["Kc"]), inputs.to_f64(self.kv["Vc"]),
                                     self.attn["batch"], 1, self.attn["heads"], self.attn["head_dim"])
        elif self.attn:
            # causal: the first `rows` tokens of the sequence need nothing from later tokens
            oracle.attn_chain(Xs, W1f, W2f, 1, rows, self.attn["heads"], self.attn["head_dim"])
        elif self.mid == self.ds.MID_SWIGLU:
            oracle.swiglu_chain(Xs, W1f, W2f)
        else:
            oracle.gemm_chain(Xs, W1f, W2f, oracle.ACT_GELU)
        dt = time.perf_counter() - t0
        why = "rows are independent" + (", the attention of a prefix being a prefix of the attention" if self.attn else "")
        return dt, rows / self.M, f"fp64 oracle timed on the first {rows} of {self.M} rows of X ({why})"


def trace_occupancy(ds, torch, wl, kind, mode, tile, sp, sc, n_tiles, slots):
    """Slot utilisation of one chain and occupancy of its final wave, from the per-tile trace
    (None, None when the chain has more tiles than the trace holds)."""
    if n_tiles > 8192:
        return None, None
    pol = ds.SyncPolicy(kind, flags=ds.FLAG_TRACE)
    call = wl.caller(pol, mode, tile, sp, sc)
    for _ in range(3):
        call()
    torch.cuda.synchronize()
    recs = pol.read_trace(n_tiles)
    pol.destroy()
    t0 = min(r.t_enter for r in recs)
    t1 = max(r.t_end for r in recs)
    busy = sum(r.t_end - r.t_ready for r in recs)
    util = busy / (slots * max(t1 - t0, 1))
    last = recs[-(n_tiles // 4 or 1):]
    dur = sorted(r.t_end - r.t_ready for r in last)[len(last) // 2]        # median tile of the last stage
    lo = t1 - dur
    final = sum(max(0, min(r.t_end, t1) - max(r.t_ready, lo)) for r in recs) / (slots * max(dur, 1))
    return util, final


def measure(args, torch, ds, wl, sp, sc, want, pol_names=None, tile=0, autotune=True):
    kinds = {"row": ds.ROWSYNC, "tile": ds.TILESYNC, "strided": ds.STRIDEDSYNC}
    modes = {"fine": ds.MODE_FINE, "fused": ds.MODE_FUSED, "streamsync": ds.MODE_STREAMSYNC, "plain": ds.MODE_PLAIN}
    pol_names = pol_names or wl.policies
    # Every (policy, launch mode) variant is warmed up, then timed in `rounds` interleaved blocks of
    # `steps` launches (the chip's clock follows its power and temperature history, so variants
    # timed one after the other are not comparable); a variant's latency is the median of its blocks.
    pols = {pn: ds.SyncPolicy(kinds[pn]) for pn in pol_names}
    pols_hw = {pn: ds.SyncPolicy(kinds[pn], flags=ds.FLAG_HW_ORDER) for pn in pol_names} if "fused_hw" in want else {}
    if tile == 0 and autotune:
        # outside the timed region: let the library time its macro-tile shapes on this chain once
        for pn in pol_names:
            wl.autotune(pols[pn], sp)
    variants = [(pn, mn) for pn in pol_names for mn in want
                if mn in ("fine", "fused") or pn == pol_names[0]]   # stream-sync / plain / block-index order: first policy only
    modes["fused_hw"] = ds.MODE_FUSED
    calls = {(pn, mn): wl.caller(pols_hw[pn] if mn == "fused_hw" else pols[pn], modes[mn], tile, sp, sc) for pn, mn in variants}
    for v in variants:
        for _ in range(args.warmup):
            calls[v]()
    if tile != 0 or not autotune:
        # The autotuner's runs also bring the chip out of its idle clocks; without them, keep it
        # busy for a tenth of a second first (measured: an HBM-bound conv pair reads 4x slower,
        # the GeMM chains 4-20 % slower, when timed cold), still outside the timed region.
        torch.cuda.synchronize()
        t_busy = time.perf_counter()
        while time.perf_counter() - t_busy < 0.1:
            for v in variants:
                calls[v]()
            torch.cuda.synchronize()
    blocks = {v: [] for v in variants}
    for _ in range(args.rounds):
        for v in variants:
            blocks[v].append(time_block(torch, calls[v], sp, args.steps))
    results = {v: sorted(b)[len(b) // 2] for v, b in blocks.items()}
    # the fine-grained variants: two streams (FINE) or one dispatch (FUSED), per policy
    fine = {v: results[v] for v in variants if v[1] in ("fine", "fused")}
    best = min(fine, key=fine.get) if fine else variants[0]
    # the headline: W warm-up launches, then exactly K timed launches of the best variant
    for _ in range(args.warmup):
        calls[best]()
    lat = time_block(torch, calls[best], sp, args.steps)
    best_plan = wl.plan(pols[best[0]], tile)
    for pol in list(pols.values()) + list(pols_hw.values()):
        pol.status()
        pol.destroy()
    return dict(plan=best_plan, results=results, blocks=blocks, best=best, lat=lat, kinds=kinds, modes=modes,
                ss=results.get((pol_names[0], "streamsync")), plain=results.get((pol_names[0], "plain")),
                hw=results.get((pol_names[0], "fused_hw")))


def roofline(plan, lat_us):
    flops, nbytes = plan.flops, plan.bytes
    tflops = flops / (lat_us * 1e-6) / 1e12
    if (nbytes / 8e12) > (flops / (PEAK_BF16_TFLOPS * 1e12)):
        roof = {"bound": "hbm", "achieved": nbytes / (lat_us * 1e-6) / 1e9, "peak": 8000.0, "unit": "GB/s"}
    else:
        roof = {"bound": "mfma", "achieved": tflops, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s"}
    roof["frac"] = roof["achieved"] / roof["peak"]
    return roof, tflops


def tile_label(ds, tile):
    """'128x192', or '128x192 deep' for the shapes that also exist with a 4- or 8-stage operand pipeline."""
    tm, tn = ds.tile_shape(tile)
    deep = tile in (ds.TILE_64x64_DEEP, ds.TILE_128x192_DEEP, ds.TILE_128x128_DEEP)
    return f"{tm}x{tn}" + (" deep" if deep else "")


def sweep(args, torch, ds, inputs):
    """All configurations -> markdown table."""
    sp, sc = torch.cuda.Stream(), torch.cuda.Stream()
    if args.sweep_set == "resnet":
        # the paper's second conv workload (Fig. 7): ResNet-38's pairs of 3x3 convolutions, 56x56x64 ... 7x7x512
        cases = [("resnet_conv", dict(hw=hw, channels=ch, batch=b))
                 for hw, ch in ((56, 64), (28, 128), (14, 256), (7, 512)) for b in (1, 8, 32)]
    elif args.sweep_set == "generation":
        # token generation with cached keys and values: S = 1, S' in {512, 2048}, B in {1, 4} (Section V)
        cases = [("gpt3_attn_gen", dict(batch=b, cached=c)) for b in (1, 4) for c in (512, 2048)]
    elif args.sweep_set == "vgg_layers":
        # chains of four convolutions: VGG-19's layer groups at 256 and 512 channels (Section V)
        cases = [("vgg_layer", dict(hw=hw, channels=ch, batch=b)) for hw, ch in ((56, 256), (28, 512), (14, 512)) for b in (1, 16)]
    else:
        cases = [("cfg1", dict())]
        cases += [("gpt3_mlp", dict(M=m)) for m in inputs.CFG2["Ms"]]
        cases += [("llama_mlp", dict(M=m)) for m in inputs.CFG3["Ms"]]
        # the weight-streaming sizes once more with the weights packed K-blocked (a static, one-off repack)
        cases += [("gpt3_mlp", dict(M=m, w_layout="kblocked")) for m in inputs.CFG2["Ms"] if m <= 64]
        cases += [("llama_mlp", dict(M=m, w_layout="kblocked")) for m in inputs.CFG3["Ms"] if m <= 64]
        cases += [("gpt3_attn", dict(M=m)) for m in inputs.CFG4["Ms"]]
        cases += [("vgg_conv", dict(hw=hw, channels=ch, batch=b)) for hw, ch in inputs.CFG5["stages"] for b in (1, 16)]
    lines = ["| workload | tile | P / (mid) / C tiles | slots | waves ss / fine | best fine-grained us (policy/launch) | two streams us | "
             "stream-sync us | plain us | block-index order us | speedup vs ss | vs plain | TFLOP/s | roofline | slot util. | final wave |",
             "|---|---|---|---|---|---|---|---|---|---|---|---|---|---|---|---|"]
    fmt = lambda v: "-" if v is None else f"{v:.2f}"
    for kind, kw in cases:
        wl = Workload(torch, ds, inputs, kind, **kw)
        r = measure(args, torch, ds, wl, sp, sc, ["fine", "fused", "fused_hw", "streamsync", "plain"], autotune=not args.no_autotune)
        plan, lat = r["plan"], r["lat"]
        two = min(v for (pn, mn), v in r["results"].items() if mn == "fine")
        roof, tflops = roofline(plan, lat)
        n_tiles = plan.n_prod + plan.n_mid + plan.n_cons
        util, final = trace_occupancy(ds, torch, wl, r["kinds"][r["best"][0]], r["modes"][r["best"][1]], 0, sp, sc,
                                      n_tiles, plan.slots)
        mid = f" / {plan.n_mid}" if plan.n_mid else ""
        lines.append(
            f"| {wl.name} | {tile_label(ds, plan.tile_prod)} | {plan.n_prod}{mid} / {plan.n_cons} | {plan.slots} | "
            f"{plan.waves_streamsync} / {plan.waves_fine} | {lat:.1f} ({r['best'][0]}/{r['best'][1]}) | {two:.1f} | {r['ss']:.1f} | "
            f"{r['plain']:.1f} | {r['hw']:.1f} | {r['ss'] / lat:.3f} | {r['plain'] / lat:.3f} | {tflops:.0f} | "
            f"{roof['bound']} {100 * roof['frac']:.1f} % | {fmt(util)} | {fmt(final)} |")
        print(lines[-1], file=sys.stderr, flush=True)
        del wl
        torch.cuda.empty_cache()
    with open(args.sweep, "w") as f:
        f.write("\n".join(lines) + "\n")
    print(json.dumps({"sweep": args.sweep, "rows": len(lines) - 2}))


def policy_table(args, torch, ds, inputs):
    """For every GeMM-chain size of the paper: run the library's policy search (each kind autotuned, fastest
    remembered), then time each kind and an AUTOSYNC policy in interleaved blocks, one dispatch per chain."""
    sp, sc = torch.cuda.Stream(), torch.cuda.Stream()
    kinds = [("row", ds.ROWSYNC), ("tile", ds.TILESYNC), ("strided", ds.STRIDEDSYNC)]
    cases = [("gpt3_mlp", dict(M=m)) for m in inputs.CFG2["Ms"]]
    cases += [("llama_mlp", dict(M=m)) for m in inputs.CFG3["Ms"]]
    cases += [("gpt3_attn", dict(M=m)) for m in inputs.CFG4["Ms"]]
    lines = ["| workload | Row us (tile) | Tile us (tile) | Strided us (tile) | search keeps | AUTOSYNC us | waits per chain Row / Tile |",
             "|---|---|---|---|---|---|---|"]
    for kind, kw in cases:
        wl = Workload(torch, ds, inputs, kind, **kw)
        auto = ds.SyncPolicy(ds.AUTOSYNC)
        kept, kept_tile, _ = ds.gemm_chain_autotune_policy(wl.X, wl.W1t, wl.H, wl.W2t, wl.Y, auto, mid=wl.mid, stream=sp, **wl.extra)
        pols, calls, tiles = {}, {}, {}
        for pn, k in kinds:
            if pn == "strided" and not wl.attn:
                continue
            pols[pn] = ds.SyncPolicy(k)
            tiles[pn] = wl.plan(pols[pn]).tile_prod          # the tile the search remembered for this kind
            calls[pn] = wl.caller(pols[pn], ds.MODE_FUSED, 0, sp, sc)
        pols["auto"] = auto
        calls["auto"] = wl.caller(auto, ds.MODE_FUSED, 0, sp, sc)
        for c in calls.values():
            for _ in range(args.warmup):
                c()
        blocks = {k: [] for k in calls}
        for _ in range(args.rounds):
            for k, c in calls.items():
                blocks[k].append(time_block(torch, c, sp, args.steps))
        med = {k: sorted(b)[len(b) // 2] for k, b in blocks.items()}
        waits = []
        for pn, k in kinds[:2]:                              # counted in one extra launch of a counting policy
            cp = ds.SyncPolicy(k, flags=ds.FLAG_COUNT)
            wl.caller(cp, ds.MODE_FUSED, 0, sp, sc)()
            torch.cuda.synchronize()
            waits.append(str(cp.status().waits))
            cp.destroy()
        cell = lambda pn: f"{med[pn]:.1f} ({tile_label(ds, tiles[pn])})" if pn in med else "-"
        names = {ds.ROWSYNC: "Row", ds.TILESYNC: "Tile", ds.STRIDEDSYNC: "Strided"}
        lines.append(f"| {wl.name} | {cell('row')} | {cell('tile')} | {cell('strided')} | {names[kept]} ({tile_label(ds, kept_tile)}) | "
                     f"{med['auto']:.1f} | {' / '.join(waits)} |")
        print(lines[-1], file=sys.stderr, flush=True)
        for pol in pols.values():
            pol.destroy()
        del wl
        torch.cuda.empty_cache()
    with open(args.policy_table, "w") as f:
        f.write("\n".join(lines) + "\n")
    print(json.dumps({"policy_table": args.policy_table, "rows": len(lines) - 2}))


def ablation(args, torch, ds, wl):
    """Latency of the workload under each launch mode and with the paper's optimisations (Section IV-C:
    load/wait reordering, custom tile order) switched off, interleaved blocks, markdown table."""
    sp, sc = torch.cuda.Stream(), torch.cuda.Stream()
    kinds = {"row": ds.ROWSYNC, "tile": ds.TILESYNC, "strided": ds.STRIDEDSYNC}
    modes = {"fine": ds.MODE_FINE, "fused": ds.MODE_FUSED, "streamsync": ds.MODE_STREAMSYNC, "plain": ds.MODE_PLAIN}
    pols, calls, rows = [], {}, []
    tuner = ds.SyncPolicy(kinds[wl.policies[0]])
    tile = args.tile or wl.autotune(tuner, sp)          # one tile shape for every row of the table
    tuner.destroy()
    for pn in wl.policies:
        # "one dispatch" here means persistent workgroups drawing from the dispatch queues, so that
        # the last row of each group isolates the block-index order
        for label, flags, mn in ((f"{pn}, one dispatch", ds.FLAG_QUEUE_ORDER, "fused"), (f"{pn}, two streams", 0, "fine"),
                                 (f"{pn}, one dispatch, wait before the weights are requested",
                                  ds.FLAG_NO_REORDER | ds.FLAG_QUEUE_ORDER, "fused"),
                                 (f"{pn}, one dispatch, one workgroup per tile in hardware order", ds.FLAG_HW_ORDER, "fused")):
            pol = ds.SyncPolicy(kinds[pn], flags=flags)
            pols.append(pol)
            calls[label] = wl.caller(pol, modes[mn], tile, sp, sc)
    base = ds.SyncPolicy(kinds[wl.policies[0]])
    pols.append(base)
    calls["stream sync (same kernels, one stream)"] = wl.caller(base, modes["streamsync"], tile, sp, sc)
    calls["plain (hooks compiled out)"] = wl.caller(base, modes["plain"], tile, sp, sc)
    ok = {}
    for k, c in calls.items():
        try:
            for _ in range(args.warmup):
                c()
            torch.cuda.synchronize()
            ok[k] = c
        except ds.DepsyncError as e:                     # e.g. hardware order with more tiles than slots
            rows.append(f"| {k} | not run: {e} |")
    blocks = {k: [] for k in ok}
    for _ in range(args.rounds):
        for k, c in ok.items():
            blocks[k].append(time_block(torch, c, sp, args.steps))
    for k, b in blocks.items():
        rows.append(f"| {k} | {sorted(b)[len(b) // 2]:.1f} |")
    for pol in pols:
        pol.destroy()
    tm, tn = ds.tile_shape(tile)
    with open(args.ablation, "w") as f:
        f.write(f"{wl.name}, macro-tile {tm}x{tn}\n\n| variant | chain latency (us) |\n|---|---|\n" + "\n".join(rows) + "\n")
    print(json.dumps({"ablation": args.ablation, "rows": len(rows)}))


def sync_overhead(args, torch, ds, n_cu):
    """The copy -> copy chain: what post, wait and the dispatch queues cost when the tiles do nothing
    but move bytes.  One full wave of tiles (CUs x 8 workgroups) and four waves, tile sizes 16 KiB to
    1 MiB, every launch mode, tiles named by the block index or drawn from the dispatch queues;
    interleaved blocks, median block."""
    import oracle
    sp, sc = torch.cuda.Stream(), torch.cuda.Stream()
    slots = n_cu * 8
    variants = [   # label, policy kind, flags, mode, counts as fine-grained
        ("TileSync, one dispatch, block-index order", ds.TILESYNC, ds.FLAG_HW_ORDER, ds.MODE_FUSED, True),
        ("TileSync, one dispatch, queues", ds.TILESYNC, 0, ds.MODE_FUSED, True),
        ("TileSync, two streams, queues", ds.TILESYNC, 0, ds.MODE_FINE, True),
        ("RowSync, one dispatch, block-index order", ds.ROWSYNC, ds.FLAG_HW_ORDER, ds.MODE_FUSED, True),
        ("stream sync, block-index order", ds.TILESYNC, ds.FLAG_HW_ORDER, ds.MODE_STREAMSYNC, False),
        ("stream sync, queues", ds.TILESYNC, 0, ds.MODE_STREAMSYNC, False),
        ("plain", ds.TILESYNC, 0, ds.MODE_PLAIN, False),
    ]
    rows, headline = [], None
    for waves in (1, 4):
        for tile_kib in (16, 64, 256, 1024):
            tiles = slots * waves
            n = tiles * tile_kib * 1024
            if n > (2 << 30):
                continue
            src = torch.empty(n, dtype=torch.uint8, device="cuda").random_(0, 256)
            mid, dst = torch.empty_like(src), torch.empty_like(src)
            pols, calls = [], {}
            for label, kind, flags, mode, _ in variants:
                pol = ds.SyncPolicy(kind, flags=flags)
                pols.append(pol)
                def call(pol=pol, mode=mode):
                    ds.dep_copy_chain(src, mid, dst, pol, mode=mode, tile_bytes=tile_kib * 1024,
                                      stream_producer=sp, stream_consumer=sc)
                for _ in range(args.warmup):
                    call()
                calls[label] = call
            torch.cuda.synchronize()
            assert torch.equal(dst, src)
            blocks = {k: [] for k in calls}
            for _ in range(args.rounds):
                for k, c in calls.items():
                    blocks[k].append(time_block(torch, c, sp, args.steps))
            med = {k: sorted(b)[len(b) // 2] for k, b in blocks.items()}
            fine = min(med[v[0]] for v in variants if v[4])
            ss = min(med["stream sync, block-index order"], med["stream sync, queues"])
            plain = med["plain"]
            rows.append(f"| {waves} | {tile_kib} KiB | {tiles} | {n >> 20} MiB | " + " | ".join(f"{med[v[0]]:.1f}" for v in variants) +
                        f" | {100 * (fine / plain - 1):+.1f} % | {100 * (fine / ss - 1):+.1f} % | {4.0 * n / fine * 1e-3:.0f} |")
            if waves == 1 and tile_kib == 64:
                headline = dict(n=n, tiles=tiles, med=med, plain=plain, ss=ss)
                h = src[: 64 << 20].cpu().numpy()
                t0 = time.perf_counter()
                oracle.copy_chain(h)
                cpu_s, cpu_bytes = time.perf_counter() - t0, h.size
            for pol in pols:
                pol.destroy()
            del src, mid, dst
    with open(args.sync_overhead, "w") as f:
        f.write("| waves | tile | tiles per stage | buffer | " + " | ".join(v[0] + (" (us)" if i == 0 else "") for i, v in enumerate(variants)) +
                " | best fine-grained vs plain | vs best stream sync | GB/s (best fine-grained) |\n" +
                "|" + "---|" * (len(variants) + 7) + "\n" + "\n".join(rows) + "\n")
    m = headline["med"]
    best = min((v[0] for v in variants if v[4]), key=lambda k: m[k])
    lat = m[best]
    n = headline["n"]
    out = {
        "metric": "dependent-chain latency, fine-grained sync, best of {two-stream, one-dispatch} x sync policies (median block)",
        "value": lat, "unit": "us", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": lat / 1e3,
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "u8", "data": "synthetic",
        "config": {"workload": f"copy -> copy chain, {headline['tiles']} tiles of 64 KiB per stage (one full wave of {n_cu} CUs x 8 "
                               f"workgroups), consumer tile i waits for producer tile i", "variant": best},
        "latency_us": {k: round(v, 2) for k, v in m.items()},
        "overhead_vs_plain_pct": 100 * (lat / headline["plain"] - 1),
        "speedup_vs_streamsync": headline["ss"] / lat,
        "roofline": {"bound": "hbm", "achieved": 4.0 * n / lat * 1e-3, "peak": 8000.0, "unit": "GB/s",
                     "frac": 4.0 * n / lat * 1e-3 / 8000.0, "traffic": None,
                     "kernel": "copy_chain_kernel (both stages; one dispatch in fused mode)",
                     "per_launch": {"bytes": 4.0 * n, "duration_us": lat}},
        "cpu_baseline": {"value": cpu_s * 1e6 * n / cpu_bytes, "unit": "us", "cores": 1, "kind": "oracle",
                         "sample": f"oracle copy chain timed on the first {cpu_bytes >> 20} MiB ({cpu_s:.3f} s), scaled to the buffer"},
        "table": args.sync_overhead,
    }
    print(json.dumps(out))


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
    if args.sweep:
        return sweep(args, torch, ds, inputs)
    if args.sync_overhead:
        return sync_overhead(args, torch, ds, n_cu)
    if args.policy_table:
        return policy_table(args, torch, ds, inputs)

    wl = Workload(torch, ds, inputs, args.workload, M=args.m, hw=args.hw, channels=args.channels, batch=args.batch,
                  w_layout=args.w_layout, cached=args.cached)
    M = wl.M

    if args.copy_calibration:
        src = torch.empty(args.copy_calibration << 20, dtype=torch.uint8, device="cuda").random_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    if args.ablation:
        return ablation(args, torch, ds, wl)

    sp, sc = torch.cuda.Stream(), torch.cuda.Stream()
    pol_names = wl.policies if args.policy == "auto" else [args.policy]
    want = [m for m in args.modes.split(",") if m]
    r = measure(args, torch, ds, wl, sp, sc, want, pol_names, tile=args.tile, autotune=not args.no_autotune)
    plan, lat, results, blocks = r["plan"], r["lat"], r["results"], r["blocks"]
    best_pol, best_mode = r["best"]
    ss, plain = r["ss"], r["plain"]
    roof, tflops = roofline(plan, lat)
    default_shape = args.w_layout == "rows" and (args.workload != "vgg_conv" or (args.hw, args.channels, args.batch) == (56, 256, 16))
    roof["traffic"] = MEASURED_TRAFFIC_BYTES.get((args.workload, M, best_mode)) if default_shape else None
    roof["traffic_source"] = ("rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of this command, recorded in profiles/ "
                              "(a constant from that run, not measured in this one)") if roof["traffic"] else None
    roof["kernel"] = "chain_kernel (all dispatches of one chain; one dispatch in fused mode)"
    roof["per_launch"] = {"flops": plan.flops, "bytes": plan.bytes, "duration_us": lat}
    n_tiles = plan.n_prod + plan.n_mid + plan.n_cons
    util, final = trace_occupancy(ds, torch, wl, r["kinds"][best_pol], r["modes"][best_mode], args.tile, sp, sc,
                                  n_tiles, plan.slots)

    out = {
        "metric": "dependent-chain latency, fine-grained sync, best of {two-stream, one-dispatch} x sync policies (mean of steps)",
        "value": lat, "unit": "us", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": lat / 1e3, "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": wl.name, "M": M, "policy": best_pol, "launch": best_mode,
                   # tile order of the headline variant: the library draws tiles from its dispatch queues (producer tiles
                   # always handed out first) unless every tile has a resident workgroup of its own
                   "order": "block index" if n_tiles <= plan.slots else "dispatch queues",
                   "tile": ds.tile_shape(plan.tile_prod),
                   "tile_name": tile_label(ds, plan.tile_prod),
                   "tiles_producer": plan.n_prod, "tiles_middle": plan.n_mid, "tiles_consumer": plan.n_cons,
                   "slots": plan.slots, "waves_streamsync": plan.waves_streamsync, "waves_fine": plan.waves_fine},
        "latency_us": {f"{pn}/{mn}": round(v, 2) for (pn, mn), v in results.items()},
        "latency_blocks_us": {f"{pn}/{mn}": [round(x, 1) for x in b] for (pn, mn), b in blocks.items()},
        "speedup_vs_streamsync": (ss / lat) if ss else None,
        "speedup_vs_plain": (plain / lat) if plain else None,
        # the same chain in one dispatch with tiles named by the block index (DEPSYNC_FLAG_HW_ORDER): faster by the cost of
        # the draws, but progress then rests on in-order workgroup start per XCD, so it is reported and never the headline
        "block_index_order_us": r["hw"],
        "tflops": tflops, "pct_bf16_mfma_peak": 100 * tflops / PEAK_BF16_TFLOPS,
        "slot_utilisation": util, "final_wave_occupancy": final,
        "device": {"cus": n_cu, "clock_mhz": clock_khz / 1e3},
        "roofline": roof,
    }

    if args.mfma_calibration:
        # after the chain, so that the chip is warm; random operands last
        zero = ds.mfma_calibration(True, args.mfma_calibration)
        rnd = ds.mfma_calibration(False, args.mfma_calibration)
        # a loop that issues an MFMA every cycle it can: TFLOP/s / (CUs x 4096 flop/clk) is the clock it ran at
        per_clk = n_cu * 4096.0
        out["mfma_calibration"] = {"zero_operands_tflops": zero, "random_operands_tflops": rnd,
                                   "implied_clock_mhz_zero": zero * 1e6 / per_clk, "implied_clock_mhz_random": rnd * 1e6 / per_clk,
                                   "chain_vs_random_ceiling": tflops / rnd if rnd else None}

    if not args.no_cpu_baseline:
        import oracle
        dt, frac, what = wl.cpu_oracle(args.cpu_rows)
        out["cpu_baseline"] = {
            "value": dt * 1e6 / frac, "unit": "us", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"{what}; {dt:.2f} s measured, scaled by {1 / frac:.3g} to the full chain",
            "measured_s": dt, "gflops": plan.flops * frac / dt / 1e9,
        }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
