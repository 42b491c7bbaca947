#!/usr/bin/env python3
"""Benchmark of the SwiGLU MLP hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

Workload (the configuration the headline metric is quoted on): the
Llama-3-8B-shaped MLP layer, d_model=4096, d_ff=14336, bf16, at M in
{1, 2, 4, 8, 16}.  One "step" is one pass of the whole hot path over one batch
of synthetic input: one dfk_swiglu_mlp call for each M of the set, each call on
the next of several distinct weight sets (so weights stream from HBM, never
from the 256 MB last-level cache).  Inputs are seeded synthetic tensors,
resident in HBM before the timed region.  Before timing, the profile-driven
scheduler tunes the (variant, tile) choice per M - the pre-inference step of
the method - and its picks (single launch or two kernels, per M) are named in
`metric` and `config`.

Prints ONE JSON line: value = mean microseconds per call over the step's
calls.  roofline = algorithmic HBM bytes per call / the duration of the call's
launches, against the 8 TB/s peak: `frac` is the whole call (what the target is
stated on); the call's dominant launch (the whole block where the single launch
is picked, else the gate/up kernel, two of the three matrices) is in
`roofline.dominant_kernel`, timed with HIP events around back-to-back launches
of that kernel alone.  Beside the headline: the same statistics (4 repeats x 50
launches) for every M up to 64 and a second mean over M = 1..64, 128 and 256
tokens, the other layer shapes of the workload list, and the 32-layer decode
pass replayed from a HIP graph.  cpu_baseline = the fp64 oracle on the host
cores over steps of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

D_MODEL, D_FF = 4096, 14336
M_SET = (1, 2, 4, 8, 16)
WEIGHT_SETS = 4
HBM_PEAK_GBS = 8000.0


def algorithmic_bytes(M, d_model, d_ff):
    """Three bf16 weight matrices read once + X read + Y written."""
    return 6 * d_model * d_ff + 2 * M * d_model + 2 * M * d_model


def committed_traffic():
    """HBM bytes per call (fetched + written, every launch of the call) from the committed rocprofv3 counter
    summary (FETCH_SIZE + WRITE_SIZE runs of this script; counters cannot be read from inside it): the mean over
    the headline token counts, and the dominant launch's share."""
    path = os.path.join(ROOT, "profiles", "dfk_llama3_8b_hbm_traffic.md")
    try:
        import re
        txt = open(path).read()
        call = re.search(r"hbm_bytes_per_call\s*=\s*(\d+)", txt)
        dom = re.search(r"dominant_kernel_hbm_bytes_per_launch\s*=\s*(\d+)", txt)
        return (int(call.group(1)) if call else None, int(dom.group(1)) if dom else None,
                "profiles/dfk_llama3_8b_hbm_traffic.md")
    except OSError:
        return None, None, None


def variant_name(variant, kmajor):
    """What ran, in words: the two single-launch kernels differ in where A_2 lives."""
    if variant == 2:
        return "two kernels"
    if kmajor == 4:
        return "single launch (both kernels' workgroups, A_2 through device memory)"
    if kmajor == 1:
        return "single launch (fused, A_2 in LDS)"
    return "single launch (fused)"


def stats_4x50(torch, np, fn, n_sets):
    """The paper's protocol: 4 repeats (after one untimed) of 50 launches, HIP events on the launch stream."""
    reps = []
    for rep in range(-1, 4):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for i in range(50):
            fn((rep + i) % n_sets)
        b.record()
        torch.cuda.synchronize()
        if rep >= 0:
            reps.append(a.elapsed_time(b) * 1e3 / 50)
    return {"mean_us": round(float(np.mean(reps)), 2), "std_us": round(float(np.std(reps)), 2),
            "median_us": round(float(np.median(reps)), 2)}


def decode32(args, torch, di, dfk, dev, compact=False):
    """The decode sweep: 32 distinct layers of the headline shape (11.3 GB of weights, far beyond
    any cache) chained in stream order with a weight-free RMS normalisation between them, the
    whole pass captured once in a HIP graph and replayed (the method's deployment mode: the
    scheduler's choice is baked into the graph, no dispatch cost per token).  A layer's time
    includes its normalisation launch (one small kernel)."""
    L = 32
    sweep = (1, 4, 16, 64, 256) if compact else (1, 2, 3, 4, 8, 16, 24, 32, 64, 128, 256)
    layers = [di.mlp_inputs_torch(1, D_MODEL, D_FF, seed=1000, layer=l, device=dev) for l in range(L)]
    ws = dfk.new_workspace(max(sweep), D_MODEL, D_FF, dev)
    dfk.dfk_set_workspace(ws)
    if not compact:      # (the compact form runs on the table the headline workload has tuned)
        scratch = torch.empty(dfk.dfk_tune_scratch_bytes(max(sweep), D_MODEL, D_FF, dfk.DFK_BF16, 3),
                              dtype=torch.uint8, device=dev)
        dfk.dfk_tune(list(sweep), D_MODEL, D_FF, dfk.DFK_BF16, scratch, sets=3, iters=8)
        torch.cuda.synchronize()
        del scratch
    rows = {}
    for M in sweep:
        X0 = di.mlp_inputs_torch(M, D_MODEL, D_FF, seed=0, layer=0, device=dev)["X"]
        bufs = [torch.empty_like(X0) for _ in range(L + 1)]
        ys = [torch.empty_like(X0) for _ in range(L)]

        def chain(stream=None):
            for l in range(L):
                w = layers[l]
                dfk.dfk_swiglu_mlp(bufs[l], w["Wg"], w["Wu"], w["Wd"], ys[l], stream=stream)
                dfk.dfk_rms_normalize(ys[l], bufs[l + 1], stream=stream)

        bufs[0].copy_(X0)
        chain()                                    # eager: kernel attributes get set, result to compare with
        torch.cuda.synchronize()
        eager0 = ys[0].clone()
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                chain(stream=side)
        ok = True
        for _ in range(3):
            ys[0].zero_()
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            # layer 0 sees the same input every time (later layers amplify the last-bit freedom
            # of the atomic reduction, so only their finiteness is checked)
            d0 = float((eager0.float() - ys[0].float()).abs().max() / eager0.float().abs().max())
            ok = ok and d0 <= 1e-2 and bool(torch.isfinite(bufs[L].float()).all())
        reps = max(3, args.steps // 20)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            graph.replay()
        b.record()
        torch.cuda.synchronize()
        us_layer = a.elapsed_time(b) * 1e3 / reps / L
        c, tuned = dfk.dfk_get_choice(M, D_MODEL, D_FF, dfk.DFK_BF16)
        rows[str(M)] = {"us_per_layer_in_graph": round(us_layer, 2),
                        "tb_per_s": round(algorithmic_bytes(M, D_MODEL, D_FF) / us_layer / 1e6, 3),
                        "replays_match_eager_layer0": ok, "variant": variant_name(c.variant, c.kmajor),
                        "pick": dict(c.as_dict(), tuned=tuned)}
        del graph
    out = {"workload": "decode32: 32 chained llama3-8b-shaped layers, HIP graph replay; a layer's time includes "
                       "the weight-free normalisation launch between layers", "layers": L,
           "weights_gb": round(L * 6 * D_MODEL * D_FF / 1e9, 2), "per_M": rows}
    dfk.dfk_set_workspace(None)
    del layers, ws
    torch.cuda.empty_cache()
    if compact:
        return out
    print(json.dumps(out))


def block32(args, torch, di, dfk, dev):
    """The block with its neighbours in a pre-norm decoder layer, 32 distinct layers chained and
    replayed from a HIP graph: H <- H + MLP(RMSNorm(H; w_l)).  Per token count: the one
    call that folds normalisation and residual add into the block's two launches, the same
    arithmetic as separate launches around the plain block (a normalisation kernel without the
    weight, the block, an elementwise add), and the folded call with W_down as [d_model, d_ff]."""
    L = 32
    sweep = (1, 4, 16, 64, 256)
    eps = 1e-5
    layers = [di.mlp_inputs_torch(1, D_MODEL, D_FF, seed=1000, layer=l, device=dev) for l in range(L)]
    nws = [di.to_torch(di.tensor(5000 + l, (D_MODEL,), 1.0, "bf16"), dev) for l in range(L)]
    ws = dfk.new_workspace(max(sweep), D_MODEL, D_FF, dev)
    dfk.dfk_set_workspace(ws)
    scratch = torch.empty(dfk.dfk_tune_scratch_bytes(max(sweep), D_MODEL, D_FF, dfk.DFK_BF16, 3),
                          dtype=torch.uint8, device=dev)
    dfk.dfk_tune(list(sweep), D_MODEL, D_FF, dfk.DFK_BF16, scratch, sets=3, iters=8)
    torch.cuda.synchronize()
    del scratch
    rows = {}
    for M in sweep:
        X0 = di.mlp_inputs_torch(M, D_MODEL, D_FF, seed=0, layer=0, device=dev)["X"]
        bufs = [torch.empty_like(X0) for _ in range(L + 1)]
        xn, y = torch.empty_like(X0), torch.empty_like(X0)

        def folded(stream=None):
            for l in range(L):
                w = layers[l]
                dfk.dfk_mlp_block(bufs[l], nws[l], eps, w["Wg"], w["Wu"], w["Wd"], bufs[l + 1], None, ws, stream=stream)

        def separate(stream=None):
            for l in range(L):
                w = layers[l]
                dfk.dfk_rms_normalize(bufs[l], xn, stream=stream)
                dfk.dfk_swiglu_mlp(xn, w["Wg"], w["Wu"], w["Wd"], y, stream=stream)
                torch.add(bufs[l], y, out=bufs[l + 1])

        def folded_wdt(stream=None):     # the same weights read as W_down_t [d_model, d_ff]: the time does not depend on their values
            for l in range(L):
                w = layers[l]
                dfk.dfk_mlp_block_wdt(bufs[l], nws[l], eps, w["Wg"], w["Wu"], w["Wd"].view(D_MODEL, D_FF), bufs[l + 1], None, ws,
                                      stream=stream)

        row = {}
        chains = [("folded", folded), ("separate_launches", separate)]
        if M <= 64:
            chains.append(("folded_w_down_t_layout", folded_wdt))
        for name, chain in chains:
            bufs[0].copy_(X0)
            chain()
            torch.cuda.synchronize()
            eager1 = bufs[1].clone()
            side = torch.cuda.Stream()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.stream(side):
                with torch.cuda.graph(graph, stream=side):
                    chain(stream=side)
            ok = True
            for _ in range(3):
                bufs[1].zero_()
                torch.cuda.synchronize()
                graph.replay()
                torch.cuda.synchronize()
                d1 = float((eager1.float() - bufs[1].float()).abs().max() / eager1.float().abs().max())
                ok = ok and d1 <= 1e-2 and bool(torch.isfinite(bufs[L].float()).all())
            reps = max(3, args.steps // 20)
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(reps):
                graph.replay()
            b.record()
            torch.cuda.synchronize()
            us_layer = a.elapsed_time(b) * 1e3 / reps / L
            row[name] = {"us_per_layer_in_graph": round(us_layer, 2), "replays_match_eager_layer0": ok}
            del graph
        c, tuned = dfk.dfk_get_choice(M, D_MODEL, D_FF, dfk.DFK_BF16)
        row["pick"] = dict(c.as_dict(), tuned=tuned)
        rows[str(M)] = row
    print(json.dumps({"workload": "block32: 32 chained pre-norm MLP sub-blocks H + MLP(RMSNorm(H)), llama3-8b shape, "
                                  "HIP graph replay", "layers": L, "per_M": rows}))


def shapes(args, torch, di, dfk, dev, compact=False):
    """The other layer shapes of the workload list (parity-test configurations, timed here for the record):
    scheduler tuned per shape, one call per M on three rotating weight sets."""
    out = {}
    table = [("qwen2.5-32b-shaped", 5120, 27648, (1, 8, 32, 64)),
             ("llama3-70b-shaped", 8192, 28672, (1, 16, 64, 128)),
             ("llama3-70b tp4 shard", 8192, 7168, (1, 16, 64))]
    if not compact:
        table += [# widths whose 128-k chunks do not divide evenly among the wavefronts
                  ("2304x9216 (gemma-2b-sized)", 2304, 9216, (1, 16, 64)),
                  ("3584x18944 (qwen2.5-7b-sized)", 3584, 18944, (1, 16, 64)),
                  # d_ff beyond 512 slices of 64 rows; 5.2 GB of weights per set
                  ("16384x53248 (405b-class)", 16384, 53248, (1, 16, 64, 128))]
    for name, d, ff, Ms in table:
        sets = [di.mlp_inputs_torch(1, d, ff, seed=2000, layer=l, device=dev) for l in range(3)]
        ws = dfk.new_workspace(max(Ms), d, ff, dev)
        scratch = torch.empty(dfk.dfk_tune_scratch_bytes(max(Ms), d, ff, dfk.DFK_BF16, 3), dtype=torch.uint8, device=dev)
        dfk.dfk_tune(list(Ms), d, ff, dfk.DFK_BF16, scratch, sets=3, iters=6)
        torch.cuda.synchronize()
        del scratch
        rows = {}
        for M in Ms:
            X = di.mlp_inputs_torch(M, d, ff, seed=0, layer=0, device=dev)["X"]
            Y = torch.empty_like(X)
            n = max(20, args.steps // 5)
            for it in range(-10, n):
                if it == 0:
                    torch.cuda.synchronize()
                    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    a.record()
                w = sets[it % 3]
                dfk.dfk_swiglu_mlp_ex(X, w["Wg"], w["Wu"], w["Wd"], Y, None, ws)
            b.record()
            torch.cuda.synchronize()
            us = a.elapsed_time(b) * 1e3 / n
            c, tuned = dfk.dfk_get_choice(M, d, ff, dfk.DFK_BF16)
            rows[str(M)] = {"us_per_call": round(us, 2), "tb_per_s": round(algorithmic_bytes(M, d, ff) / us / 1e6, 3),
                            "frac_of_8tbs": round(algorithmic_bytes(M, d, ff) / us / 1e6 / 8.0, 4),
                            "variant": variant_name(c.variant, c.kmajor), "pick": dict(c.as_dict(), tuned=tuned)}
            if M <= 16 and dfk.dfk_num_candidates_wdt(M, d, ff, dfk.DFK_BF16):
                # the same call with W_down as [d_model, d_ff] (the weights' values do not matter for the time)
                for it in range(-10, n):
                    if it == 0:
                        torch.cuda.synchronize()
                        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                        a.record()
                    w = sets[it % 3]
                    dfk.dfk_swiglu_mlp_wdt(X, w["Wg"], w["Wu"], w["Wd"].view(d, ff), Y, None, ws)
                b.record()
                torch.cuda.synchronize()
                us_t = a.elapsed_time(b) * 1e3 / n
                rows[str(M)]["w_down_t_layout"] = {"us_per_call": round(us_t, 2),
                                                   "frac_of_8tbs": round(algorithmic_bytes(M, d, ff) / us_t / 1e6 / 8.0, 4)}
        out[name] = {"d_model": d, "d_ff": ff, "per_M": rows}
        del sets, ws
        torch.cuda.empty_cache()
    res = {"workload": "shapes: other decode-shaped layers, bf16, scheduler tuned per shape, one call per M on "
                       "three rotating weight sets", "shapes": out}
    if compact:
        return res
    print(json.dumps(res))


def timeline(args, torch, di, dfk, dev):
    """Where the microseconds of a call go: the kernels' own time stamps (wall clock, 10 ns ticks, written by thread
    0 of every workgroup into the buffer given to dfk_set_trace_buffer) for one call of each kernel form on the
    headline shape, after warm-up calls on rotating weight sets; percentiles over the workgroups, in microseconds
    from the first workgroup's start."""
    import numpy as np
    d, ff = D_MODEL, D_FF
    forms = [
        ("single launch, A_2 in LDS (k_fused_local), atomic",
         dict(variant=1, kmajor=1, splits=256, waves=8, depth=3, reduce=1, k2_splits=0, k2_col_blocks=0),
         ((0, "start"), (2, "stage one streamed (wave 0)"), (3, "A_2 in LDS"), (4, "stage two streamed (wave 0)"),
          (5, "adds issued and drained"), (6, "arrived"), (7, "Y written (last workgroup)"))),
        ("single launch of both kernels' workgroups (k_roles_km), atomic; rows of the down workgroups follow those of the gate/up workgroups",
         dict(variant=1, kmajor=4, splits=256, waves=8, depth=4, reduce=1, k2_splits=16, k2_col_blocks=16),
         ((0, "gate/up start"), (2, "gate/up streamed (wave 0)"), (1, "A_2 stored"), (3, "down start"), (7, "down: wait over"),
          (4, "down streamed (wave 0)"))),
        ("same, counter reduction",
         dict(variant=1, kmajor=4, splits=256, waves=8, depth=4, reduce=0, k2_splits=16, k2_col_blocks=16),
         ((0, "gate/up start"), (1, "A_2 stored"), (3, "down start"), (7, "down: wait over"), (4, "down streamed (wave 0)"),
          (5, "partial sums published"), (6, "reduced / exit"))),
        ("two kernels (k_gateup_km, k_down_km), atomic",
         dict(variant=2, kmajor=1, splits=256, waves=8, depth=4, reduce=1, k2_splits=8, k2_col_blocks=32),
         ((0, "gate/up start"), (2, "gate/up streamed (wave 0)"), (1, "A_2 stored"), (3, "down start"), (4, "down streamed (wave 0)"))),
        ("same, counter reduction",
         dict(variant=2, kmajor=1, splits=256, waves=8, depth=4, reduce=0, k2_splits=8, k2_col_blocks=32),
         ((0, "gate/up start"), (1, "A_2 stored"), (3, "down start"), (4, "down streamed (wave 0)"), (5, "partial sums published"),
          (6, "reduced / exit"))),
    ]
    out = []
    for M in (1, 16):
        L = [di.mlp_inputs_torch(M, d, ff, seed=0, layer=l, device=dev) for l in range(3)]
        ws = dfk.new_workspace(M, d, ff, dev)
        for name, f, stamps in forms:
            c = dfk.dfk_config_t()
            c.path, c.a2_dtype, c.k2_rows_by_wave = dfk.DFK_PATH_MFMA, dfk.DFK_BF16, 0
            for k, v in f.items():
                setattr(c, k, v)
            if not dfk.dfk_config_valid(c, M, d, ff):
                continue
            tr = torch.zeros(1024 * 8, dtype=torch.int64, device=dev)
            Y = torch.empty_like(L[0]["X"])
            for i in range(6):
                w = L[i % 3]
                if i == 5:
                    tr.zero_()
                    dfk.dfk_set_trace_buffer(tr)
                dfk.dfk_swiglu_mlp_ex(w["X"], w["Wg"], w["Wu"], w["Wd"], Y, c, ws)
            torch.cuda.synchronize()
            dfk.dfk_set_trace_buffer(None)
            t = tr.cpu().numpy().reshape(-1, 8).astype(np.float64)
            t[t == 0] = np.nan
            us = (t - np.nanmin(t[:, 0])) / 100.0
            rows = {}
            for k, label in stamps:
                col = us[:, k]
                col = col[~np.isnan(col)]
                if col.size:
                    rows[label] = {"workgroups": int(col.size), "min": round(float(col.min()), 2),
                                   "p10": round(float(np.percentile(col, 10)), 2), "median": round(float(np.median(col)), 2),
                                   "p90": round(float(np.percentile(col, 90)), 2), "max": round(float(col.max()), 2)}
            out.append({"M": M, "form": name, "config": c.as_dict(), "us_from_first_start": rows})
        del L, ws
    print(json.dumps({"workload": "timeline: in-kernel time stamps of one call per kernel form, llama3-8b-shaped layer",
                      "note": "the stamps cost a little: a traced call runs about 1 us longer than an untraced one",
                      "timelines": out}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-tune", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="leave out the blocks beside the headline (other shapes, the 32-layer decode pass)")
    ap.add_argument("--tuning-file", default=None,
                    help="load the scheduler table from this file if it exists, else tune and save it there")
    ap.add_argument("--force", choices=["auto", "fused", "unfused"], default="auto")
    ap.add_argument("--workload", choices=["layer", "decode32", "block32", "shapes", "timeline"], default="layer",
                    help="layer (default): the headline workload; decode32: 32 chained distinct layers of the "
                         "same shape, captured once in a HIP graph and replayed, M swept 1..256; block32: the "
                         "same chain with RMS normalisation and residual add, folded into the block's launches "
                         "or as separate launches; shapes: the other layer shapes of the workload list; timeline: "
                         "the kernels' own time stamps of one call per kernel form")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU by design (one MI355X); run with --gpus 1. "
              "Values at more than one GPU are not produced.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import dfk_inputs as di
    import paper_2602_11808_amd as dfk

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.workload == "decode32":
        return decode32(args, torch, di, dfk, dev)
    if args.workload == "block32":
        return block32(args, torch, di, dfk, dev)
    if args.workload == "shapes":
        return shapes(args, torch, di, dfk, dev)
    if args.workload == "timeline":
        return timeline(args, torch, di, dfk, dev)
    M_WIDE = M_SET + (32, 64)            # the metric is quoted on M = 1..64; the target on M = 1..16
    M_ALL = M_WIDE + (128, 256)
    Mmax = max(M_ALL)

    # ---- synthetic inputs, resident in HBM
    layers = [di.mlp_inputs_torch(Mmax, D_MODEL, D_FF, seed=0, layer=l, device=dev)
              for l in range(WEIGHT_SETS)]
    X = {M: layers[0]["X"][:M].contiguous() for M in M_ALL}
    Y = {M: torch.empty_like(X[M]) for M in M_ALL}
    ws = dfk.new_workspace(Mmax, D_MODEL, D_FF, dev)
    dfk.dfk_set_workspace(ws)

    # ---- pre-inference scheduler step (not timed)
    tune_s = 0.0
    skipped = 0
    if args.tuning_file and os.path.exists(args.tuning_file):
        dfk.dfk_load_tuning(args.tuning_file)
    elif not args.no_tune:
        t0 = time.perf_counter()
        scratch = torch.empty(dfk.dfk_tune_scratch_bytes(Mmax, D_MODEL, D_FF, dfk.DFK_BF16, 3),
                              dtype=torch.uint8, device=dev)
        dfk.dfk_tune(list(M_SET), D_MODEL, D_FF, dfk.DFK_BF16, scratch, sets=3, iters=20)
        skipped += dfk.dfk_tune_skipped()[0]
        dfk.dfk_tune([32, 64, 128, 256], D_MODEL, D_FF, dfk.DFK_BF16, scratch, sets=3, iters=12)
        skipped += dfk.dfk_tune_skipped()[0]
        torch.cuda.synchronize()
        del scratch
        tune_s = time.perf_counter() - t0
        if args.tuning_file:
            dfk.dfk_save_tuning(args.tuning_file)
    picks = {}
    for M in M_ALL:
        c, tuned = dfk.dfk_get_choice(M, D_MODEL, D_FF, dfk.DFK_BF16)
        picks[str(M)] = dict(c.as_dict(), tuned=tuned)

    call = {"auto": dfk.dfk_swiglu_mlp, "fused": dfk.dfk_swiglu_mlp_fused,
            "unfused": dfk.dfk_swiglu_mlp_unfused}[args.force]
    counter = [0]

    def one_call(M):
        w = layers[counter[0] % WEIGHT_SETS]
        counter[0] += 1
        call(X[M], w["Wg"], w["Wu"], w["Wd"], Y[M])

    def step():
        for M in M_SET:
            one_call(M)

    # ---- the contract's timed region: W warm-up steps, then exactly K steps
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    ev_ms = e0.elapsed_time(e1)
    ms_per_step = wall_ms / args.steps
    calls_per_step = len(M_SET)
    us_per_call = ms_per_step * 1e3 / calls_per_step

    # ---- per M (1..64 the same way, 128 and 256 beside them): 4 repeats x 50 launches, mean +- std and median;
    # which variant ran; fraction of the 8 TB/s peak
    per_m = {}
    for M in M_ALL:
        for _ in range(5):
            one_call(M)
        torch.cuda.synchronize()
        st = stats_4x50(torch, np, lambda i, M=M: call(X[M], layers[i]["Wg"], layers[i]["Wu"], layers[i]["Wd"], Y[M]), WEIGHT_SETS)
        b = algorithmic_bytes(M, D_MODEL, D_FF)
        per_m[str(M)] = dict(st, tb_per_s=round(b / st["mean_us"] / 1e6, 3), frac_of_peak=round(b / st["mean_us"] / 1e3 / HBM_PEAK_GBS, 4),
                             variant=variant_name(picks[str(M)]["variant"], picks[str(M)]["kmajor"]) if args.force == "auto" else args.force)
    mean_wide = float(np.mean([per_m[str(M)]["mean_us"] for M in M_WIDE]))
    frac_wide = float(np.mean([per_m[str(M)]["frac_of_peak"] for M in M_WIDE]))

    # ---- each variant forced, at the headline token counts: the fused <-> two-kernel crossover
    per_variant = {}
    for name, fn in (("fused", dfk.dfk_swiglu_mlp_fused), ("two_kernel", dfk.dfk_swiglu_mlp_unfused)):
        per_variant[name] = {str(M): stats_4x50(torch, np, lambda i, M=M, fn=fn: fn(X[M], layers[i]["Wg"], layers[i]["Wu"], layers[i]["Wd"], Y[M]),
                                                WEIGHT_SETS) for M in M_SET}

    # ---- the same block with the down projection's weights in a linear layer's own [out, in] layout
    # (W_down_t [d_model, d_ff], dfk_swiglu_mlp_wdt): its down kernel sums nothing across workgroups.  Beside the
    # headline, which stays on the layout the paper writes (Y = A_2 W_down with W_down [d_ff, d_model]).
    wdt = {}
    wd_t = []
    for l in layers:
        t = torch.empty((D_MODEL, D_FF), dtype=l["Wd"].dtype, device=dev)
        dfk.dfk_transpose_w_down(l["Wd"], t)
        wd_t.append(t)
    for M in M_WIDE:
        c, tuned = dfk.dfk_get_choice_wdt(M, D_MODEL, D_FF, dfk.DFK_BF16)
        st = stats_4x50(torch, np, lambda i, M=M: dfk.dfk_swiglu_mlp_wdt(X[M], layers[i]["Wg"], layers[i]["Wu"], wd_t[i], Y[M], None, ws),
                        WEIGHT_SETS)
        b = algorithmic_bytes(M, D_MODEL, D_FF)
        wdt[str(M)] = dict(st, frac_of_peak=round(b / st["mean_us"] / 1e3 / HBM_PEAK_GBS, 4), pick=dict(c.as_dict(), tuned=tuned))
    wdt_block = {"layout": "W_down_t [d_model, d_ff]; two kernels, the down kernel's workgroups own slices of d_model",
                 "mean_us_per_call_M_1_to_16": round(float(np.mean([wdt[str(M)]["mean_us"] for M in M_SET])), 2),
                 "mean_frac_of_peak_M_1_to_16": round(float(np.mean([wdt[str(M)]["frac_of_peak"] for M in M_SET])), 4),
                 "per_M_4x50": wdt}
    del wd_t

    # ---- read-stream ceiling of this machine (plain 128-bit streaming reads), and one write-only kernel of known
    # size; both also calibrate the FETCH_SIZE / WRITE_SIZE counters
    sink = torch.zeros(2, dtype=torch.int32, device=dev)
    srcs = [l[k] for l in layers for k in ("Wg", "Wu", "Wd")]
    for s in srcs[:3]:
        dfk.dfk_stream_read(s, sink)
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for s in srcs:
        dfk.dfk_stream_read(s, sink)
    b.record()
    torch.cuda.synchronize()
    read_small_gbs = sum(s.numel() * 2 for s in srcs) / (a.elapsed_time(b) * 1e-3) / 1e9
    # launches that read as many bytes as a whole call does (the three matrices of a layer in one buffer),
    # rotating over the weight sets, back to back
    whole = [torch.cat([l["Wg"].reshape(-1), l["Wu"].reshape(-1), l["Wd"].reshape(-1)]) for l in layers]
    for s in whole:
        dfk.dfk_stream_read(s, sink)
    torch.cuda.synchronize()
    reps = 4
    a.record()
    for _ in range(reps):
        for s in whole:
            dfk.dfk_stream_read(s, sink)
    b.record()
    torch.cuda.synchronize()
    read_gbs = reps * sum(s.numel() * 2 for s in whole) / (a.elapsed_time(b) * 1e-3) / 1e9
    del whole
    # the gate/up kernel's own memory pattern without its work (same slices, wavefronts, pieces and order)
    pat_waves = max(set(p["waves"] for p in picks.values() if p.get("kmajor") == 1), default=8)
    pat_splits = 256
    for l in layers:
        dfk.dfk_read_gateup_pattern(l["Wg"], l["Wu"], pat_splits, pat_waves, sink)
    torch.cuda.synchronize()
    a.record()
    for _ in range(reps):
        for l in layers:
            dfk.dfk_read_gateup_pattern(l["Wg"], l["Wu"], pat_splits, pat_waves, sink)
    b.record()
    torch.cuda.synchronize()
    pattern_us = a.elapsed_time(b) * 1e3 / (reps * len(layers))
    fill_target = torch.empty(64 << 20, dtype=torch.bfloat16, device=dev)     # 128 MiB written once
    dfk.dfk_fill_synthetic(fill_target, 1.0, 1)
    torch.cuda.synchronize()
    del fill_target

    # ---- per-launch durations of the scheduler's picks, HIP events on the launch stream around
    # back-to-back launches of each kernel alone (weights rotating over 3 synthetic sets in a scratch buffer)
    scratch = torch.empty(dfk.dfk_tune_scratch_bytes(max(M_WIDE), D_MODEL, D_FF, dfk.DFK_BF16, 3),
                          dtype=torch.uint8, device=dev)
    kernels = {}
    for M in M_WIDE:
        c, _ = dfk.dfk_get_choice(M, D_MODEL, D_FF, dfk.DFK_BF16)
        iters = max(30, args.steps // 4)
        us1, us2 = dfk.dfk_time_kernels(c, M, D_MODEL, D_FF, dfk.DFK_BF16, scratch, sets=3, iters=iters)
        kernels[str(M)] = {"first_launch_us": round(us1, 2), "second_launch_us": round(us2, 2),
                           "variant": variant_name(c.variant, c.kmajor)}
        if c.variant == dfk.DFK_VARIANT_FUSED and c.kmajor == 4:
            # one launch that holds the workgroups of both kernels: the launch as a whole, and beside it its two
            # parts launched alone (gate/up workgroups only; down workgroups only, waiting for nobody)
            whole_us = dfk.dfk_time_config(c, M, D_MODEL, D_FF, dfk.DFK_BF16, scratch, sets=3, iters=iters)
            kernels[str(M)] = {"first_launch_us": round(whole_us, 2), "second_launch_us": 0.0,
                               "gateup_workgroups_alone_us": round(us1, 2), "down_workgroups_alone_us": round(us2, 2),
                               "variant": variant_name(c.variant, c.kmajor)}
    del scratch

    # ---- roofline.  The bound is HBM.  `frac` is the whole call: algorithmic bytes of a call (three matrices
    # once + X + Y) / the time of all its launches, from the contract's timed region.  The dominant launch of a
    # call (the whole block where the single launch is picked, else the gate/up kernel, which reads two of the
    # three matrices) is reported beside it from back-to-back launches of that kernel alone.
    def first_launch_bytes(M):
        fused = picks[str(M)]["variant"] == dfk.DFK_VARIANT_FUSED
        return (6 if fused else 4) * D_MODEL * D_FF + (4 if fused else 2) * M * D_MODEL
    k_bytes = sum(first_launch_bytes(M) for M in M_SET) / calls_per_step
    k_us = sum(kernels[str(M)]["first_launch_us"] for M in M_SET) / calls_per_step
    k_achieved = k_bytes / k_us / 1e3   # GB/s
    mean_bytes = sum(algorithmic_bytes(M, D_MODEL, D_FF) for M in M_SET) / calls_per_step
    ev_us_per_call = ev_ms * 1e3 / (args.steps * calls_per_step)
    achieved = mean_bytes / ev_us_per_call / 1e3   # GB/s
    traffic_call, traffic_dom, traffic_src = committed_traffic()
    roofline = {"bound": "hbm", "kernel": "every launch of a call (the scheduler's pick per M, see config.variant_per_M)",
                "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4),
                "algorithmic_bytes_per_call": int(mean_bytes), "us_per_call": round(ev_us_per_call, 2),
                "traffic": traffic_call, "traffic_source": traffic_src,
                "dominant_kernel": {"kernel": "first launch of the call: the whole block where the single launch is picked, "
                                              "else the gate/up kernel", "achieved": round(k_achieved, 1),
                                    "frac": round(k_achieved / HBM_PEAK_GBS, 4), "algorithmic_bytes_per_launch": int(k_bytes),
                                    "us_per_launch": round(k_us, 2), "traffic": traffic_dom},
                # plain streaming reads on the same box: launches of a whole call's size / of one matrix
                "read_stream_ceiling_gbs": round(read_gbs, 1),
                "read_stream_one_matrix_gbs": round(read_small_gbs, 1),
                "frac_of_read_stream_ceiling": round(achieved / read_gbs, 4),
                # a read-only kernel with the gate/up kernel's slices, wavefronts, 256-byte pieces and tile order
                "gateup_pattern_read_us": round(pattern_us, 2),
                "gateup_pattern_read_gbs": round(4 * D_MODEL * D_FF / pattern_us / 1e3, 1)}

    # ---- the fp64 oracle on the host cores: whole steps of the same workload until ~12 s of CPU
    # work have been done (+ parity of the GPU path on every call of the first of those steps)
    cpu = None
    parity = None
    if not args.no_cpu_baseline:
        from oracle import oracle
        cores = oracle.default_threads()
        hosts = [{k: di.to_numpy(v) for k, v in l.items()} for l in layers]
        worst = 0.0
        cpu_s, calls, step_i = 0.0, 0, 0
        while cpu_s < 12.0 and step_i < 64:
            h = hosts[step_i % WEIGHT_SETS]
            t0 = time.perf_counter()
            refs = {M: oracle.swiglu_mlp(hosts[0]["X"][:M], h["Wg"], h["Wu"], h["Wd"], nthreads=cores)
                    for M in M_SET}
            cpu_s += time.perf_counter() - t0
            calls += len(M_SET)
            if step_i < WEIGHT_SETS:
                w = layers[step_i]
                for M in M_SET:
                    call(X[M], w["Wg"], w["Wu"], w["Wd"], Y[M])
                    torch.cuda.synchronize()
                    y = di.as_f64(di.to_numpy(Y[M]))
                    worst = max(worst, float(np.max(np.abs(y - refs[M])) / np.max(np.abs(refs[M]))))
            step_i += 1
        cpu = {"value": round(cpu_s * 1e6 / calls, 1), "unit": "us/call", "cores": cores,
               "kind": "oracle",
               "sample": f"{step_i} steps of the same workload (M=1,2,4,8,16 once each per step, weight sets "
                         f"rotating), {calls} calls, {cpu_s:.1f} s of fp64 CPU work"}
        parity = {"max_rel_err_vs_oracle": worst, "tolerance": 2e-2,
                  "checked": f"every call of the first {min(step_i, WEIGHT_SETS)} steps, all outputs"}
        del hosts

    # ---- beside the headline (not part of `value`): the other layer shapes and the 32-layer decode pass
    extras = {}
    if not args.no_extras:
        dfk.dfk_set_workspace(None)
        del layers, X, Y, ws, srcs
        torch.cuda.empty_cache()
        extras["shapes"] = shapes(args, torch, di, dfk, dev, compact=True)
        extras["decode32"] = decode32(args, torch, di, dfk, dev, compact=True)

    variant_per_m = {str(M): (variant_name(picks[str(M)]["variant"], picks[str(M)]["kmajor"]) if args.force == "auto" else args.force) for M in M_SET}
    names = sorted(set(variant_per_m.values()))
    out = {
        "metric": "SwiGLU MLP us/call (" + ("scheduler's pick per M: " + ", ".join(
            f"{v} at M={'/'.join(m for m in variant_per_m if variant_per_m[m] == v)}" for v in names)) +
                  "), d=4096 ff=14336 bf16, mean over M in {1,2,4,8,16}",
        "value": round(us_per_call, 2), "unit": "us/call",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "llama3-8b-shaped SwiGLU MLP layer, d_model=4096 d_ff=14336, "
                               "M in {1,2,4,8,16}, one call per M per step, 4 rotating weight sets",
                   "entry": args.force, "calls_per_step": calls_per_step, "variant_per_M": variant_per_m},
        "whole_call_frac_of_peak": round(achieved / HBM_PEAK_GBS, 4),
        "achieved_tb_per_s": round(achieved / 1e3, 3),
        "second_headline_M_1_to_64": {"mean_us_per_call": round(mean_wide, 2), "mean_frac_of_peak": round(frac_wide, 4),
                                      "token_counts": list(M_WIDE), "protocol": "4 repeats x 50 launches per M"},
        "per_M_4x50": per_m, "per_variant_4x50": per_variant, "w_down_t_layout": wdt_block,
        "per_M_launches": kernels, "scheduler_picks": picks,
        "tune_seconds": round(tune_s, 2), "tune_candidates_skipped": skipped,
        "roofline": roofline, "cpu_baseline": cpu, "parity": parity,
    }
    out.update(extras)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
