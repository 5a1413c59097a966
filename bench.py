#!/usr/bin/env python3
"""Benchmark of the MixLLM quantized linear hot path on one MI355X.

A "step" is one pass of the whole hot path (activation quantizer + mixed W4/W8-A8 linear)
over the four linear layers of one Llama-3-8B decoder block (QKV, O, gate+up, down) at M
tokens, on seeded synthetic inputs that are already resident in HBM.  Weight buffers are
rotated over several copies so that no step finds its weights in the 256 MB memory-side cache.

Default run:  decode leg (M = 1; the `value` of the JSON line, in GB/s of algorithmic bytes)
followed by short extra legs (other decode M, prefill M = 2048 in TOPS) that are reported in
the same JSON line under "sweep" / "prefill".  `--workload prefill` makes the prefill leg the
primary one; `--workload 70b` runs the Llama-3.1-70B-shaped block over M in {1, 16, 64, 256, 2048};
`--workload stack` runs 32 blocks back to back with an uneven 8-bit share per layer at M in {1, 256}.
Every leg carries mean, median and minimum time per step, the time of its dominant kernel, and both
as fractions of the roofline min(HBM, int8 MFMA) for its algorithmic bytes and operations.
One JSON line is printed on stdout; progress goes to stderr.
"""
import hashlib
import argparse
import json
import os
import sys
import time

import numpy as np

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published
INT8_PEAK_TOPS = 5000.0      # MI355X dense int8 MFMA, published
MALL_BYTES = 256 << 20


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def layer_alg_bytes(K, N, n8, M):
    """Algorithmic bytes of one linear launch: every stored weight byte once (4-bit rows:
    K/2 + 2.5 K/128; 8-bit rows: K + 2; 4 B of channel index per row), activations and
    token scales in, fp16 outputs out."""
    n4 = N - n8
    w = n4 * (K // 2 + 2.5 * K / 128) + n8 * (K + 2) + 4 * N
    return w + M * K + 2 * M + 2 * M * N


def quant_alg_bytes(K, M):
    return 2 * M * K + M * K + 2 * M


def roofline_seconds(nbytes, ops):
    """Time the roofline allows: whichever of the HBM stream and the int8 MFMA work takes longer."""
    return max(nbytes / (HBM_PEAK_GBS * 1e9), ops / (INT8_PEAK_TOPS * 1e12))


def roofline_entry(nbytes, ops, seconds):
    """A `roofline` object for work of `nbytes` algorithmic bytes and `ops` operations done in `seconds`."""
    t_hbm, t_mfma = nbytes / (HBM_PEAK_GBS * 1e9), ops / (INT8_PEAK_TOPS * 1e12)
    if t_hbm >= t_mfma:
        ach, peak, unit, bound = nbytes / seconds / 1e9, HBM_PEAK_GBS, "GB/s", "hbm"
    else:
        ach, peak, unit, bound = ops / seconds / 1e12, INT8_PEAK_TOPS, "TOP/s", "mfma"
    return {"bound": bound, "achieved": ach, "peak": peak, "unit": unit, "frac": ach / peak,
            "frac_of_min_hbm_mfma": max(t_hbm, t_mfma) / seconds}


def source_sha(*names):
    """sha256 (16 hex digits) over the kernel sources a stored counter figure belongs to, comments and
    white space left out (a reworded comment does not make a measurement stale)."""
    import re
    h = hashlib.sha256()
    root = os.path.join(os.path.dirname(os.path.abspath(__file__)), "paper_2412_14590_amd", "csrc")
    for n in names:
        with open(os.path.join(root, n), "r") as f:
            text = f.read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        text = re.sub(r"//[^\n]*", "", text)
        h.update("".join(text.split()).encode())
    return h.hexdigest()[:16]


def salience_bench(args, torch, mx, synth, dev):
    """Global precision search (Sec. 3.2) on synthetic (W, G): the salience kernel on the gate+up
    shaped layer (K = 4096, N = 28672; it reads W and G once: 4 bytes per weight) and the top-T
    selection over the saliences of a 32-block stack (1.38 M channels, T = 10 %)."""
    K, N = synth.LLAMA3_8B["gate_up"]
    W = torch.from_numpy(synth.make_w(N, K, seed=0, tag="w/gate_up")).to(dev)
    G = (torch.randn((N, K), device=dev, generator=torch.Generator(device=dev).manual_seed(3)) * 0.05).half()
    sal = mx.channel_salience(W, G)
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = max(5, min(args.steps, 50))
    for _ in range(3):
        mx.channel_salience(W, G, out=sal)
    a.record()
    for _ in range(reps):
        mx.channel_salience(W, G, out=sal)
    b.record()
    torch.cuda.synchronize()
    t_sal = a.elapsed_time(b) * 1e-3 / reps
    bytes_sal = 4.0 * N * K + 4 * N
    rng = np.random.default_rng(0)
    stack = [torch.from_numpy(np.exp(rng.standard_normal(n) + rng.standard_normal()).astype(np.float32)).to(dev)
             for _ in range(32) for n in (6144, 4096, 28672, 4096)]
    total = sum(int(t.numel()) for t in stack)
    mx.select_salient(stack, total // 10)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(5):
        chosen = mx.select_salient(stack, total // 10)
    torch.cuda.synchronize()
    t_sel = (time.perf_counter() - t0) / 5
    log(f"[salience] gate+up layer: {t_sal * 1e6:.1f} us, {bytes_sal / t_sal / 1e9:.0f} GB/s; selection of {total // 10} of "
        f"{total} channels over {len(stack)} layers: {t_sel * 1e3:.2f} ms (host call to host result)")
    result = {"metric": "mixed W4/W8-A8 linear TOPS + HBM GB/s at M=1..2048 (% roofline)", "value": bytes_sal / t_sal / 1e9,
              "unit": "GB/s", "n_gpus": 1, "steps": reps, "warmup": 3, "ms_per_step": t_sal * 1e3, "higher_is_better": True,
              "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
              "config": {"workload": "global precision search (Sec. 3.2): channel salience of a K=4096, N=28672 layer from "
                                     "fp16 W and G; value = its algorithmic bytes (4 per weight) / time"},
              "roofline": {"bound": "hbm", "achieved": bytes_sal / t_sal / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                           "frac": bytes_sal / t_sal / 1e9 / HBM_PEAK_GBS, "traffic": None,
                           "kernel": "channel_salience_kernel, K=4096 N=28672"},
              "selection": {"layers": len(stack), "channels": total, "T": total // 10, "ms": t_sel * 1e3,
                            "chosen_per_layer_min_max": [min(len(c) for c in chosen), max(len(c) for c in chosen)]}}
    if not args.no_cpu:
        from oracle import ref
        rows = 2048
        Wh, Gh = W[:rows].cpu().numpy(), G[:rows].cpu().numpy()
        t1 = time.perf_counter()
        ref.channel_salience(Wh, Gh)
        t_cpu = time.perf_counter() - t1
        result["cpu_baseline"] = {"value": 4.0 * rows * K / t_cpu / 1e9, "unit": "GB/s", "cores": ref.num_threads(),
                                  "kind": "oracle", "sample": f"the first {rows} channels of the same layer ({t_cpu * 1e3:.0f} ms)"}
    return result


def share_sweep(args, torch, mx, synth, dev):
    """The grid of the paper's single-linear study (Sec. 5.2: K = 4096, N in {4096, 14336},
    8-bit shares 0 / 10 / 20 / 50 / 100 %, token counts 1..1024), on seeded synthetic weights:
    time of the whole path from fp16 activations (quantizer + mixed linear) and of the linear alone,
    each against the roofline min(HBM, int8 MFMA) of its algorithmic bytes and operations.  Every
    figure is the mean over `reps` launches replayed from a HIP graph, weights rotating over
    enough copies to stay out of the memory-side cache."""
    K, rows = 4096, []
    shares = [0.0, 0.10, 0.20, 0.50, 1.0]
    Ms = [1, 16, 64, 256, 1024]

    def graph_time(fn, reps):
        for i in range(min(reps, 8)):
            fn(i)
        torch.cuda.synchronize()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        g = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(g, stream=side):
                for i in range(reps):
                    fn(i)
        torch.cuda.current_stream().wait_stream(side)
        g.replay()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(3):
            g.replay()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) * 1e-3 / (3 * reps)

    for N in (4096, 14336):
        W = torch.from_numpy(synth.make_w(N, K, seed=0, tag=f"w/sweep{N}")).to(dev)
        order = synth.salience_order(W.cpu().numpy(), seed=0)
        for f in shares:
            n8 = synth.n8_for(N, f)
            L0 = mx.quantize_weights(W, np.sort(order[:n8]).astype(np.int32))
            n_c = max(2, -(-2 * MALL_BYTES // L0.weight_bytes()))
            Ls = [L0] + [L0.clone() for _ in range(n_c - 1)]
            for M in Ms:
                x = torch.from_numpy(synth.make_x(M, K, seed=7, tag="x/sweep")).to(dev)
                xq, xs = mx.quantize_activations(x)
                y = torch.empty((M, N), dtype=torch.float16, device=dev)
                ws = torch.empty(mx.query_sizes(M, K, N, n8)["workspace_bytes"], dtype=torch.uint8, device=dev)
                reps = 60 if M <= 64 else 30
                t_path = graph_time(lambda i: mx.linear_fp16(x, Ls[i % n_c], out=y, workspace=ws), reps)
                t_lin = graph_time(lambda i: mx.mixed_linear(xq, xs, Ls[i % n_c], out=y, workspace=ws), reps)
                nb, ops = layer_alg_bytes(K, N, n8, M), 2.0 * M * N * K
                row = {"N": N, "share8": f, "n8": n8, "M": M, "path_us": t_path * 1e6, "linear_us": t_lin * 1e6,
                       "linear_GBps": nb / t_lin / 1e9, "linear_TOPS": ops / t_lin / 1e12,
                       "roofline": roofline_entry(nb, ops, t_lin)}
                rows.append(row)
                log(f"[sweep] N={N} share={f:.2f} M={M}: path {row['path_us']:.1f} us, linear {row['linear_us']:.1f} us, "
                    f"{row['linear_GBps']:.0f} GB/s, {row['linear_TOPS']:.0f} TOPS, "
                    f"{row['roofline']['frac_of_min_hbm_mfma']:.2f} of min(HBM, MFMA)")
            del Ls
            torch.cuda.empty_cache()
    ref_row = next(r for r in rows if r["N"] == 14336 and r["share8"] == 0.10 and r["M"] == 1)
    return {"metric": "mixed W4/W8-A8 linear TOPS + HBM GB/s at M=1..2048 (% roofline)", "value": ref_row["linear_GBps"],
            "unit": "GB/s", "n_gpus": 1, "steps": 60, "warmup": 8, "ms_per_step": ref_row["linear_us"] * 1e-3,
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int8", "data": "synthetic",
            "config": {"workload": "single linear K=4096, N in {4096, 14336}, 8-bit share 0..100 %, M in {1, 16, 64, 256, 1024}; "
                                   "value = the linear at N=14336, 10 % 8-bit, M=1"},
            "roofline": ref_row["roofline"], "rows": rows}


def shape_sweep(args, torch, mx, synth, dev):
    """Every layer of a decoder block x token counts x kernel choices: the library's own choice (with
    and without the optional scratch of the linear), the tiled kernel in each block shape, the kernel
    for a few dozen tokens, the decode kernel - time of the linear alone, launches replayed from a HIP
    graph with the weights rotating over >= 512 MB of copies, against min(HBM, int8 MFMA).  This is the
    measurement behind the dispatch rules (which kernel, which block shape, whether K is split); a
    library built with other launch constants (MIXLLM_EXTRA_FLAGS / MIXLLM_LIB_OUT of the build,
    MIXLLM_LIB of the binding) is measured the same way."""
    Ms = [int(m) for m in args.ms.split(",")]
    paths = {"auto": mx.PATH_AUTO, "tiled_32x128": mx.PATH_PREFILL_32, "tiled_64x128": mx.PATH_PREFILL_64,
             "tiled_128x128": mx.PATH_PREFILL_128, "few_dozen_tokens": mx.PATH_MID, "decode": mx.PATH_DECODE}

    def graph_time(fn, reps):
        for i in range(4):
            fn(i)
        torch.cuda.synchronize()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        g = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(g, stream=side):
                for i in range(reps):
                    fn(i)
        torch.cuda.current_stream().wait_stream(side)
        g.replay()
        torch.cuda.synchronize()
        best = float("inf")
        for _ in range(3):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            g.replay()
            b.record()
            torch.cuda.synchronize()
            best = min(best, a.elapsed_time(b) * 1e-3 / reps)
        return best

    rows = []
    for name, K, N, sigma, n_out in synth.model_layers(args.model):
        W = torch.from_numpy(synth.make_w(N, K, sigma, n_out, seed=0, tag="w/" + name)).to(dev)
        n8 = synth.n8_for(N, 0.10)
        L0 = mx.quantize_weights(W, torch.randperm(N, device=dev, generator=torch.Generator(device=dev).manual_seed(1))[:n8].to(torch.int32))
        del W
        n_c = max(2, -(-2 * MALL_BYTES // L0.weight_bytes()))
        Ls = [L0] + [L0.clone() for _ in range(n_c - 1)]
        for M in Ms:
            x = torch.from_numpy(synth.make_x(M, K, seed=7, tag="x/" + name)).to(dev)
            xq, xs = mx.quantize_activations(x)
            y = torch.empty((M, N), dtype=torch.float16, device=dev)
            ws = torch.empty(max(16, mx.query_sizes(M, K, N, n8)["linear_workspace_bytes"]), dtype=torch.uint8, device=dev)
            big = torch.empty(64 << 20, dtype=torch.uint8, device=dev)       # room for any K split of a forced block shape
            nb, ops = layer_alg_bytes(K, N, n8, M), 2.0 * M * N * K
            row = {"layer": name, "K": K, "N": N, "n8": n8, "M": M, "us": {}}
            # a replay walks all n_c copies (>= 512 MB): every launch reads its weights from HBM, as in a step of the model
            reps = max(20 if M <= 512 else 8, n_c)
            graph_time(lambda i: mx.mixed_linear(xq, xs, Ls[i % n_c], out=y), reps)   # clocks settle before the first figure
            for pn, pv in paths.items():
                for scratch in ((None, ws) if pn == "auto" else (big,) if pn.startswith("tiled") else (None,)):
                    key = pn + ("" if pn != "auto" else "+scratch" if scratch is not None else "")
                    try:
                        t = graph_time(lambda i: mx.mixed_linear(xq, xs, Ls[i % n_c], pv, out=y, workspace=scratch), reps)
                    except mx.MixllmError:
                        continue
                    row["us"][key] = round(t * 1e6, 1)
            t_auto = row["us"]["auto+scratch"] * 1e-6
            row["roofline"] = roofline_entry(nb, ops, t_auto)
            rows.append(row)
            log(f"[shapes] {name} K={K} N={N} M={M}: {json.dumps(row['us'])}  auto+scratch {row['roofline']['frac_of_min_hbm_mfma']:.2f} of min(HBM, MFMA)")
        del Ls, L0
        torch.cuda.empty_cache()
    ref_row = max(rows, key=lambda r: (r["K"] * r["N"], -r["M"]))
    return {"metric": "mixed W4/W8-A8 linear TOPS + HBM GB/s at M=1..2048 (% roofline)", "value": ref_row["roofline"]["achieved"],
            "unit": ref_row["roofline"]["unit"], "n_gpus": 1, "steps": 20, "warmup": 4, "ms_per_step": ref_row["us"]["auto+scratch"] * 1e-3,
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int8", "data": "synthetic",
            "config": {"workload": f"single linears of the {args.model} block, M in {Ms}, every kernel choice; value = the largest layer at the "
                                   f"smallest M, library's choice", "library": os.environ.get("MIXLLM_LIB", "in-tree build")},
            "roofline": ref_row["roofline"], "rows": rows}


def block_timeline(args, torch, mx, synth, dev):
    """Where the blocks of the tiled kernel spend their time: needs a library built with
    MIXLLM_EXTRA_FLAGS=-DMIXLLM_STAMPS (thread 0 of every block then records the 100 MHz clock at kernel
    entry, after the prologue's loads have landed, after the K loop, after its drain, after the epilogue's
    stores are issued and after they are acknowledged).  One layer (--layer of --model) at --m tokens,
    single launches over >= 512 MB of rotating weight copies; medians over the launches of per-block means."""
    import ctypes as C
    lib = mx.lib()
    if not hasattr(lib, "mixllm_debug_set_stamps"):
        log("bench.py: --workload timeline needs a library built with MIXLLM_EXTRA_FLAGS=-DMIXLLM_STAMPS (set MIXLLM_LIB to it)")
        sys.exit(2)
    lib.mixllm_debug_set_stamps.argtypes = [C.c_void_p]
    lib.mixllm_debug_set_stamps.restype = C.c_int
    name, K, N, sigma, n_out = next(l for l in synth.model_layers(args.model) if l[0] == args.layer)
    M = args.m if args.m is not None else 2048
    path = {"auto": mx.PATH_PREFILL, "32": mx.PATH_PREFILL_32, "64": mx.PATH_PREFILL_64, "128": mx.PATH_PREFILL_128}[args.block_rows]
    W = torch.from_numpy(synth.make_w(N, K, sigma, n_out, seed=0, tag="w/" + name)).to(dev)
    n8 = synth.n8_for(N, 0.10)
    L0 = mx.quantize_weights(W, torch.randperm(N, device=dev, generator=torch.Generator(device=dev).manual_seed(1))[:n8].to(torch.int32))
    del W
    n_c = max(2, -(-2 * MALL_BYTES // L0.weight_bytes()))
    Ls = [L0] + [L0.clone() for _ in range(n_c - 1)]
    x = torch.from_numpy(synth.make_x(M, K, seed=7, tag="x/" + name)).to(dev)
    xq, xs = mx.quantize_activations(x)
    y = torch.empty((M, N), dtype=torch.float16, device=dev)
    ws = torch.empty(max(16, mx.query_sizes(M, K, N, n8)["linear_workspace_bytes"]), dtype=torch.uint8, device=dev)
    # one row per block; an upper bound of the grid (smallest block shape, two partial column tiles, 8 K parts, padding to the XCDs)
    n_rows = -(-M // 32) * (-(-N // 128) + 2) * 8 + 64
    if n_rows > 1 << 20:
        log("bench.py: --workload timeline: too many blocks for the stamp array")
        sys.exit(2)
    stamps = torch.zeros((n_rows, 8), dtype=torch.int64, device=dev)
    for L in Ls:
        mx.mixed_linear(xq, xs, L, path, out=y, workspace=ws)
    torch.cuda.synchronize()
    rows = []
    for L in Ls * 2:
        stamps.zero_()
        torch.cuda.synchronize()
        assert lib.mixllm_debug_set_stamps(stamps.data_ptr()) == 0
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        mx.mixed_linear(xq, xs, L, path, out=y, workspace=ws)
        b.record()
        torch.cuda.synchronize()
        assert lib.mixllm_debug_set_stamps(None) == 0
        st = stamps.cpu().numpy().astype(np.float64)
        st = st[st[:, 5] > 0]
        t0 = st[:, 0].min()
        four, eight = st[st[:, 1] > 0], st[st[:, 1] == 0]      # only blocks of the 4-bit part carry the inner stamps
        d = lambda i, j: float((four[:, i] - four[:, j]).mean()) / 100.0
        rows.append([a.elapsed_time(b) * 1e3, len(st), d(1, 0), d(2, 1), d(3, 2), d(4, 3), d(5, 4), float(st[:, 5].max() - t0) / 100.0,
                     float((eight[:, 5] - eight[:, 0]).mean()) / 100.0 if len(eight) else 0.0, len(eight)])
    m = np.median(np.array(rows), axis=0)
    keys = ["launch_us_by_events", "blocks", "prologue_us", "k_loop_us", "drain_and_last_rescale_us", "epilogue_issue_us", "store_ack_us",
            "first_entry_to_last_exit_us", "entry_to_exit_of_an_8bit_block_us", "blocks_8bit"]
    tl = {k: round(float(v), 2) for k, v in zip(keys, m)}
    log(f"[timeline] {name} K={K} N={N} M={M} block rows {args.block_rows}: {json.dumps(tl)}")
    ops = 2.0 * M * N * K
    return {"metric": "mixed W4/W8-A8 linear TOPS + HBM GB/s at M=1..2048 (% roofline)", "value": ops / (tl["launch_us_by_events"] * 1e-6) / 1e12,
            "unit": "TOP/s", "n_gpus": 1, "steps": 2 * n_c, "warmup": n_c, "ms_per_step": tl["launch_us_by_events"] * 1e-3, "higher_is_better": True,
            "scaling": "weak", "vs_baseline": None, "dtype": "int8", "data": "synthetic",
            "config": {"workload": f"single launches of the tiled kernel with clock stamps, layer {name} K={K} N={N}, M={M}, block rows {args.block_rows}",
                       "library": os.environ.get("MIXLLM_LIB", "in-tree build")},
            "timeline_of_a_4bit_block": tl}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", choices=["decode", "prefill", "70b", "stack", "share-sweep", "salience", "shapes", "timeline"], default="decode",
                    help="decode / prefill: one Llama-3-8B-shaped block at M = 1 / 2048 (plus the other token counts as extra "
                         "legs); 70b: one Llama-3.1-70B-shaped block, M in {1, 16, 64, 256, 2048}; stack: 32 8B-shaped blocks "
                         "back to back with an uneven 8-bit share per layer, M in {1, 256}; share-sweep: single linears "
                         "K=4096, N in {4096, 14336}, 8-bit shares 0..100 %%, M = 1..1024 (the grid of the paper's "
                         "single-linear study, Sec. 5.2); salience: the global precision search of Sec. 3.2; shapes: every "
                         "layer of a block (--model) x token counts (--ms) x kernel choice, the measurement behind the dispatch rules; "
                         "timeline: clock stamps inside the blocks of the tiled kernel (needs a library built with -DMIXLLM_STAMPS)")
    ap.add_argument("--layer", choices=["qkv", "o", "gate_up", "down"], default="gate_up", help="layer of --workload timeline")
    ap.add_argument("--block-rows", choices=["auto", "32", "64", "128"], default="auto", help="token rows of a block in --workload timeline")
    ap.add_argument("--model", choices=["8b", "70b"], default="8b", help="layer shapes of --workload shapes")
    ap.add_argument("--ms", default="32,64,128,256,512", help="token counts of --workload shapes, comma separated")
    ap.add_argument("--m", type=int, default=None, help="tokens of the primary leg (default 1; 2048 for --workload prefill)")
    ap.add_argument("--no-extras", action="store_true", help="primary leg only (for profiling)")
    ap.add_argument("--no-graph", action="store_true", help="launch every kernel from Python instead of replaying a HIP graph")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also launch a plain 1 GiB copy kernel (reference for scaling FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build is single-GPU by construction (one process, one MI355X); "
            "--gpus above 1 is not supported")
        sys.exit(2)

    import torch
    import paper_2412_14590_amd as mx
    from paper_2412_14590_amd import synth

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    mx.lib()   # fail loudly if the HIP library is missing
    dev = torch.device("cuda:0")
    if args.workload == "salience":
        print(json.dumps(salience_bench(args, torch, mx, synth, dev)), flush=True)
        return
    if args.workload == "share-sweep":
        print(json.dumps(share_sweep(args, torch, mx, synth, dev)), flush=True)
        return
    if args.workload == "timeline":
        print(json.dumps(block_timeline(args, torch, mx, synth, dev)))
        return
    if args.workload == "shapes":
        print(json.dumps(shape_sweep(args, torch, mx, synth, dev)), flush=True)
        return
    M0 = args.m if args.m is not None else (2048 if args.workload == "prefill" else 1)

    # ---- inputs (seeded, synthetic) --------------------------------------------------------
    # `layers`: the linears of one step, in launch order.  decode / prefill / 70b: the four linears
    # of one decoder block, 10 % of the channels at 8 bits; stack: 32 blocks of the 8B shapes with
    # the per-layer 8-bit share of synth.uneven_fractions (0..40 %, mean 10 %) - the fp16 weights
    # of a layer kind are drawn once and shared by the 32 blocks, each block quantizes them with
    # its own share (what is measured is the kernels' balance across shares, not the values).
    t0 = time.time()
    model = "70b" if args.workload == "70b" else "8b"
    kinds = {}
    for name, K, N, sigma, n_out in synth.model_layers(model):
        W = synth.make_w(N, K, sigma, n_out, seed=0, tag="w/" + name)
        kinds[name] = (K, N, W, synth.salience_order(W, seed=0))
        log(f"[bench] weights {name}: K={K} N={N}  ({time.time() - t0:.1f}s)")
    if args.workload == "stack":
        shares = synth.uneven_fractions(32, seed=0)
        specs = [(f"{name}.{blk}", name, shares[(blk, name)]) for blk in range(32) for name in kinds]
    else:
        specs = [(name, name, 0.10) for name in kinds]
    layers, packed0 = [], []
    for lname, kind, f in specs:
        K, N, W, order = kinds[kind]
        n8 = synth.n8_for(N, f)
        lay = synth.LayerInputs(lname, K, N, n8, W, np.sort(order[:n8]).astype(np.int32))
        layers.append(lay)
    Wd = {k: torch.from_numpy(v[2]).to(dev) for k, v in kinds.items()}
    packed0 = [mx.quantize_weights(Wd[kind], lay.salient_idx) for lay, (_, kind, _) in zip(layers, specs)]
    torch.cuda.synchronize()
    del Wd
    set_bytes = sum(p.weight_bytes() for p in packed0)
    n_copies = max(1 if set_bytes >= 2 * MALL_BYTES else 2, -(-2 * MALL_BYTES // set_bytes))   # >= 512 MB between reuses
    copies = [packed0] + [[p.clone() for p in packed0] for _ in range(n_copies - 1)]
    log(f"[bench] {len(layers)} linears per step, packed weights {set_bytes / 1e6:.1f} MB, {n_copies} rotating copies")

    # granularity of the scales: the measured default (one activation scale per token, one scale per
    # 8-bit channel) or the paper's (both per group of 128, Sec. 4.1); the paper's gets a leg of its own
    mode = {"copies": copies, "act_group": None, "w8_group": None}

    def make_acts(M):
        xk = {k: torch.from_numpy(synth.make_x(M, v[0], seed=7, tag="x/" + k)).to(dev) for k, v in kinds.items()}
        xs_ = [xk[kind] for _, kind, _ in specs]
        ws_bytes = max(mx.query_sizes(M, l.K, l.N, l.n8, mode["act_group"], mode["w8_group"])["workspace_bytes"] for l in layers)
        yk = {k: torch.empty((M, v[1]), dtype=torch.float16, device=dev) for k, v in kinds.items()}
        wsp = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
        # (None, None, y, workspace) per linear: the linears of a step run one after the other on one
        # stream, so layers of one kind share an output tensor and all share the workspace
        bufs = [(None, None, yk[specs[li][1]], wsp) for li in range(len(layers))]
        return xs_, bufs

    # Order of the linear launches as the GPU executes them (layer indices; a captured graph adds
    # its launches at every replay).  The decode kernel launches one block per CU whatever the
    # layer, so a kernel trace of this run needs this list to tell the layers apart.
    executed, recording = [], [None]

    def note(li):
        (executed if recording[0] is None else recording[0]).append(li)

    def step(i, xs_, bufs):
        ws = mode["copies"][i % n_copies]
        for li in range(len(layers)):
            # the whole hot path from fp16 activations: one fused kernel where the library has one
            # (a few tokens of a short row), otherwise activation quantizer + linear
            mx.linear_fp16(xs_[li], ws[li], act_group=mode["act_group"], out=bufs[li][2], workspace=bufs[li][3])
            note(li)

    def time_steps(M, steps, warmup):
        """Seconds per step: {"mean", "median", "min"}.  Decode steps are launch bound when driven from
        Python (8 ctypes calls of ~5 us each), so n_copies consecutive steps (one per weight copy) are
        captured into one HIP graph and replayed; the graph's output is checked against eager launches.
        The mean is wall time over all timed steps between two synchronizations; median and minimum are
        over the timed units (one graph replay = n_copies steps, or one eager step), each between two
        events on the launch stream."""
        xs_, bufs = make_acts(M)
        use_graph = not args.no_graph and M <= 256      # launch bound when driven from Python up to a few hundred tokens
        for i in range(max(warmup, n_copies) if not use_graph else n_copies):
            step(i, xs_, bufs)
        torch.cuda.synchronize()
        if use_graph:
            last = {id(b[2]): b[2] for b in bufs}
            eager = {k: v.clone() for k, v in last.items()}          # y of the last eager step (copy n_copies - 1)
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            graph = torch.cuda.CUDAGraph()
            recording[0] = []
            with torch.cuda.stream(side):
                with torch.cuda.graph(graph, stream=side):
                    for i in range(n_copies):
                        step(i, xs_, bufs)
            captured, recording[0] = recording[0], None
            torch.cuda.current_stream().wait_stream(side)

            def unit():
                graph.replay()
                executed.extend(captured)

            for rep in range(3):                          # replay check, with eager work in between
                for v in last.values():
                    v.zero_()
                unit()
                torch.cuda.synchronize()
                for k, v in last.items():
                    assert torch.equal(eager[k], v), "HIP graph replay differs from eager launch"
            per_unit, n_warm, n_units = n_copies, max(1, warmup // n_copies), max(1, -(-steps // n_copies))
        else:
            count = [0]

            def unit():
                step(count[0], xs_, bufs)
                count[0] += 1

            per_unit, n_warm, n_units = 1, warmup, steps
        for _ in range(n_warm):
            unit()
        torch.cuda.synchronize()
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(n_units + 1)]
        t = time.perf_counter()
        evs[0].record()
        for k in range(n_units):
            unit()
            evs[k + 1].record()
        torch.cuda.synchronize()
        mean = (time.perf_counter() - t) / (n_units * per_unit)
        per = np.array([evs[k].elapsed_time(evs[k + 1]) for k in range(n_units)]) * 1e-3 / per_unit
        return {"mean": mean, "median": float(np.median(per)), "min": float(per.min())}

    def time_dominant(M, reps, li):
        """Average duration of one launch of the linear kernel of layer `li`: `reps` launches
        (weight copies rotating) recorded into one HIP graph, the replay bracketed by one pair
        of HIP events on the launch stream, so that neither Python nor event handling sits
        between two launches.  This is the figure a rocprofv3 kernel trace of the same kernel
        has to agree with.  Also returned: the mean over launches that each have their own event
        pair (includes ~2 us of event and launch handling per launch)."""
        xs_, bufs = make_acts(M)
        _, _, y, ws = bufs[li]
        xq, xsc = mx.quantize_activations(xs_[li])
        # copies of this layer's weights to rotate over: at least 512 MB between two uses of one
        own = [c[li] for c in copies]
        while sum(p.weight_bytes() for p in own) < 2 * MALL_BYTES:
            own.append(own[0].clone())

        def one(i):
            # the launch the step makes for this layer: for a single token the decode kernel
            # that quantizes its own activations, otherwise the linear after the quantizer
            if M == 1:
                mx.linear_fp16(xs_[li], own[i % len(own)], out=y, workspace=ws)
            else:
                mx.mixed_linear(xq, xsc, own[i % len(own)], out=y, workspace=ws)
            note(li)

        for i in range(max(10, reps)):      # warm: clocks settle over tens of milliseconds at large M
            one(i)
        torch.cuda.synchronize()

        def burst():
            for i in range(reps):
                one(i)

        replay = burst
        if not args.no_graph:
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            graph = torch.cuda.CUDAGraph()
            recording[0] = []
            with torch.cuda.stream(side):
                with torch.cuda.graph(graph, stream=side):
                    burst()
            captured, recording[0] = recording[0], None
            torch.cuda.current_stream().wait_stream(side)

            def replay():
                graph.replay()
                executed.extend(captured)
        replay()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        nrep = 3
        a.record()
        for _ in range(nrep):
            replay()
        b.record()
        torch.cuda.synchronize()
        t_graph = a.elapsed_time(b) * 1e-3 / (reps * nrep)
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for i, (a, b) in enumerate(evs):
            a.record()
            one(i)
            b.record()
        torch.cuda.synchronize()
        ts = np.array([a.elapsed_time(b) for a, b in evs]) * 1e-3
        return t_graph, float(ts.mean())

    def step_bytes(M):
        return sum(layer_alg_bytes(l.K, l.N, l.n8, M) + quant_alg_bytes(l.K, M) for l in layers)

    def step_ops(M):
        return sum(2.0 * M * l.K * l.N for l in layers)

    dom = max(range(len(layers)), key=lambda i: (layers[i].K * layers[i].N, layers[i].n8))   # gate_up (stack: its largest 8-bit share)

    def leg(M, steps, warmup, reps):
        first = len(executed)
        t = time_steps(M, steps, warmup)
        sec = t["mean"]
        k_graph, k_pair = time_dominant(M, reps, dom)
        launches = executed[first:]
        l = layers[dom]
        kb, ko = layer_alg_bytes(l.K, l.N, l.n8, M), 2.0 * M * l.K * l.N
        out = {"M": M, "launches": launches, "ms_per_step": sec * 1e3, "ms_per_step_median": t["median"] * 1e3,
               "ms_per_step_min": t["min"] * 1e3, "GBps": step_bytes(M) / sec / 1e9, "TOPS": step_ops(M) / sec / 1e12,
               # the step (quantizers + linears of all layers) and its dominant kernel against min(HBM, int8 MFMA)
               "step_roofline": roofline_entry(step_bytes(M), step_ops(M), sec),
               "dominant_kernel": {"layer": l.name, "us_per_launch": k_graph * 1e6,
                                   "us_with_own_event_pair": k_pair * 1e6,
                                   "GBps": kb / k_graph / 1e9, "TOPS": ko / k_graph / 1e12,
                                   "roofline": roofline_entry(kb, ko, k_graph)}}
        log(f"[bench] M={M}: {out['ms_per_step']:.4f} ms/step (median {out['ms_per_step_median']:.4f}, min "
            f"{out['ms_per_step_min']:.4f}), {out['GBps']:.0f} GB/s, {out['TOPS']:.1f} TOPS, "
            f"{out['step_roofline']['frac_of_min_hbm_mfma']:.2f} of min(HBM, MFMA); {l.name} kernel {k_graph * 1e6:.1f} us "
            f"per launch ({k_pair * 1e6:.1f} with its own event pair), {out['dominant_kernel']['roofline']['frac_of_min_hbm_mfma']:.2f}")
        return out

    decode_like = M0 <= 16
    primary = leg(M0, args.steps, args.warmup if decode_like else max(args.warmup, 40), min(args.steps, 200) if decode_like else 30)
    l = layers[dom]
    roof = dict(primary["dominant_kernel"]["roofline"])
    # HBM bytes per launch of that kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this
    # same command (scaled by a plain copy of known size); measured offline and kept under profiles/
    # together with a hash of the kernel's sources: a figure measured on other sources is not reported
    roof["traffic"] = None
    tpath = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "hbm_traffic.json")
    if os.path.exists(tpath) and args.workload in ("decode", "prefill"):
        rec = json.load(open(tpath)).get(("decode" if decode_like else "prefill") + f"_m{M0}_{l.name}")
        if isinstance(rec, dict):
            srcs = rec.get("sources", [])
            if rec.get("sources_sha16") == source_sha(*srcs):
                roof["traffic"] = rec.get("bytes")
            else:
                roof["traffic_note"] = "stored counter figure belongs to other kernel sources: not reported"
    roof["algorithmic"] = layer_alg_bytes(l.K, l.N, l.n8, M0) if roof["bound"] == "hbm" else 2.0 * M0 * l.K * l.N
    roof["kernel"] = f"mixed_linear {'decode' if decode_like else 'prefill'} path, layer {l.name} K={l.K} N={l.N} M={M0}"
    roof["us_per_launch"] = primary["dominant_kernel"]["us_per_launch"]

    what = {"decode": "Llama-3-8B-shaped decoder-block linears (QKV, O, gate+up, down)",
            "prefill": "Llama-3-8B-shaped decoder-block linears (QKV, O, gate+up, down)",
            "70b": "Llama-3.1-70B-shaped decoder-block linears (QKV, O, gate+up, down)",
            "stack": "32 Llama-3-8B-shaped decoder blocks back to back (128 linears), 8-bit share per layer 0..40 % (mean 10 %)"}
    result = {
        "metric": "mixed W4/W8-A8 linear TOPS + HBM GB/s at M=1..2048 (% roofline)",
        "value": primary["GBps"] if decode_like else primary["TOPS"],
        "unit": "GB/s" if decode_like else "TOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": primary["ms_per_step"], "ms_per_step_median": primary["ms_per_step_median"],
        "ms_per_step_min": primary["ms_per_step_min"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "config": {"workload": f"{what[args.workload]}, {'decode' if decode_like else 'prefill'} M={M0}, "
                               f"{'10% int8 channels' if args.workload != 'stack' else 'uneven int8 share'}, int4 g128, "
                               f"per-token int8 activations, fp16 out",
                   "M": M0, "weight_copies_rotated": n_copies},
        "step_GBps": primary["GBps"], "step_TOPS": primary["TOPS"],
        "step_roofline": primary["step_roofline"],
        "roofline": roof,
    }
    # order of the primary leg's linear launches, run-length encoded: [[layer names of one period], repeats]
    runs, seq, i = [], primary["launches"], 0
    period = list(range(len(layers)))
    while i < len(seq):
        if seq[i:i + len(period)] == period:
            pat = period
        else:
            pat = [seq[i]]
        n = 0
        while seq[i:i + len(pat)] == pat:
            n, i = n + 1, i + len(pat)
        runs.append([[layers[j].name for j in pat] if len(pat) <= 8 else f"all {len(pat)} linears in order", n])
    result["linear_launch_order"] = runs

    # ---- measured ceilings of this GPU (context for the published peaks) ----------------------
    if not args.no_extras:
        from paper_2412_14590_amd import probe
        result["measured_ceilings"] = {"hbm_read_GBps_4GiB": probe.hbm_read_gbs(),
                                       "mfma_int8_TOPS_register_resident": probe.mfma_int8_tops(4),
                                       "us_per_launch_of_a_near_empty_kernel_in_a_graph": probe.kernel_floor_us()}
        log(f"[bench] measured ceilings: {result['measured_ceilings']}")
    if args.copy_probe:
        from paper_2412_14590_amd import probe
        a = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        b = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        a.fill_(1)
        for _ in range(3):
            probe.copy(a, b)
        torch.cuda.synchronize()
        del a, b

    # ---- extra legs ------------------------------------------------------------------------
    if not args.no_extras:
        if args.workload == "70b":
            extra_ms = [m for m in (1, 16, 64, 256, 2048) if m != M0]
        elif args.workload == "stack":
            extra_ms = [m for m in (1, 256) if m != M0]
        else:
            extra_ms = [2, 4, 8, 16, 64, 256] if decode_like else [512, 8192]
        sweep = []
        for M in extra_ms:
            small = M <= 16
            sweep.append(leg(M, max(20, args.steps // 4) if small else 40, 5 if small else 40, 50 if small else 30))
        if args.workload in ("decode", "prefill"):
            other = leg(2048 if decode_like else 1, 40 if decode_like else 100, 40 if decode_like else 3, 30)
            other["roofline"] = other["dominant_kernel"]["roofline"]
            result["prefill" if decode_like else "decode"] = other
            sweep_all = sweep + [other]
        else:
            sweep_all = sweep
        for extra in sweep_all:
            del extra["launches"]
        result["sweep"] = sweep
    if not args.no_extras and args.workload in ("decode", "prefill"):
        # the paper's granularity (activation scales per token and group, 8-bit weight scales per
        # group): the whole step, same shapes, same launch method
        Wd = {k: torch.from_numpy(v[2]).to(dev) for k, v in kinds.items()}
        packed_p = [mx.quantize_weights(Wd[kind], lay.salient_idx, w8_group=128) for lay, (_, kind, _) in zip(layers, specs)]
        del Wd
        mode.update(copies=[packed_p] + [[p.clone() for p in packed_p] for _ in range(n_copies - 1)],
                    act_group=128, w8_group=128)
        gran = []
        for M in (1, 16, 2048):
            small = M <= 16
            t = time_steps(M, 50 if small else 40, 5 if small else 40)
            sec = t["mean"]
            gran.append({"M": M, "ms_per_step": sec * 1e3, "ms_per_step_median": t["median"] * 1e3, "ms_per_step_min": t["min"] * 1e3,
                         "GBps": step_bytes(M) / sec / 1e9, "TOPS": step_ops(M) / sec / 1e12,
                         "step_roofline": roofline_entry(step_bytes(M), step_ops(M), sec)})
            log(f"[bench] scales per group of 128 (activations and 8-bit weights), M={M}: {sec * 1e3:.4f} ms/step")
        result["paper_granularity"] = {"act_group": 128, "w8_group": 128, "legs": gran,
                                       "note": "GBps / TOPS use the algorithmic bytes / operations of the default granularity"}
        mode.update(copies=copies, act_group=None, w8_group=None)

    # ---- CPU baseline: the oracle as it stands, on a bounded sample ---------------------------
    if not args.no_cpu:
        from oracle import ref
        t1 = time.time()
        Ms = M0 if decode_like else 8       # prefill: a sample of 8 token rows of the same layers
        sample = list(range(min(4, len(layers))))     # stack: the four linears of the first block
        Ls = [ref.quantize_weights(layers[i].W, layers[i].salient_idx) for i in sample]
        log(f"[bench] oracle weight quantization {time.time() - t1:.1f}s (not timed)")
        xs_h = [synth.make_x(Ms, layers[i].K, seed=7, tag="x/" + specs[i][1]) for i in sample]
        reps, t_cpu = 0, 0.0
        while t_cpu < 10.0 and reps < 5000:
            t = time.perf_counter()
            for xh, L in zip(xs_h, Ls):
                xq, xsc = ref.quantize_act(xh)
                ref.mixed_linear(xq, xsc, L)
            t_cpu += time.perf_counter() - t
            reps += 1
        sec = t_cpu / reps
        sb = sum(layer_alg_bytes(layers[i].K, layers[i].N, layers[i].n8, Ms) + quant_alg_bytes(layers[i].K, Ms) for i in sample)
        so = sum(2.0 * Ms * layers[i].K * layers[i].N for i in sample)
        val = (sb / sec / 1e9) if decode_like else (so / sec / 1e12)
        result["cpu_baseline"] = {"value": val, "unit": result["unit"], "cores": ref.num_threads(), "kind": "oracle",
                                  "sample": f"{reps} passes of {'the same 4 layers' if len(layers) == 4 else 'the 4 layers of the first block'} "
                                            f"at M={Ms} tokens ({sec * 1e3:.1f} ms per pass), all channels, all groups"}
        log(f"[bench] cpu oracle: {val:.3g} {result['unit']} on {ref.num_threads()} threads")

    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
