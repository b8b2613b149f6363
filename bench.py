"""Benchmark of the VATP hot path on one MI355X.

One "step" is one pass of the whole hot path over one batch of synthetic input that is
already resident in HBM: prompt scoring (vatp_prefill_score), the prompt prune
(vatp_select_compact), then T decode steps, each followed by the eviction back to the budget,
for every layer of the workload: by default through vatp_decode_prune_step (only the rows that
changed are rewritten), with --decode-route separate through vatp_decode_step +
vatp_select_compact (three launches, the whole cache is copied every step).

The default workload is the largest one that fits one GPU, llama7b_stack (32 layers, batch 8,
prompt 4096, 256 decode steps: 25.8 GB of prompt tensors, 2.3 GB touched per token step), whose
figures are the headline fields of the ONE JSON line printed.  With the default workload the
line also carries `per_workload`: the same measurements, in short, for the other four named
workloads (fewer timed steps each).  The byte and flop formulas behind `roofline` are the
algorithmic_* functions below.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
import traceback

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import torch  # noqa: E402

import vatp_synth as vs  # noqa: E402

HBM_PEAK_GBPS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0
FP32_VECTOR_PEAK_TFLOPS = 157.3


def algorithmic_flops_prefill(cfg, lens, window=None):
    """Both scoring passes, causal lower triangle only: 2 passes * 2*d flops per (query, key<=query) pair and
    query head (n_heads counts K/V heads, each with q_per_kv query heads); with a history window only the last
    window+1 query rows count."""
    def pairs(L):
        first = 0 if window is None else max(0, L - 1 - window)
        return (L * (L + 1) - first * (first + 1)) // 2
    return sum(cfg.n_heads * cfg.q_per_kv * 2 * 2 * cfg.head_dim * pairs(L) for L in lens) * cfg.layers


def algorithmic_bytes_decode(cfg, n_rows, budget):
    """(decode_step bytes, select_compact bytes) for one unit with n_rows rows after the append."""
    elt = 4 if cfg.dtype == "fp32" else 2
    row = cfg.head_dim * elt
    keep = min(n_rows, budget)
    score = n_rows * row + 8 * n_rows                 # K read once; S read + written
    select = 8 * n_rows + 4 * keep                    # S, nrm read; kept_idx written
    compact = 4 * row * keep + 24 * keep              # K, V rows read + written; S, nrm, pos read + written
    return score, select + compact


def algorithmic_bytes_fused(cfg, n_rows, budget, rows_moved):
    """vatp_decode_prune_step for one unit: K read once, S and nrm read, the new scores written, and
    only the rows from the first changed one on copied to the other cache set (K, V, nrm, pos)."""
    elt = 4 if cfg.dtype == "fp32" else 2
    row = cfg.head_dim * elt
    keep = min(n_rows, budget)
    return n_rows * row + 8 * n_rows + 4 * keep + rows_moved * (4 * row + 16)


def algorithmic_bytes_window(cfg, n_rows, window, rows_moved):
    """Extra bytes of the history-window step per unit: the leaving weight read and the new one written
    per row (plus the row's column index), the new row's column cleared, and the column index moved."""
    return 12 * n_rows + 4 * window + 8 * rows_moved


def fused_step_kernels(cfg, lens, budgets, window):
    """Names of the kernels one vatp_decode_prune_step call launches for this workload (the library's rule:
    a single launch with one workgroup per head when there are at least 128 heads of at most 1024 rows and
    neither grouped queries nor a history window; otherwise the logits launch plus the evict-and-copy launch)."""
    rows = max(min(L, B) for L, B in zip(lens, budgets)) + 1
    if window is None and cfg.q_per_kv == 1 and cfg.batch * cfg.n_heads >= 128 and rows <= 1024:
        return "decode_prune_one_kernel"
    first = "decode_logits_group_kernel" if cfg.q_per_kv > 1 else "decode_logits_kernel"
    return first + " + decode_prune_kernel"


def measure(args, workload, steps, warmup, main_line):
    """Runs one workload and returns its JSON object.  main_line: this is the workload of the headline fields
    (machine yardsticks, input digests and the CPU baseline are taken only there)."""
    from paper_2406_12335_amd.runner import PrunedKVCache
    import paper_2406_12335_amd as vatp

    dev = torch.device("cuda:0")
    cfg = vs.CONFIGS[workload]
    if args.layers:
        cfg = vs.scaled(cfg, layers=args.layers)
    if args.decode_steps is not None:
        cfg = vs.scaled(cfg, decode_steps=args.decode_steps)
    for field, value in (("batch", args.batch), ("budget_pct", args.budget_pct), ("recent", args.recent),
                         ("n_heads", args.heads), ("q_per_kv", args.q_per_kv)):
        if value is not None:
            cfg = vs.scaled(cfg, **{field: value})
    T = cfg.decode_steps
    fused = args.decode_route == "fused"
    window = args.window
    layers = [vs.make_inputs(cfg, seed=args.seed, layer=l, device=dev) for l in range(cfg.layers)]
    digests = {}
    if main_line:
        for l in range(min(cfg.layers, args.digest_layers)):
            digests.update({"layer%d.%s" % (l, k): v[:16] for k, v in vs.buffer_digests(layers[l]).items()})
    lens, budgets = layers[0].lens, layers[0].budgets
    for inp in layers:      # per-step views of the new tokens, made once (indexing costs host time per call)
        inp.step_qkv = [(inp.qd[t], inp.kd[t], inp.vd[t]) for t in range(T)]
    ctx = vatp.vatp_create(0)
    caches = [PrunedKVCache(cfg.batch, cfg.n_heads, cfg.head_dim, cfg.torch_dtype(), cfg.n_sink_keep, cfg.recent,
                            budgets, dev, ctx=ctx, window=window, q_per_kv=cfg.q_per_kv) for _ in layers]
    new_pos = [[L + t for L in lens] for t in range(T)]

    def one_step(ev=None):
        """ev: optional dict of event lists, filled with (start, end) pairs per phase."""
        def mark():
            e = torch.cuda.Event(enable_timing=True)
            e.record()
            return e
        for inp, cache in zip(layers, caches):
            e0 = mark() if ev is not None else None
            cache.prefill_score(inp.Q, inp.K, inp.V, lens)
            e1 = mark() if ev is not None else None
            cache.prune_prompt(inp.K, inp.V)
            e2 = mark() if ev is not None else None
            if ev is not None:
                ev["prefill_score"].append((e0, e1))
                ev["prompt_prune"].append((e1, e2))
        e3 = mark() if ev is not None else None
        for t in range(T):
            for inp, cache in zip(layers, caches):
                if fused:
                    cache.decode_prune_step(*inp.step_qkv[t], new_pos[t])
                else:
                    cache.decode_step(*inp.step_qkv[t], new_pos[t])
                    cache.prune()
        if ev is not None:
            ev["decode_loop"].append((e3, mark()))

    copy_gbps = gemm_tflops = None
    if args.copy_calibration and main_line:
        src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device=dev)          # 256 MiB
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.neg(src, out=dst)               # reads 256 MiB, writes 256 MiB (an op nothing else in this file uses)
        torch.cuda.synchronize()
        del src, dst

    if main_line:
        # yardstick beside the data-sheet HBM figure: what a plain device-to-device copy reaches here
        src = torch.empty(128 * 1024 * 1024, dtype=torch.float32, device=dev).normal_()      # 512 MiB
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        c0.record()
        for _ in range(10):
            dst.copy_(src)
        c1.record()
        torch.cuda.synchronize()
        copy_gbps = 10 * 2 * src.numel() * 4 / (c0.elapsed_time(c1) * 1e-3) / 1e9
        del src, dst
        # the vendor library's bf16 GEMM (8192^3, random operands): what the matrix cores sustain here on a plain product
        ga = torch.randn(8192, 8192, device=dev).to(torch.bfloat16)
        gb = torch.randn(8192, 8192, device=dev).to(torch.bfloat16)
        for _ in range(3):
            gc = torch.matmul(ga, gb)
        torch.cuda.synchronize()
        c0.record()
        for _ in range(5):
            gc = torch.matmul(ga, gb)
        c1.record()
        torch.cuda.synchronize()
        gemm_tflops = 5 * 2 * 8192 ** 3 / (c0.elapsed_time(c1) * 1e-3) / 1e12
        del ga, gb, gc

    for _ in range(warmup):
        one_step()
    torch.cuda.synchronize()
    ev = {"prefill_score": [], "prompt_prune": [], "decode_loop": []}
    t0 = time.perf_counter()
    for _ in range(steps):
        one_step(ev)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / steps

    def total_ms(pairs):
        return sum(a.elapsed_time(b) for a, b in pairs)

    prefill_ms = total_ms(ev["prefill_score"]) / steps          # all layers of one step
    prune_ms = total_ms(ev["prompt_prune"]) / steps
    decode_ms = total_ms(ev["decode_loop"]) / steps

    # Replays outside the timed region.  Each is a loop bracketed by ONE pair of events on the stream
    # the library launches on (event pairs around single calls inside a deep queue proved unreliable).
    def timed(fn):
        a = torch.cuda.Event(enable_timing=True); a.record()
        fn()
        b = torch.cuda.Event(enable_timing=True); b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b)

    def reset():
        for inp, cache in zip(layers, caches):
            cache.prefill_score(inp.Q, inp.K, inp.V, lens)
            cache.prune_prompt(inp.K, inp.V)
        torch.cuda.synchronize()

    n_calls = max(1, T * cfg.layers)
    sep_loop_ms = dec_call_ms = sel_call_ms = 0.0
    if window is None and T:
        # (1) the decode loop through the separate calls
        def separate_loop():
            for t in range(T):
                for inp, cache in zip(layers, caches):
                    cache.decode_step(*inp.step_qkv[t], new_pos[t])
                    cache.prune()
        reset()
        sep_loop_ms = timed(separate_loop)
        # (2) each entry point by itself, T calls on the steady-state shape (the cache holds its budget, the
        # step appends one row, the prune removes one): the row counts are put back after every call
        reset()
        base = [list(c.lens) for c in caches]

        def decode_only():
            for t in range(T):
                for inp, cache, n0 in zip(layers, caches, base):
                    cache.decode_step(*inp.step_qkv[t], new_pos[t])
                    cache.lens = list(n0)
        dec_call_ms = timed(decode_only) / n_calls
        for inp, cache in zip(layers, caches):
            cache.decode_step(*inp.step_qkv[0], new_pos[0])
        grown = [(c.cur, list(c.lens)) for c in caches]

        def prune_only():
            for t in range(T):
                for cache, (cur0, n1) in zip(caches, grown):
                    cache.prune()
                    cache.cur, cache.lens = cur0, list(n1)
        sel_call_ms = timed(prune_only) / n_calls

    # (3) the fused route: whole loop timed; in a second pass the per-head count of rows it had to move is
    # read back after every step (min of the two `synced` arrays = first rewritten row)
    fused_bytes, fused_rows_moved = 0, 0
    host_us_per_call = 0.0

    def fused_loop():
        # host cost of enqueueing one call: taken over the first calls only, while the device queue still has room
        # (once it is full the host waits for the GPU and the figure would just repeat the GPU's time per call)
        nonlocal host_us_per_call
        probe = min(n_calls, 192)
        done = 0
        t_host = time.perf_counter()
        for t in range(T):
            for inp, cache in zip(layers, caches):
                cache.decode_prune_step(*inp.step_qkv[t], new_pos[t])
                done += 1
                if done == probe:
                    host_us_per_call = (time.perf_counter() - t_host) * 1e6 / probe
    reset()
    fused_call_ms = timed(fused_loop) / n_calls
    reset()
    for t in range(T):
        for inp, cache in zip(layers, caches):
            n_after = [n + 1 for n in cache.lens]
            cache.decode_prune_step(*inp.step_qkv[t], new_pos[t])
            first = torch.minimum(cache.synced[0], cache.synced[1]).view(cfg.batch, cfg.n_heads).cpu()
            for bb in range(cfg.batch):
                keep = min(n_after[bb], budgets[bb])
                moved = (keep - first[bb]).clamp_(min=0)
                fused_rows_moved += int(moved.sum())
                fused_bytes += sum(algorithmic_bytes_fused(cfg, n_after[bb], budgets[bb], int(m)) for m in moved)
                if window is not None:
                    fused_bytes += sum(algorithmic_bytes_window(cfg, n_after[bb], window, int(m)) for m in moved)
    torch.cuda.synchronize()

    # algorithmic work
    flops = algorithmic_flops_prefill(cfg, lens, window)
    n_tokens = sum(lens) * cfg.layers
    dec_bytes = sel_bytes = 0          # over the T steps of the trajectory (the separate route's loop)
    dec_call_bytes = sel_call_bytes = 0   # one call at the steady-state shape (the isolated loops)
    cur = [min(L, B) for L, B in zip(lens, budgets)]
    for b in range(cfg.batch):
        s, c = algorithmic_bytes_decode(cfg, cur[b] + 1, budgets[b])
        dec_call_bytes += s * cfg.n_heads
        sel_call_bytes += c * cfg.n_heads
    for t in range(T):
        for b in range(cfg.batch):
            s, c = algorithmic_bytes_decode(cfg, cur[b] + 1, budgets[b])
            dec_bytes += s * cfg.n_heads
            sel_bytes += c * cfg.n_heads
        cur = [min(n + 1, B) for n, B in zip(cur, budgets)]
    dec_bytes *= cfg.layers
    sel_bytes *= cfg.layers

    mfma = cfg.dtype == "bf16"
    peak_tf = MFMA_BF16_PEAK_TFLOPS if mfma else FP32_VECTOR_PEAK_TFLOPS
    # (only for the named workloads as they are: an overridden shape, grouped queries or a window have no profile)
    as_named = window is None and cfg == vs.CONFIGS.get(cfg.name)
    profiled = PROFILED_TRAFFIC_BYTES.get(cfg.name if as_named else None, {})
    traffic = profiled.get("bytes_per_call", {})
    prefill_tflops = flops / (prefill_ms * 1e-3) / 1e12 if prefill_ms > 0 else 0.0
    prefill_kernels = "prefill_mfma_kernel<rowstat> + prefill_mfma_kernel<colsum, value norms inside>" \
        if mfma and cfg.head_dim == 128 else "l1norm_kernel + prefill_rowstat_generic + prefill_colsum_generic"
    roof_prefill = {"kernel": "vatp_prefill_score = " + prefill_kernels if window is None
                    else "vatp_prefill_score_window = rowstat over key ranges + merge + colsum with rows and norms",
                    "bound": "mfma" if mfma else "alu",
                    "achieved": round(prefill_tflops, 3), "peak": peak_tf, "unit": "TFLOP/s",
                    "frac": round(prefill_tflops / peak_tf, 5), "traffic": traffic.get("prefill_score"),
                    "avg_launch_ms": round(prefill_ms / cfg.layers, 5),
                    # both passes recompute the logits; the rate of distinct (query, key) products is half of `achieved`
                    "single_pass_TFLOPs": round(prefill_tflops / 2, 3)}
    loop_bytes = fused_bytes if fused else dec_bytes + sel_bytes
    decode_gbps = loop_bytes / (decode_ms * 1e-3) / 1e9 if decode_ms > 0 and T else 0.0
    # the fused call's duration: from the events around the decode loops of the timed steps when that loop ran
    # through it (the default), else from the replay
    fused_ms_per_call = decode_ms / n_calls if fused and T else fused_call_ms
    fused_gbps = fused_bytes / n_calls / (fused_ms_per_call * 1e-3) / 1e9 if T and fused_ms_per_call > 0 else 0.0
    fused_kernels = fused_step_kernels(cfg, lens, budgets, window)
    roof_fused = {"kernel": ("vatp_decode_prune_step = " if window is None else "vatp_decode_prune_step_window = ") + fused_kernels,
                  "bound": "hbm",
                  "achieved": round(fused_gbps, 2), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                  "frac": round(fused_gbps / HBM_PEAK_GBPS, 5), "traffic": traffic.get("decode_prune_step"),
                  "avg_launch_ms": round(fused_ms_per_call, 5),
                  "algorithmic_bytes_per_call": int(fused_bytes / n_calls),
                  "host_enqueue_us_per_call": round(host_us_per_call, 2),
                  # for orientation only, not used in `achieved`: the bytes the out-of-place route moves for the
                  # same step (K read, S read + written, whole cache copied), over this route's time
                  "out_of_place_equivalent_GBps": round((dec_bytes + sel_bytes) / n_calls / (fused_ms_per_call * 1e-3) / 1e9, 2)
                  if T and fused_ms_per_call > 0 and window is None else None,
                  "rows_moved_per_head_step": round(fused_rows_moved / max(1, n_calls * cfg.batch * cfg.n_heads), 2)}
    dec_k_gbps = dec_call_bytes / (dec_call_ms * 1e-3) / 1e9 if T and dec_call_ms > 0 else 0.0
    sel_k_gbps = sel_call_bytes / (sel_call_ms * 1e-3) / 1e9 if T and sel_call_ms > 0 else 0.0
    roof_decode = {"kernel": "vatp_decode_step = decode_logits_kernel + decode_finish_kernel", "bound": "hbm",
                   "achieved": round(dec_k_gbps, 2), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                   "frac": round(dec_k_gbps / HBM_PEAK_GBPS, 5), "traffic": traffic.get("decode_step"),
                   "avg_launch_ms": round(dec_call_ms, 5), "algorithmic_bytes_per_call": dec_call_bytes}
    roof_gather = {"kernel": "vatp_select_compact = gather_kernel (evict-one select + compact)", "bound": "hbm",
                   "achieved": round(sel_k_gbps, 2), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                   "frac": round(sel_k_gbps / HBM_PEAK_GBPS, 5), "traffic": traffic.get("select_compact"),
                   "avg_launch_ms": round(sel_call_ms, 5), "algorithmic_bytes_per_call": sel_call_bytes}
    if fused:
        phases = {"prefill_score": prefill_ms, "decode_prune_step": fused_ms_per_call * n_calls}
    else:
        phases = {"prefill_score": prefill_ms, "decode_step": dec_call_ms * n_calls,
                  "select_compact": sel_call_ms * n_calls}
    dominant = max(phases, key=phases.get)
    roofline_all = {"prefill_score": roof_prefill, "decode_prune_step": roof_fused}
    if window is None:
        roofline_all.update({"decode_step": roof_decode, "select_compact": roof_gather})
    roofline = dict(roofline_all[dominant])
    # `traffic` is not counted in this run: it is the figure of the committed rocprofv3 counter summary named here
    roofline["traffic_source"] = profiled.get("source") if roofline.get("traffic") is not None else None

    out = {
        "metric": "prefill scoring tokens/s (% MFMA peak) + decode prune step GB/s (% HBM peak)",
        "value": round(n_tokens / (prefill_ms * 1e-3), 1) if prefill_ms > 0 else 0.0,
        "unit": "tokens/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if mfma else "f32", "data": "synthetic",
        "config": {"workload": cfg.name, "batch": cfg.batch, "layers": cfg.layers, "n_heads": cfg.n_heads,
                   "q_per_kv": cfg.q_per_kv,
                   "head_dim": cfg.head_dim, "prompt_len": lens if cfg.ragged else cfg.prompt_len,
                   "budget_pct": cfg.budget_pct, "recent": cfg.recent, "n_sink": cfg.n_sink_keep,
                   "decode_steps": T, "decode_route": args.decode_route, "score": "accumulated (Eq. 2)" if window is None
                   else "history window w=%d (Eq. 3)" % window,
                   "kept_idx_written_every_step": True},
        "prefill_ms": round(prefill_ms, 4), "prompt_prune_ms": round(prune_ms, 4), "decode_loop_ms": round(decode_ms, 4),
        "prefill_pct_mfma_peak": round(100 * roof_prefill["frac"], 3) if mfma else None,
        "decode_prune_GBps": round(decode_gbps, 2),
        "decode_prune_pct_hbm_peak": round(100 * decode_gbps / HBM_PEAK_GBPS, 3),
        "roofline": roofline,
        "roofline_all": roofline_all,
        # the same decode loop through either route (event times of replays outside the timed steps)
        "decode_loop_ms_by_route": {"fused": round(fused_call_ms * n_calls / 1, 4),
                                    "separate": round(sep_loop_ms, 4) if window is None else None},
    }
    if main_line:
        # read + write rate of a plain 512 MiB device copy (torch copy_) on this machine, for comparison with
        # the 8000 GB/s data-sheet figure the fractions are taken against
        out["measured_copy_GBps"] = round(copy_gbps, 1)
        # rate of the vendor library's 8192^3 bf16 GEMM on this machine, beside the 2500 TFLOP/s data-sheet figure
        out["measured_gemm_TFLOPs"] = round(gemm_tflops, 1)
        # first 16 hex digits of the SHA-256 of each generated buffer (seed %d; see vatp_synth.buffer_digests)
        out["input_sha256"] = digests
        if not args.no_cpu_baseline:
            out["cpu_baseline"] = cpu_baseline(cfg, layers[0], args.cpu_seconds)
    for c in caches:
        c.close()
    vatp.vatp_destroy(ctx)
    return out


def condensed(r):
    """The figures of one workload that go into `per_workload`."""
    keep = ("kernel", "bound", "achieved", "peak", "unit", "frac", "traffic", "avg_launch_ms")
    return {"config": r["config"], "dtype": r["dtype"], "steps": r["steps"], "warmup": r["warmup"],
            "value": r["value"], "unit": r["unit"], "ms_per_step": r["ms_per_step"],
            "prefill_ms": r["prefill_ms"], "prompt_prune_ms": r["prompt_prune_ms"], "decode_loop_ms": r["decode_loop_ms"],
            "decode_loop_ms_by_route": r["decode_loop_ms_by_route"],
            "roofline_all": {k: {f: v[f] for f in keep} for k, v in r["roofline_all"].items()}}


def run(args):
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (got --gpus %d)" % args.gpus, file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    if args.window is not None and args.decode_route != "fused":
        print("bench.py: history-window scores run through the fused decode route only", file=sys.stderr)
        sys.exit(2)
    import paper_2406_12335_amd as vatp
    vatp.load()
    torch.cuda.set_device(0)
    out = measure(args, args.workload, args.steps, args.warmup, True)
    overridden = any(v is not None for v in (args.batch, args.budget_pct, args.recent, args.heads, args.q_per_kv,
                                             args.decode_steps, args.window)) or args.layers
    if args.workload == DEFAULT_WORKLOAD and not args.no_per_workload and not overridden:
        # the other named workloads, in short; a failure there is reported in its entry and does not cost the line
        out["per_workload"] = {}
        for name in ("tiny", "llama7b_layer", "long32k", "ragged16"):
            torch.cuda.empty_cache()
            try:
                out["per_workload"][name] = condensed(measure(args, name, args.other_steps, 1, False))
            except Exception as e:      # noqa: BLE001
                out["per_workload"][name] = {"error": "%s: %s" % (type(e).__name__, e),
                                             "traceback": traceback.format_exc().splitlines()[-3:]}
    print(json.dumps(out), flush=True)


DEFAULT_WORKLOAD = "llama7b_stack"

# HBM bytes per call of an entry point (fetch + write, all of its kernels), as counted by rocprofv3 --pmc
# FETCH_SIZE / WRITE_SIZE runs of this file and scaled by what the same counters read for the plain copy of
# --copy-calibration.  NOT measured by the run that prints them: a static table, copied from the committed
# summary named in "source", which also gives the commands and the commit of the kernels they were counted on.
PROFILED_TRAFFIC_BYTES = {
    "llama7b_stack": {"source": "profiles/llama7b_stack_profile.md",
                      "bytes_per_call": {"prefill_score": 2066138097, "decode_step": 57657290, "select_compact": 232478387,
                                         "decode_prune_step": 71321155}},
    "llama7b_layer": {"source": "profiles/llama7b_layer_profile.md",
                      "bytes_per_call": {"prefill_score": 185835398, "decode_step": 18042753, "select_compact": 72825985,
                                         "decode_prune_step": 21342131}},
    "long32k": {"source": "profiles/long32k_profile.md",
                "bytes_per_call": {"prefill_score": 2388075236, "decode_step": 28734910, "select_compact": 116525482,
                                   "decode_prune_step": 35609948}},
    "ragged16": {"source": "profiles/ragged16_profile.md",
                 "bytes_per_call": {"prefill_score": 5967520750, "decode_step": 204590432, "select_compact": 830405693,
                                    "decode_prune_step": 250674872}},
    "tiny": {"source": "profiles/tiny_profile.md",
             "bytes_per_call": {"prefill_score": 2462884, "decode_step": 258267, "select_compact": 594541,
                                "decode_prune_step": 525967}},
}


def cpu_baseline(cfg, inp, budget_s):
    """The float64 oracle, as it stands, timed on this machine's host cores on a bounded sample of
    the same workload: prompt scoring of sequence 0 (all heads, one layer, prompt truncated only if
    the estimate exceeds the time budget) and a few decode-and-prune steps at the steady-state size."""
    import numpy as np
    from oracle import vatp_oracle as orc
    threads = orc.max_threads()
    L, B = inp.lens[0], inp.budgets[0]
    H, d = cfg.n_heads, cfg.head_dim
    est_rate = 0.6e9 * threads                         # (query, key) pairs * d per second, rough
    Ls = L
    grp = cfg.q_per_kv
    while Ls > 256 and grp * H * (Ls * Ls / 2) * d / est_rate > budget_s:
        Ls //= 2
    Q = inp.Q[0, :, :Ls].double().cpu().numpy()
    K = inp.K[0, :, :Ls].double().cpu().numpy()
    t0 = time.perf_counter()
    if grp == 1:
        orc.prefill_scores_units(Q, K, [Ls] * H)
    else:
        orc.prefill_scores_group_units(Q.reshape(H, grp, Ls, d), K, [Ls] * H)
    dt = time.perf_counter() - t0
    out = {"value": round(Ls / dt, 2), "unit": "tokens/s", "cores": threads, "kind": "oracle",
           "sample": "prompt scoring (both softmax passes of the float64 oracle), all %d heads of one layer, "
                     "first %d of %d prompt tokens of sequence 0; %.2f s" % (H * grp, Ls, L, dt)}
    if grp > 1:
        return out          # (the oracle's many-heads decode routine takes one query per K/V head)
    # decode + prune at the steady-state cache size n = B + 1, a few steps, all heads of sequence 0
    n = min(B, L) + 1
    import ctypes
    rng = np.random.default_rng(0)
    Kc = np.ascontiguousarray(inp.K[0, :, :n].double().cpu().numpy()) if n <= inp.K.shape[2] else rng.standard_normal((H, n, d))
    Vc = np.ascontiguousarray(inp.V[0, :, :n].double().cpu().numpy()) if n <= inp.V.shape[2] else rng.standard_normal((H, n, d))
    Sc = rng.random((H, n)) + 0.1
    nr = np.abs(Vc).sum(-1)
    qv = inp.qd[0, 0].double().cpu().numpy() if inp.qd.shape[0] else rng.standard_normal((H, d))
    Ko, Vo, So, No = np.zeros_like(Kc), np.zeros_like(Vc), np.zeros_like(Sc), np.zeros_like(Sc)
    kept = np.zeros((H, n), dtype=np.int32)
    n_arr = np.full(H, n, dtype=np.int64); B_arr = np.full(H, n - 1, dtype=np.int64); n_out = np.zeros(H, dtype=np.int64)
    f64 = lambda a: a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))
    i64 = lambda a: a.ctypes.data_as(ctypes.POINTER(ctypes.c_int64))
    if n - 1 >= cfg.n_sink_keep + cfg.recent:
        steps = 16
        t0 = time.perf_counter()
        for _ in range(steps):
            orc.lib().vatp_oracle_decode_prune_units(f64(qv), f64(Kc), f64(Vc), f64(Sc), f64(nr), H, n, i64(n_arr), d,
                                                     orc.default_scale(d), i64(B_arr), cfg.n_sink_keep, cfg.recent,
                                                     f64(Ko), f64(Vo), f64(So), f64(No),
                                                     kept.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), i64(n_out))
        dt2 = (time.perf_counter() - t0) / steps
        s_bytes, c_bytes = algorithmic_bytes_decode(cfg, n, n - 1)
        out["decode_prune_GBps"] = round((s_bytes + c_bytes) * H / dt2 / 1e9, 3)
        out["sample"] += "; decode+prune: %d steps at n=%d rows, all heads of sequence 0, %.3f s per step, GB/s over the " \
                         "same algorithmic bytes as the GPU figure" % (steps, n, dt2)
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default=DEFAULT_WORKLOAD, choices=sorted(vs.CONFIGS))
    ap.add_argument("--no-per-workload", action="store_true",
                    help="with the default workload: leave out the short measurements of the other four workloads")
    ap.add_argument("--other-steps", type=int, default=3, help="timed steps of each workload in per_workload")
    ap.add_argument("--digest-layers", type=int, default=1,
                    help="layers whose generated buffers are hashed (SHA-256) into the line; 0 = none")
    ap.add_argument("--layers", type=int, default=0, help="override the number of layers of the workload")
    ap.add_argument("--decode-steps", type=int, default=None)
    ap.add_argument("--batch", type=int, default=None, help="override the batch size of the workload")
    ap.add_argument("--budget-pct", type=int, default=None, help="override the KV budget (percent of the prompt)")
    ap.add_argument("--recent", type=int, default=None, help="override the recent window R")
    ap.add_argument("--heads", type=int, default=None, help="override the number of (K/V) heads of the workload")
    ap.add_argument("--q-per-kv", type=int, default=None,
                    help="grouped-query attention: query heads per K/V head (default 1, the paper's models)")
    ap.add_argument("--decode-route", default="fused", choices=["fused", "separate"],
                    help="fused: vatp_decode_prune_step; separate: vatp_decode_step + vatp_select_compact")
    ap.add_argument("--window", type=int, default=None,
                    help="history-window scores (Eq. 3) with this window instead of accumulated scores (Eq. 2)")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=15.0)
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also launch three plain 256 MiB -> 256 MiB element-wise kernels (torch.neg: a known traffic "
                         "figure to scale rocprofv3's FETCH_SIZE / WRITE_SIZE against)")
    run(ap.parse_args())


if __name__ == "__main__":
    main()
