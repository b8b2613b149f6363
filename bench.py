"""Benchmark of the VATP hot path on one MI355X.

One "step" is one pass of the whole hot path over one batch of synthetic input that is
already resident in HBM: prompt scoring (vatp_prefill_score), the prompt prune
(vatp_select_compact), then T decode steps of vatp_decode_step + vatp_select_compact, for
every layer of the workload.  Prints ONE JSON line (see the design doc for the byte and flop
formulas behind `roofline`).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import torch  # noqa: E402

import vatp_synth as vs  # noqa: E402

HBM_PEAK_GBPS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0
FP32_VECTOR_PEAK_TFLOPS = 157.3


def algorithmic_flops_prefill(cfg, lens):
    """Both scoring passes, causal lower triangle only: 2 passes * 2*d flops per (query, key<=query) pair."""
    return sum(cfg.n_heads * 2 * 2 * cfg.head_dim * (L * (L + 1) // 2) for L in lens) * cfg.layers


def algorithmic_bytes_decode(cfg, n_rows, budget):
    """(decode_step bytes, select_compact bytes) for one unit with n_rows rows after the append."""
    elt = 4 if cfg.dtype == "fp32" else 2
    row = cfg.head_dim * elt
    keep = min(n_rows, budget)
    score = n_rows * row + 8 * n_rows                 # K read once; S read + written
    select = 8 * n_rows + 4 * keep                    # S, nrm read; kept_idx written
    compact = 4 * row * keep + 24 * keep              # K, V rows read + written; S, nrm, pos read + written
    return score, select + compact


def run(args):
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (got --gpus %d)" % args.gpus, file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    from paper_2406_12335_amd.runner import PrunedKVCache
    import paper_2406_12335_amd as vatp
    vatp.load()

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    cfg = vs.CONFIGS[args.workload]
    if args.layers:
        cfg = vs.scaled(cfg, layers=args.layers)
    if args.decode_steps is not None:
        cfg = vs.scaled(cfg, decode_steps=args.decode_steps)
    T = cfg.decode_steps
    layers = [vs.make_inputs(cfg, seed=args.seed, layer=l, device=dev) for l in range(cfg.layers)]
    lens, budgets = layers[0].lens, layers[0].budgets
    ctx = vatp.vatp_create(0)
    caches = [PrunedKVCache(cfg.batch, cfg.n_heads, cfg.head_dim, cfg.torch_dtype(), cfg.n_sink_keep, cfg.recent,
                            budgets, dev, ctx=ctx) for _ in layers]
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
                cache.decode_step(inp.qd[t], inp.kd[t], inp.vd[t], new_pos[t])
                cache.prune()
        if ev is not None:
            ev["decode_loop"].append((e3, mark()))

    if args.copy_calibration:
        src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device=dev)          # 256 MiB
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.mul(src, 1.0, out=dst)          # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        one_step()
    torch.cuda.synchronize()
    ev = {"prefill_score": [], "prompt_prune": [], "decode_loop": []}
    t0 = time.perf_counter()
    for _ in range(args.steps):
        one_step(ev)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps

    def total_ms(pairs):
        return sum(a.elapsed_time(b) for a, b in pairs)

    prefill_ms = total_ms(ev["prefill_score"]) / args.steps          # all layers of one step
    prune_ms = total_ms(ev["prompt_prune"]) / args.steps
    decode_ms = total_ms(ev["decode_loop"]) / args.steps

    # instrumented replay (outside the timed region): split the decode loop per entry point
    split = {"decode_step": [], "select_compact": []}
    for inp, cache in zip(layers, caches):
        cache.prefill_score(inp.Q, inp.K, inp.V, lens)
        cache.prune_prompt(inp.K, inp.V)
    for t in range(T):
        for inp, cache in zip(layers, caches):
            a = torch.cuda.Event(enable_timing=True); a.record()
            cache.decode_step(inp.qd[t], inp.kd[t], inp.vd[t], new_pos[t])
            b = torch.cuda.Event(enable_timing=True); b.record()
            cache.prune()
            c = torch.cuda.Event(enable_timing=True); c.record()
            split["decode_step"].append((a, b))
            split["select_compact"].append((b, c))
    torch.cuda.synchronize()
    n_calls = max(1, T * cfg.layers)
    dec_call_ms = total_ms(split["decode_step"]) / n_calls
    sel_call_ms = total_ms(split["select_compact"]) / n_calls

    # algorithmic work
    flops = algorithmic_flops_prefill(cfg, lens)
    n_tokens = sum(lens) * cfg.layers
    dec_bytes = sel_bytes = 0
    cur = [min(L, B) for L, B in zip(lens, budgets)]
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
    prefill_tflops = flops / (prefill_ms * 1e-3) / 1e12 if prefill_ms > 0 else 0.0
    roof_prefill = {"kernel": "vatp_prefill_score (l1norm + rowstat + colsum)", "bound": "mfma" if mfma else "alu",
                    "achieved": round(prefill_tflops, 3), "peak": peak_tf, "unit": "TFLOP/s",
                    "frac": round(prefill_tflops / peak_tf, 5), "traffic": None,
                    "avg_launch_ms": round(prefill_ms / cfg.layers, 5)}
    decode_gbps = (dec_bytes + sel_bytes) / (decode_ms * 1e-3) / 1e9 if decode_ms > 0 and T else 0.0
    dec_k_gbps = dec_bytes / n_calls / (dec_call_ms * 1e-3) / 1e9 if T and dec_call_ms > 0 else 0.0
    sel_k_gbps = sel_bytes / n_calls / (sel_call_ms * 1e-3) / 1e9 if T and sel_call_ms > 0 else 0.0
    roof_decode = {"kernel": "decode_score_kernel", "bound": "hbm", "achieved": round(dec_k_gbps, 2),
                   "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(dec_k_gbps / HBM_PEAK_GBPS, 5),
                   "traffic": None, "avg_launch_ms": round(dec_call_ms, 5)}
    roof_gather = {"kernel": "gather_kernel (evict-one select + compact)", "bound": "hbm",
                   "achieved": round(sel_k_gbps, 2), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                   "frac": round(sel_k_gbps / HBM_PEAK_GBPS, 5), "traffic": None,
                   "avg_launch_ms": round(sel_call_ms, 5)}
    phases = {"prefill_score": prefill_ms, "decode_step": dec_call_ms * n_calls, "select_compact": sel_call_ms * n_calls}
    dominant = max(phases, key=phases.get)
    roofline = {"prefill_score": roof_prefill, "decode_step": roof_decode, "select_compact": roof_gather}[dominant]

    out = {
        "metric": "prefill scoring tokens/s (% MFMA peak) + decode prune step GB/s (% HBM peak)",
        "value": round(n_tokens / (prefill_ms * 1e-3), 1) if prefill_ms > 0 else 0.0,
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if mfma else "f32", "data": "synthetic",
        "config": {"workload": cfg.name, "batch": cfg.batch, "layers": cfg.layers, "n_heads": cfg.n_heads,
                   "head_dim": cfg.head_dim, "prompt_len": lens if cfg.ragged else cfg.prompt_len,
                   "budget_pct": cfg.budget_pct, "recent": cfg.recent, "n_sink": cfg.n_sink_keep,
                   "decode_steps": T},
        "prefill_ms": round(prefill_ms, 4), "prompt_prune_ms": round(prune_ms, 4), "decode_loop_ms": round(decode_ms, 4),
        "prefill_pct_mfma_peak": round(100 * roof_prefill["frac"], 3) if mfma else None,
        "decode_prune_GBps": round(decode_gbps, 2),
        "decode_prune_pct_hbm_peak": round(100 * decode_gbps / HBM_PEAK_GBPS, 3),
        "roofline": roofline,
        "roofline_all": {"prefill_score": roof_prefill, "decode_step": roof_decode, "select_compact": roof_gather},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, layers[0], args.cpu_seconds)
    for c in caches:
        c.close()
    vatp.vatp_destroy(ctx)
    print(json.dumps(out), flush=True)


def cpu_baseline(cfg, inp, budget_s):
    """The float64 oracle, as it stands, timed on this machine's host cores on a bounded sample."""
    import numpy as np
    from oracle import vatp_oracle as orc
    threads = orc.max_threads()
    b = 0
    L = inp.lens[b]
    # sample: prompt scoring of `threads` heads of sequence 0, prompt truncated so the work stays bounded
    n_units = min(cfg.n_heads, threads)
    est_rate = 1.2e9                                   # key-query pairs * d per second per core, rough
    Ls = L
    while Ls > 256 and (Ls * Ls / 2) * cfg.head_dim / est_rate > budget_s:
        Ls //= 2
    Q = inp.Q[b, :n_units, :Ls].double().cpu().numpy()
    K = inp.K[b, :n_units, :Ls].double().cpu().numpy()
    t0 = time.perf_counter()
    orc.prefill_scores_units(Q, K, [Ls] * n_units)
    dt = time.perf_counter() - t0
    # tokens/s of prompt scoring for the sampled shape: all heads of a layer must be scored per token
    head_passes = n_units / cfg.n_heads
    return {"value": round(Ls * head_passes / dt, 2), "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "sample": "prompt scoring (both softmax passes of the oracle), %d of %d heads, first %d of %d prompt "
                      "tokens of sequence 0, one layer; %.2f s" % (n_units, cfg.n_heads, Ls, L, dt)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="llama7b_layer", choices=sorted(vs.CONFIGS))
    ap.add_argument("--layers", type=int, default=0, help="override the number of layers of the workload")
    ap.add_argument("--decode-steps", type=int, default=None)
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=15.0)
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also launch three plain 256 MiB -> 256 MiB element-wise copies (a known traffic "
                         "figure to scale rocprofv3's FETCH_SIZE / WRITE_SIZE against)")
    run(ap.parse_args())


if __name__ == "__main__":
    main()
