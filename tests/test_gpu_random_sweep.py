"""Seeded random configurations through the trajectory harness: dtype, head dimension, query heads per K/V head,
ragged batches, prompt lengths around the tile sizes, budgets down to F + R, both decode routes, history windows,
value norms, cache capacity beyond the budget."""
import random
import sys

import pytest

import parity
import vatp_synth as vs

pytestmark = pytest.mark.gpu


def _say(msg):
    print("[case] " + msg, flush=True)
    sys.stdout.flush()


def _draw(rng, big):
    dtype = "bf16" if big else rng.choice(["bf16", "bf16", "fp32"])
    d = 128 if big else rng.choice([64, 128, 128])
    g = rng.choice([1, 1, 1, 2, 3, 4, 8, 16])
    H = rng.choice([1, 2, 9, 33, 70] if big else [1, 2, 3, 5])
    b = rng.choice([1, 1, 2, 3])
    L = rng.choice([255, 257, 700, 1025, 1300, 2049, 2500, 3100] if big else
                   [1, 2, 17, 63, 64, 65, 127, 129, 255, 257, 300, 511, 513, 700, 1025, 1300])
    if dtype == "fp32" or d == 64:
        L = min(L, 520)
    R, F = rng.choice([0, 1, 4, 16, 33]), rng.choice([0, 1, 2, 5])
    pct, T = rng.choice([10, 30, 50, 90, 100]), rng.choice([0, 1, 5, 9])
    fused = rng.random() < 0.6
    window = rng.choice([None, None, 0, 3, 50, 400]) if fused else None
    ragged = (1, L) if rng.random() < 0.4 and L > 1 else None
    cfg = vs.scaled(vs.CONFIGS["llama7b_layer"], batch=b, n_heads=H, head_dim=d, prompt_len=L, dtype=dtype, n_sinks=min(F, L),
                    budget_pct=pct, recent=R, decode_steps=T, q_per_kv=g, ragged=ragged)
    return cfg, F, R, fused, window, rng.randrange(1 << 20), rng.choice([0, 0, 1, 2, 3]), rng.choice([None, None, 1, 7, 130])


@pytest.mark.parametrize("big,count,seed", [(False, 150, 11), (True, 16, 12)])
def test_random_configurations(gpu_device, big, count, seed):
    rng = random.Random(seed)
    for case in range(count):
        cfg, F, R, fused, window, sd, norm_kind, slack = _draw(rng, big)
        inp = vs.make_inputs(cfg, seed=sd)
        inp.budgets = [max(B, F + R) for B in inp.budgets]
        _say("%d: %s d=%d g=%d H=%d lens=%s R=%d F=%d B=%s T=%d fused=%s window=%s seed=%d" % (
            case, cfg.dtype, cfg.head_dim, cfg.q_per_kv, cfg.n_heads, inp.lens, R, F, inp.budgets, cfg.decode_steps, fused,
            window, sd) + " norm=%d slack=%s" % (norm_kind, slack))
        units = None
        if big:
            units = [(bb, hh) for bb in range(cfg.batch) for hh in sorted({0, cfg.n_heads - 1})][:3]
        cap_cache = None if slack is None else max(inp.budgets) + 1 + slack        # rows allocated beyond the budget
        parity.run_trajectory(inp, gpu_device, fused=fused, window=window, n_sink=F, units=units, norm_kind=norm_kind,
                              cap_cache=cap_cache)
