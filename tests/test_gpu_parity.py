"""GPU parity: the HIP path, called through the C ABI, against the float64 CPU oracle."""
import sys

import numpy as np
import pytest
import torch

import parity
import vatp_synth as vs
from oracle import vatp_oracle as orc
import paper_2406_12335_amd as vatp
from paper_2406_12335_amd.runner import PrunedKVCache

pytestmark = pytest.mark.gpu


def _say(msg):
    print("[case] " + msg, flush=True)
    sys.stdout.flush()


# ------------------------------------------------------------------ whole trajectories

def test_tiny_config_every_unit_every_step(gpu_device):
    cfg = vs.CONFIGS["tiny"]
    _say("tiny fp32 full trajectory")
    rep = parity.run_trajectory(vs.make_inputs(cfg, seed=0), gpu_device)
    assert rep.units_checked == 4 and rep.prune_events == 4 * 33
    _say("tiny report %r" % rep)


@pytest.mark.parametrize("dtype,d,L,T,pct,R,F,seed", [
    ("bf16", 128, 700, 24, 50, 64, 2, 1),      # several tiles and a ragged tail
    ("bf16", 64, 333, 16, 30, 16, 2, 2),
    ("fp32", 128, 257, 12, 50, 32, 20, 3),     # the paper's F = 20
    ("fp32", 64, 130, 12, 20, 8, 0, 4),        # no forced prefix
    ("bf16", 128, 300, 10, 50, 148, 2, 5),     # B = F + R: sinks + window only
])
def test_reduced_size_trajectories(gpu_device, dtype, d, L, T, pct, R, F, seed):
    cfg = vs.scaled(vs.CONFIGS["llama7b_layer"], n_heads=3, head_dim=d, prompt_len=L, dtype=dtype,
                    budget_pct=pct, recent=R, decode_steps=T)
    _say("reduced %s d=%d L=%d T=%d pct=%d R=%d F=%d" % (dtype, d, L, T, pct, R, F))
    rep = parity.run_trajectory(vs.make_inputs(cfg, seed=seed), gpu_device, n_sink=F)
    _say("report %r" % rep)


def test_ragged_batch_small(gpu_device):
    cfg = vs.scaled(vs.CONFIGS["ragged16"], batch=5, n_heads=2, ragged=(1, 300), decode_steps=6, recent=4,
                    n_sinks=1)
    inp = vs.make_inputs(cfg, seed=7)
    # budgets below F + R are not allowed: lift tiny ones
    inp.budgets = [max(b, cfg.n_sinks + cfg.recent) for b in inp.budgets]
    _say("ragged small lens=%s budgets=%s" % (inp.lens, inp.budgets))
    rep = parity.run_trajectory(inp, gpu_device)
    _say("report %r" % rep)


@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("bf16", 64), ("fp32", 64), ("fp32", 128)])
def test_prompt_scores_at_tile_edges(gpu_device, dtype, d):
    """Prompt lengths just below, at and above every tile size the kernels use."""
    lens = [1, 2, 31, 33, 63, 64, 65, 127, 129, 255, 256, 257, 511, 513, 770]
    cfg = vs.scaled(vs.CONFIGS["llama7b_layer"], batch=len(lens), n_heads=2, head_dim=d, dtype=dtype,
                    decode_steps=0, n_sinks=1)
    inp = vs.make_inputs(vs.scaled(cfg, prompt_len=max(lens)), seed=21)
    # shorten the sequences by hand: rows past a sequence's length hold junk on purpose
    inp.lens = lens
    for t in (inp.Q, inp.K, inp.V):
        for b, L in enumerate(lens):
            t[b, :, L:] = 77.0
    _say("tile edges %s d=%d" % (dtype, d))
    dev = gpu_device
    cache = PrunedKVCache(cfg.batch, 2, d, cfg.torch_dtype(), 0, 0, [max(lens)] * len(lens), dev)
    try:
        cache.prefill_score(inp.Q.to(dev), inp.K.to(dev), inp.V.to(dev), lens)
        torch.cuda.synchronize()
        S, nrm = cache.S_prompt.cpu(), cache.nrm_prompt.cpu()
    finally:
        cache.close()
    rtol = parity.rtol_for(cfg.torch_dtype())
    for b, L in enumerate(lens):
        for h in range(2):
            want = orc.prefill_scores(inp.Q[b, h, :L].double().numpy(), inp.K[b, h, :L].double().numpy())
            parity.assert_scores_close(S[b, h, :L].numpy(), want, rtol, "S len %d head %d" % (L, h))
            parity.assert_scores_close(nrm[b, h, :L].numpy(), orc.l1norm(inp.V[b, h, :L].double().numpy()), rtol, "nrm")


def test_llama7b_layer_full_size(gpu_device):
    cfg = vs.CONFIGS["llama7b_layer"]
    _say("llama7b_layer full size: prompt pass on all 32 heads, decode on 8 heads")
    inp = vs.make_inputs(cfg, seed=0)
    S = _prompt_scores_gpu(inp, gpu_device)
    lens = inp.lens
    Qh = inp.Q[0].double().numpy()
    Kh = inp.K[0].double().numpy()
    S_or = orc.prefill_scores_units(Qh, Kh, [lens[0]] * cfg.n_heads)
    for h in range(cfg.n_heads):
        parity.assert_scores_close(S[0, h].cpu().numpy(), S_or[h], 1e-3, "prompt S head %d" % h)
    units = [(0, h) for h in (0, 5, 11, 13, 17, 22, 29, 31)]
    rep = parity.run_trajectory(inp, gpu_device, units=units, prefill_oracle={(0, h): S_or[h] for _, h in units})
    _say("report %r" % rep)


@pytest.mark.parametrize("layer,units,steps", [
    (3, [(0, 0), (3, 17), (7, 31), (5, 8)], 256),
    (29, [(2, 9), (6, 24)], 96),                     # a second layer of the stack (its own seeded tensors)
])
def test_llama7b_stack_one_layer_full_size(gpu_device, layer, units, steps):
    cfg = vs.CONFIGS["llama7b_stack"]
    _say("llama7b_stack layer %d, batch 8 x 32 heads, units %s, %d steps" % (layer, units, steps))
    inp = vs.make_inputs(cfg, seed=0, layer=layer, device=gpu_device)
    rep = parity.run_trajectory(inp, gpu_device, units=units, steps=steps)
    _say("report %r" % rep)


def test_ragged16_full_size(gpu_device):
    cfg = vs.CONFIGS["ragged16"]
    inp = vs.make_inputs(cfg, seed=0, device=gpu_device)
    order = np.argsort(inp.lens)
    units = [(int(order[0]), 3), (int(order[-1]), 30), (int(order[8]), 12)]
    _say("ragged16 full size lens=%s units=%s" % (inp.lens, units))
    rep = parity.run_trajectory(inp, gpu_device, units=units)
    _say("report %r" % rep)


def test_long32k_full_size(gpu_device):
    """Prompt of 32768 rows.  Four heads get the oracle's whole prompt pass (Eq. 1-2 over all 32768 query rows,
    about half a minute of host time with one thread per head) and every one of their scores is compared; two of
    them then go through the prompt prune (judged on the oracle's scores) and the 64 decode steps.  All 32 heads:
    the invariants, and the last 384 keys against the oracle."""
    cfg = vs.CONFIGS["long32k"]
    _say("long32k full size: every score of 4 heads, invariants on all heads, tail of S on 3 more, decode on 2 heads")
    inp = vs.make_inputs(cfg, seed=0, device=gpu_device)
    S = _prompt_scores_gpu(inp, gpu_device)
    L = cfg.prompt_len
    tot = S.double().sum(-1).cpu().numpy()
    np.testing.assert_allclose(tot, L, rtol=1e-5)           # every softmax row sums to one
    assert torch.all(S[..., 0] >= 1.0 - 1e-6) and torch.all(S[..., L - 1] <= 1.0 + 1e-6) and torch.all(S > 0)
    j0 = L - 384
    for h in (0, 14, 31):
        want = orc.prefill_scores_tail(inp.Q[0, h].double().cpu().numpy(), inp.K[0, h].double().cpu().numpy(), j0)
        parity.assert_scores_close(S[0, h, j0:].cpu().numpy(), want, 1e-3, "tail S head %d" % h)
    full = [2, 27, 9, 20]
    _say("long32k: oracle prompt pass of heads %s" % full)
    Qh = np.stack([inp.Q[0, h].double().cpu().numpy() for h in full])
    Kh = np.stack([inp.K[0, h].double().cpu().numpy() for h in full])
    S_or = orc.prefill_scores_units(Qh, Kh, [L] * len(full))
    worst = 0.0
    for i, h in enumerate(full):
        worst = max(worst, parity.assert_scores_close(S[0, h].cpu().numpy(), S_or[i], 1e-3, "prompt S head %d" % h))
    _say("long32k: %d scores compared, worst relative error %.3g" % (len(full) * L, worst))
    rep = parity.run_trajectory(inp, gpu_device, units=[(0, 2), (0, 27)],
                                prefill_oracle={(0, 2): S_or[0], (0, 27): S_or[1]})
    _say("report %r" % rep)


def _prompt_scores_gpu(inp, device):
    cfg = inp.cfg
    cache = PrunedKVCache(cfg.batch, cfg.n_heads, cfg.head_dim, cfg.torch_dtype(), cfg.n_sink_keep, cfg.recent,
                          inp.budgets, device)
    try:
        cache.prefill_score(inp.Q.to(device), inp.K.to(device), inp.V.to(device), inp.lens)
        torch.cuda.synchronize()
        return cache.S_prompt.clone()
    finally:
        cache.close()


@pytest.mark.parametrize("jump", [40.0, 90.0, 150.0, 230.0])
def test_prompt_scores_with_a_late_dominant_key(gpu_device, jump):
    """One key far into the prompt whose logits tower over everything before it, by `jump` in the base-2
    domain: the running maximum of the row statistics has to follow it (150 and 230 exceed what fp32 could
    hold relative to the first keys' maximum), and the scores must still match the oracle."""
    d, L, H = 128, 700, 2
    g = torch.Generator().manual_seed(int(jump))
    u = torch.nn.functional.normalize(torch.randn(H, 1, d, generator=g), dim=-1)
    Q = (torch.randn(1, H, L, d, generator=g) + 10.0 * u).to(torch.bfloat16)
    K = torch.randn(1, H, L, d, generator=g)
    # <q, k*> ~ 10 |k*| for every query, so the logit is about jump when |k*| = jump * sqrt(d) / (10 log2 e)
    K[0, :, 100] = (jump * d ** 0.5 / (10.0 * 1.4427)) * u[:, 0]
    K = K.to(torch.bfloat16)
    V = torch.randn(1, H, L, d, generator=g).to(torch.bfloat16)
    _say("late dominant key, jump %.0f" % jump)
    cache = PrunedKVCache(1, H, d, torch.bfloat16, 2, 8, [L // 2], gpu_device)
    try:
        cache.prefill_score(Q.to(gpu_device), K.to(gpu_device), V.to(gpu_device), [L])
        torch.cuda.synchronize()
        S = cache.S_prompt.cpu().double().numpy()
    finally:
        cache.close()
    for h in range(H):
        want = orc.prefill_scores(Q[0, h].double().numpy(), K[0, h].double().numpy())
        assert np.all(np.isfinite(S[0, h]))
        # scores below 1e-30 belong to keys that every later query ignores next to the dominant one
        parity.assert_scores_close(S[0, h], want, 1e-3, "late dominant key, head %d" % h, atol=1e-30)
        assert abs(S[0, h].sum() - L) < 1e-3 * L


# ------------------------------------------------------------------ selection in isolation

@pytest.mark.parametrize("n,B,F,R,seed", [
    (4096, 2048, 2, 64, 0), (2049, 2048, 2, 64, 1), (1000, 999, 0, 0, 2), (1500, 300, 20, 100, 3),
    (70, 70, 2, 4, 4), (50, 80, 2, 4, 5), (300, 66, 2, 64, 6), (5000, 1, 0, 0, 7), (1025, 1024, 0, 1024, 8),
    (33000, 3276, 4, 128, 9),
    (20000, 6000, 2, 64, 10),          # 32 keys per thread in registers
    (70000, 7000, 4, 128, 11),         # beyond 64 keys per thread: the kernel that re-reads S and nrm per pass
    (1000000, 200, 2, 64, 12),         # a million rows, few survivors (the oracle picks them one at a time)
])
def test_select_compact_bit_exact_with_planted_ties(gpu_device, n, B, F, R, seed):
    """Same binary32 S and nrm on both sides, decision in binary32 on both sides: identical sets."""
    _say("select n=%d B=%d F=%d R=%d" % (n, B, F, R))
    H, d = 3, 64
    g = torch.Generator().manual_seed(seed)
    S = torch.rand(1, H, n, generator=g) * 3
    nrm = torch.rand(1, H, n, generator=g) * 50
    # exact ties: quantise some products, zero some norms
    S[0, 1] = torch.round(S[0, 1] * 4) / 4
    nrm[0, 1] = torch.round(nrm[0, 1])
    nrm[0, 2, torch.randint(0, n, (max(n // 10, 1),), generator=g)] = 0.0
    K = torch.randn(1, H, n, d, generator=g)
    V = torch.randn(1, H, n, d, generator=g)
    pos = torch.arange(n, dtype=torch.int32).expand(1, H, n).contiguous()
    cap_out = min(n, B) + 3
    ctx = vatp.vatp_create(0)
    try:
        dev = gpu_device
        out = dict(K=torch.zeros(1, H, cap_out, d), V=torch.zeros(1, H, cap_out, d), S=torch.zeros(1, H, cap_out),
                   nrm=torch.zeros(1, H, cap_out), pos=torch.zeros(1, H, cap_out, dtype=torch.int32),
                   kept=torch.full((1, H, cap_out), -1, dtype=torch.int32))
        out = {k: v.to(dev) for k, v in out.items()}
        p = vatp.Params(1, H, d, torch.float32, F, R, n, [n], [B], cap_out=cap_out)
        vatp.vatp_select_compact(ctx, p, K.to(dev), V.to(dev), S.to(dev), nrm.to(dev), pos.to(dev), out["K"],
                                 out["V"], out["S"], out["nrm"], out["pos"], out["kept"])
        torch.cuda.synchronize()
    finally:
        vatp.vatp_destroy(ctx)
    nk = min(n, B)
    for h in range(H):
        # Both sides are given the same binary32 S and nrm, and both decide in the kernel's precision: the
        # importance handed to the oracle's selection is the binary32 product (rounded here, in the test's
        # input preparation, not in the oracle).
        I = (S[0, h].numpy().astype(np.float32) * nrm[0, h].numpy().astype(np.float32)).astype(np.float64)
        want = orc.select(I, B, F, R)
        got = out["kept"][0, h, :nk].cpu().numpy()
        np.testing.assert_array_equal(got, want)
        assert torch.all(out["kept"][0, h, nk:] == -1)                      # nothing written past the survivors
        idx = torch.from_numpy(want.astype(np.int64))
        assert torch.equal(out["K"][0, h, :nk].cpu(), K[0, h, idx]) and torch.equal(out["V"][0, h, :nk].cpu(), V[0, h, idx])
        assert torch.equal(out["S"][0, h, :nk].cpu(), S[0, h, idx]) and torch.equal(out["nrm"][0, h, :nk].cpu(), nrm[0, h, idx])
        assert torch.equal(out["pos"][0, h, :nk].cpu(), pos[0, h, idx])


# ------------------------------------------------------------------ properties

def test_uniform_value_norms_reduce_to_attention_only_ranking(gpu_device):
    cfg = vs.scaled(vs.CONFIGS["llama7b_layer"], n_heads=2, prompt_len=600, decode_steps=0)
    inp = vs.make_inputs(cfg, seed=11)
    g = torch.Generator().manual_seed(5)
    inp.V = (torch.randint(0, 2, inp.V.shape, generator=g).float() * 2 - 1).to(torch.bfloat16)   # |v|_1 = d exactly
    _say("uniform norms")
    cache = PrunedKVCache(1, 2, 128, torch.bfloat16, 2, 64, inp.budgets, gpu_device)
    try:
        dev = gpu_device
        cache.prefill_score(inp.Q.to(dev), inp.K.to(dev), inp.V.to(dev), inp.lens)
        cache.prune_prompt(inp.K.to(dev), inp.V.to(dev))
        torch.cuda.synchronize()
        assert torch.all(cache.nrm_prompt == 128.0)
        for h in range(2):
            S32 = cache.S_prompt[0, h].cpu().double().numpy()
            want = orc.select(S32, inp.budgets[0], 2, 64)       # attention-only ranking of the same scores
            np.testing.assert_array_equal(cache.kept_idx[0, h, :inp.budgets[0]].cpu().numpy(), want)
    finally:
        cache.close()


def test_prompt_pass_is_deterministic_and_leaves_padding_alone(gpu_device):
    cfg = vs.scaled(vs.CONFIGS["ragged16"], batch=3, n_heads=2, ragged=(100, 400), decode_steps=0)
    inp = vs.make_inputs(cfg, seed=3)
    _say("determinism lens=%s" % inp.lens)
    runs = []
    for _ in range(2):
        cache = PrunedKVCache(3, 2, 128, torch.bfloat16, 2, 64, [max(b, 66) for b in inp.budgets], gpu_device)
        try:
            dev = gpu_device
            cache.S_prompt = torch.full((3, 2, inp.cap), -7.0, device=dev)
            cache.nrm_prompt = torch.full((3, 2, inp.cap), -7.0, device=dev)
            cache.prefill_score(inp.Q.to(dev), inp.K.to(dev), inp.V.to(dev), inp.lens)
            torch.cuda.synchronize()
            runs.append((cache.S_prompt.cpu(), cache.nrm_prompt.cpu()))
        finally:
            cache.close()
    assert torch.equal(runs[0][0], runs[1][0]) and torch.equal(runs[0][1], runs[1][1])
    for b, L in enumerate(inp.lens):
        assert torch.all(runs[0][0][b, :, L:] == -7.0) and torch.all(runs[0][1][b, :, L:] == -7.0)
        assert torch.all(runs[0][0][b, :, :L] > 0)


def test_entry_points_report_errors_on_device(gpu_device):
    ctx = vatp.vatp_create(0)
    try:
        t = torch.zeros(1, 1, 8, 64, device=gpu_device)
        s = torch.zeros(1, 1, 8, device=gpu_device)
        p = vatp.Params(1, 1, 64, torch.float32, 0, 0, 8, [8], [4])
        with pytest.raises(vatp.VatpError) as e:
            vatp.vatp_prefill_score(ctx, p, t, t, t, s, s, None)
        assert e.value.status == -5                                          # workspace missing
        with pytest.raises(vatp.VatpError) as e:
            vatp.vatp_select_compact(ctx, p, t, t, s, s, None, t, t, s, s, None, s.int())
        assert e.value.status == -2                                          # output aliases input
    finally:
        vatp.vatp_destroy(ctx)


# ------------------------------------------------------------------ edge cases

def test_empty_and_one_token_sequences_in_a_batch(gpu_device):
    """A sequence of length 0 (nothing to score, nothing to keep) next to lengths 1 and 70."""
    lens = [0, 1, 70, 0]
    cfg = vs.scaled(vs.CONFIGS["llama7b_layer"], batch=4, n_heads=2, prompt_len=70, decode_steps=5, recent=3,
                    n_sinks=1, budget_pct=50)
    inp = vs.make_inputs(cfg, seed=31)
    inp.lens = lens
    inp.budgets = [4, 4, 35, 6]
    _say("empty sequences lens=%s budgets=%s" % (lens, inp.budgets))
    rep = parity.run_trajectory(inp, gpu_device, cap_cache=40)
    assert rep.units_checked == 8
    _say("report %r" % rep)


def test_custom_scale_and_untracked_positions(gpu_device):
    cfg = vs.scaled(vs.CONFIGS["llama7b_layer"], n_heads=2, prompt_len=200, decode_steps=3)
    inp = vs.make_inputs(cfg, seed=32)
    dev = gpu_device
    d, L, Bq, F, R = 128, 200, 100, 2, 64
    scale = 0.05
    ctx = vatp.vatp_create(0)
    try:
        p = vatp.Params(1, 2, d, torch.bfloat16, F, R, L, [L], [Bq], cap_out=Bq + 1, scale=scale)
        ws = torch.empty(vatp.vatp_workspace_bytes(ctx, p, vatp.CALL_PREFILL_SCORE), dtype=torch.uint8, device=dev)
        Q, K, V = inp.Q.to(dev), inp.K.to(dev), inp.V.to(dev)
        S = torch.zeros(1, 2, L, device=dev)
        nrm = torch.zeros(1, 2, L, device=dev)
        vatp.vatp_prefill_score(ctx, p, Q, K, V, S, nrm, ws)
        Ko = torch.zeros(1, 2, Bq + 1, d, dtype=torch.bfloat16, device=dev)
        Vo = torch.zeros_like(Ko)
        So = torch.zeros(1, 2, Bq + 1, device=dev)
        No = torch.zeros_like(So)
        kept = torch.zeros(1, 2, Bq + 1, dtype=torch.int32, device=dev)
        vatp.vatp_select_compact(ctx, p, K, V, S, nrm, None, Ko, Vo, So, No, None, kept)     # pos not tracked
        pd = vatp.Params(1, 2, d, torch.bfloat16, F, R, Bq + 1, [Bq], [Bq], scale=scale)
        wsd = torch.empty(vatp.vatp_workspace_bytes(ctx, pd, vatp.CALL_DECODE_STEP), dtype=torch.uint8, device=dev)
        vatp.vatp_decode_step(ctx, pd, inp.qd[0].to(dev), inp.kd[0].to(dev), inp.vd[0].to(dev), Ko, Vo, So, No, None,
                              None, wsd)
        torch.cuda.synchronize()
    finally:
        vatp.vatp_destroy(ctx)
    for h in range(2):
        o = orc.OracleHead(d, c=scale)
        o.prefill(inp.Q[0, h].double().numpy(), inp.K[0, h].double().numpy(), inp.V[0, h].double().numpy())
        parity.assert_scores_close(S[0, h].cpu().numpy(), o.S, 1e-3, "S with custom scale")
        kept_or = o.prune(Bq, F, R)
        np.testing.assert_array_equal(kept[0, h, :Bq].cpu().numpy(), kept_or)
        o.append_and_score(inp.qd[0, 0, h].double().numpy(), inp.kd[0, 0, h].double().numpy(),
                           inp.vd[0, 0, h].double().numpy(), L)
        parity.assert_scores_close(So[0, h, :Bq + 1].cpu().numpy(), o.S, 1e-3, "decode S with custom scale")
        parity.assert_scores_close(No[0, h, :Bq + 1].cpu().numpy(), o.nrm, 1e-3, "decode nrm")


def test_decode_on_a_long_cache_and_determinism(gpu_device):
    """One head with 70001 cached rows (hundreds of chunks), run twice: identical bits, oracle parity."""
    n0, d = 70001, 64
    g = torch.Generator().manual_seed(41)
    K = torch.randn(1, 1, n0 + 1, d, generator=g)
    V = torch.randn(1, 1, n0 + 1, d, generator=g)
    S0 = torch.rand(1, 1, n0 + 1, generator=g) * 2
    nrm0 = V.abs().sum(-1)
    q, k, v = (torch.randn(1, 1, d, generator=g) * 1.5 for _ in range(3))
    _say("long-cache decode n0=%d" % n0)
    dev = gpu_device
    outs = []
    ctx = vatp.vatp_create(0)
    try:
        p = vatp.Params(1, 1, d, torch.float32, 0, 0, n0 + 1, [n0], None)
        ws = torch.empty(vatp.vatp_workspace_bytes(ctx, p, vatp.CALL_DECODE_STEP), dtype=torch.uint8, device=dev)
        for _ in range(2):
            Kd, Vd, Sd, Nd = K.to(dev).clone(), V.to(dev).clone(), S0.to(dev).clone(), nrm0.to(dev).clone()
            Kd[0, 0, n0] = 7.0          # stale junk in the slot of the new row
            Sd[0, 0, n0] = 123.0
            pos = torch.arange(n0 + 1, dtype=torch.int32, device=dev).view(1, 1, -1).clone()
            vatp.vatp_decode_step(ctx, p, q.to(dev), k.to(dev), v.to(dev), Kd, Vd, Sd, Nd, pos, [555], ws)
            torch.cuda.synchronize()
            outs.append((Kd.cpu(), Vd.cpu(), Sd.cpu(), Nd.cpu(), pos.cpu()))
    finally:
        vatp.vatp_destroy(ctx)
    for a, b in zip(outs[0], outs[1]):
        assert torch.equal(a, b)
    Kd, Vd, Sd, Nd, pos = outs[0]
    assert torch.equal(Kd[0, 0, n0], k[0, 0]) and torch.equal(Vd[0, 0, n0], v[0, 0]) and pos[0, 0, n0] == 555
    Kfull = torch.cat([K[0, 0, :n0], k[0]], 0).double().numpy()
    S_in = np.concatenate([S0[0, 0, :n0].double().numpy(), np.zeros(1)])
    S_or, _ = orc.decode_scores(q[0, 0].double().numpy(), Kfull, S_in)
    parity.assert_scores_close(Sd[0, 0].numpy(), S_or, 1e-5, "long-cache decode S")
    assert abs(float(Nd[0, 0, n0]) - float(v.abs().sum())) < 1e-4


def test_misaligned_pointers_are_rejected(gpu_device):
    ctx = vatp.vatp_create(0)
    try:
        base = torch.zeros(1 * 1 * 8 * 64 + 8, dtype=torch.bfloat16, device=gpu_device)
        t_bad = base[1:1 + 512].view(1, 1, 8, 64)           # 2 bytes off a 16-byte boundary
        t_ok = base[:512].view(1, 1, 8, 64)
        s = torch.zeros(1, 1, 8, device=gpu_device)
        p = vatp.Params(1, 1, 64, torch.bfloat16, 0, 0, 8, [8], [4])
        ws = torch.empty(4096, dtype=torch.uint8, device=gpu_device)
        with pytest.raises(vatp.VatpError) as e:
            vatp.vatp_prefill_score(ctx, p, t_bad, t_ok, t_ok, s, s.clone(), ws)
        assert e.value.status == -2
    finally:
        vatp.vatp_destroy(ctx)
