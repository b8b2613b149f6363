"""GPU parity of vatp_decode_prune_step (decode step + eviction in two launches, rewriting only
the rows that changed): against the oracle through whole trajectories, and bit for bit
against the route through vatp_decode_attend_step + vatp_select_compact."""
import sys

import numpy as np
import pytest
import torch

import parity
import vatp_synth as vs
import paper_2406_12335_amd as vatp
from paper_2406_12335_amd.runner import PrunedKVCache

pytestmark = pytest.mark.gpu


def _say(msg):
    print("[case] " + msg, flush=True)
    sys.stdout.flush()


@pytest.mark.parametrize("name,kw", [
    ("tiny", {}),
    ("llama7b_layer", dict(n_heads=4, prompt_len=777, decode_steps=24)),
    ("ragged16", dict(batch=6, n_heads=2, decode_steps=10, recent=8, ragged=(1, 600))),
    # 128 heads or more with short caches take the single-launch route
    ("tiny", dict(batch=4, n_heads=32, prompt_len=96, decode_steps=12, recent=8)),
    ("llama7b_layer", dict(batch=2, n_heads=64, prompt_len=150, decode_steps=8, recent=16)),
])
def test_fused_trajectory_against_oracle(gpu_device, name, kw):
    cfg = vs.scaled(vs.CONFIGS[name], **kw) if kw else vs.CONFIGS[name]
    _say("fused trajectory %s %r" % (name, kw))
    inp = vs.make_inputs(cfg, seed=31)
    # budgets below F + R are not allowed: lift tiny ones
    inp.budgets = [max(b, cfg.n_sinks + cfg.recent) for b in inp.budgets]
    _say("lens=%s budgets=%s" % (inp.lens[:8], inp.budgets[:8]))
    rep = parity.run_trajectory(inp, gpu_device, fused=True)
    _say("report %r" % rep)
    assert rep.prune_events > 0


def _twin_caches(dev, b, H, d, tdt, F, R, budgets, cap):
    return [PrunedKVCache(b, H, d, tdt, F, R, budgets, dev, cap_cache=cap) for _ in range(2)]


def _seed_state(caches, lens, g, d, tdt, dev, weak_rows=None):
    """Puts the same synthetic cache state (as if left by a prompt prune) into set 0 of each cache."""
    a = caches[0]
    b, H, cap = a.batch, a.n_heads, a.cap
    K = (torch.randn(b, H, cap, d, generator=g) * 1.2).to(tdt)
    V = (torch.randn(b, H, cap, d, generator=g) * torch.exp(0.5 * torch.randn(b, H, cap, 1, generator=g))).to(tdt)
    S = torch.rand(b, H, cap, generator=g) + 0.5
    if weak_rows:
        for (bb, hh, r) in weak_rows:       # a row that will lose: almost no value norm
            V[bb, hh, r] = (V[bb, hh, r].float() * 1e-4).to(tdt)
    nrm = V.float().abs().sum(-1)
    pos = torch.arange(cap, dtype=torch.int32).expand(b, H, cap).contiguous()
    for c in caches:
        c.K[0].copy_(K.to(dev)); c.V[0].copy_(V.to(dev)); c.S[0].copy_(S.to(dev)); c.nrm[0].copy_(nrm.to(dev))
        c.pos[0].copy_(pos.to(dev))
        for t in (c.K[1], c.V[1]):
            t.fill_(7.0)                    # the other set starts as garbage
        c.S[1].fill_(-3.0); c.nrm[1].fill_(-3.0); c.pos[1].fill_(-3)
        c.cur = 0
        c.lens = list(lens)
        c._synced_valid = False


@pytest.mark.parametrize("dtype,d,H,lens,budgets,R,F,steps", [
    ("bf16", 128, 3, [300, 290, 64], [300, 300, 70], 16, 2, 14),   # at budget, growing, growing then at budget
    ("fp32", 64, 3, [129, 40, 128], [129, 129, 129], 8, 0, 10),
    ("bf16", 64, 3, [513, 512, 100], [513, 513, 513], 32, 4, 9),
    ("fp32", 128, 3, [70, 70, 3], [70, 70, 70], 5, 1, 8),
    # 128 heads and more: the steps without attention output take the single-launch route
    ("bf16", 128, 43, [300, 290, 64], [300, 300, 70], 16, 2, 8),
    ("fp32", 64, 64, [1000, 129], [1000, 140], 8, 0, 7),
    ("bf16", 64, 32, [5, 130, 129, 257], [9, 130, 200, 257], 3, 1, 9),
    # the single-launch route at the edges of what it stores ahead of the eviction decision
    ("bf16", 128, 64, [400, 390], [400, 400], 0, 0, 9),        # no window, no prefix: the appended row is a candidate
    ("bf16", 128, 64, [400, 390], [400, 400], 127, 2, 9),      # window + 1 rows = all the rows stored ahead
    ("bf16", 128, 64, [400, 250], [400, 400], 128, 2, 9),      # window one row longer than that
    ("bf16", 64, 64, [700, 690], [700, 700], 200, 1, 9),       # much longer: part of the window is copied afterwards
    ("fp32", 128, 64, [300, 100], [300, 300], 40, 0, 9),       # 32 lanes per row
    ("bf16", 128, 65, [1023, 1000], [1023, 1023], 64, 2, 6),   # 1024 rows after the append: the route's limit
])
def test_fused_step_is_bit_identical_to_the_two_call_route(gpu_device, dtype, d, H, lens, budgets, R, F, steps):
    """Same K, V, S, nrm, pos, kept_idx and attention output as vatp_decode_attend_step followed by
    vatp_select_compact, step after step; includes heads whose evicted row lies far from the window."""
    dev = gpu_device
    tdt = torch.float32 if dtype == "fp32" else torch.bfloat16
    b = len(lens)
    cap = max(budgets) + 1
    g = torch.Generator().manual_seed(5)
    _say("fused vs two calls %s d=%d lens=%s budgets=%s" % (dtype, d, lens, budgets))
    classic, fused = _twin_caches(dev, b, H, d, tdt, F, R, budgets, cap)
    try:
        weak = [(0, 1, F + 3), (0, 2, lens[0] // 2), (1, 0, F + 1), (1, H - 1, F)]
        _seed_state([classic, fused], lens, g, d, tdt, dev, weak_rows=weak)
        ws_att = torch.empty(vatp.vatp_workspace_bytes(classic.ctx, classic._p_dec, vatp.CALL_DECODE_ATTEND_STEP) + 256,
                             dtype=torch.uint8, device=dev)
        for t in range(steps):
            q, k, v = ((torch.randn(b, H, d, generator=g) * 1.5).to(tdt).to(dev) for _ in range(3))
            new_pos = [1000 + t] * b
            out_c = torch.zeros(b, H, d, device=dev)
            out_f = torch.ones(b, H, d, device=dev)
            # two-call route (with attention output)
            c = classic.cur
            classic._p_dec.set_len(classic.lens)
            vatp.vatp_decode_attend_step(classic.ctx, classic._p_dec, q, k, v, classic.K[c], classic.V[c], classic.S[c],
                                         classic.nrm[c], classic.pos[c], new_pos, out_c, ws_att)
            classic.lens = [n + 1 for n in classic.lens]
            classic.prune()
            # fused route; every third step without kept_idx and without the attention output
            plain = t % 3 == 2
            fused.decode_prune_step(q, k, v, new_pos, out=None if plain else out_f, want_kept_idx=not plain)
            torch.cuda.synchronize()
            assert classic.lens == fused.lens
            cc, fc = classic.cur, fused.cur
            for bb, n in enumerate(fused.lens):
                for name in ("K", "V", "S", "nrm", "pos"):
                    x, y = getattr(classic, name)[cc][bb, :, :n], getattr(fused, name)[fc][bb, :, :n]
                    assert torch.equal(x, y), "step %d sequence %d: %s differs" % (t, bb, name)
                if not plain:
                    assert torch.equal(classic.kept_idx[bb, :, :n], fused.kept_idx[bb, :, :n]), "kept_idx differs"
            if not plain:
                assert torch.equal(out_c, out_f), "attention output differs at step %d" % t
    finally:
        torch.cuda.synchronize()
        classic.close(); fused.close()


def test_fused_step_rejects_more_than_one_eviction_and_aliases(gpu_device):
    dev = gpu_device
    b, H, d, cap = 1, 2, 128, 40
    c = PrunedKVCache(b, H, d, torch.bfloat16, 1, 4, [30], dev, cap_cache=cap)
    try:
        x = torch.zeros(b, H, d, dtype=torch.bfloat16, device=dev)
        c.lens = [31]                       # 32 rows after the append: two would have to leave
        with pytest.raises(vatp.VatpError) as e:
            c.decode_prune_step(x, x, x, [0])
        assert e.value.status == vatp.binding.E_BUDGET
        c.lens = [30]
        c.synced[1] = c.synced[0]           # the two count arrays must be distinct
        with pytest.raises(vatp.VatpError) as e:
            c.decode_prune_step(x, x, x, [0])
        assert e.value.status == vatp.binding.E_SHAPE
    finally:
        c.close()


@pytest.mark.parametrize("name,kw,w", [
    ("tiny", dict(decode_steps=40), 7),                                      # the whole prompt leaves the window
    ("tiny", dict(decode_steps=12), 0),
    ("tiny", dict(decode_steps=10, prompt_len=40), 100),                      # window longer than prompt + decode
    ("llama7b_layer", dict(n_heads=3, prompt_len=500, decode_steps=30, recent=10), 16),
    ("llama7b_layer", dict(n_heads=2, head_dim=64, prompt_len=333, decode_steps=20, recent=10), 400),
    ("ragged16", dict(batch=5, n_heads=2, decode_steps=14, recent=8, ragged=(1, 400)), 9),
])
def test_history_window_trajectory_against_oracle(gpu_device, name, kw, w):
    """Scores over a history window (Eq. 3): windowed prompt pass, prompt prune with its history, fused steps."""
    cfg = vs.scaled(vs.CONFIGS[name], **kw)
    _say("history window %d, %s %r" % (w, name, kw))
    inp = vs.make_inputs(cfg, seed=44)
    inp.budgets = [max(b, cfg.n_sinks + cfg.recent) for b in inp.budgets]
    _say("lens=%s budgets=%s" % (inp.lens[:8], inp.budgets[:8]))
    rep = parity.run_trajectory(inp, gpu_device, fused=True, window=w)
    _say("report %r" % rep)
    assert rep.prune_events > 0
    assert rep.admitted_near_ties <= max(1, rep.prune_events // 50)      # differences inside the band stay rare


@pytest.mark.parametrize("dtype,w", [("fp32", 3), ("bf16", 5)])
def test_windowed_score_stays_relative_after_large_weights_leave(gpu_device, dtype, w):
    """One key draws almost all of the attention for a few steps and almost none afterwards: its windowed
    score falls by five orders of magnitude once the large weights have left the window.  A plain fp32
    running sum keeps a residue of about 2^-24 of the LARGE score (a relative error of a per cent here);
    the score carried in two floats must still match the oracle to the ordinary relative tolerance."""
    d, L, T, row = 64, 40, 14, 10
    cfg = vs.scaled(vs.CONFIGS["tiny"], n_heads=2, head_dim=d, prompt_len=L, dtype=dtype, decode_steps=T, recent=4,
                    n_sinks=0)
    inp = vs.make_inputs(cfg, seed=77)
    inp.budgets = [L + T + 1]                      # nothing is evicted: the row lives through the whole run
    k = inp.K[0, :, row].float()
    unit = k / k.norm(dim=-1, keepdim=True)
    for t in range(T):
        # scaled logit of the chosen key: +9 for four steps (weight close to 1), -12 afterwards
        want = 9.0 if t < 4 else -12.0
        q = unit * (want * d ** 0.5 / k.norm(dim=-1, keepdim=True)) + 0.05 * inp.qd[t, 0].float()
        inp.qd[t, 0] = q.to(inp.qd.dtype)
    _say("windowed score after large weights leave, %s, w=%d" % (dtype, w))
    rep = parity.run_trajectory(inp, gpu_device, fused=True, window=w, n_sink=0, cap_cache=L + T + 2)
    _say("report %r" % rep)
    assert rep.admitted_near_ties == 0


@pytest.mark.parametrize("dtype,d,lens,w", [
    ("bf16", 128, [2500, 130], 400),        # two key ranges, window inside the second block
    ("bf16", 128, [4096, 4095], 400),
    ("bf16", 128, [2049, 2048], 255),
    ("bf16", 128, [300, 64], 1000),         # window longer than the prompt
    ("bf16", 128, [2112, 1], 63),
    ("bf16", 128, [4100, 257], 0),
    ("bf16", 128, [700, 699], 256),
    ("fp32", 64, [700, 65], 100),
    ("bf16", 64, [1000, 3], 300),
    ("fp32", 128, [130, 129], 64),
])
def test_windowed_prompt_scores_and_attention_rows(gpu_device, dtype, d, lens, w):
    """vatp_prefill_score_window: S over the last w+1 query rows (Eq. 3) and those rows themselves."""
    H = 2
    cfg = vs.scaled(vs.CONFIGS["llama7b_layer"], batch=len(lens), n_heads=H, head_dim=d, dtype=dtype,
                    prompt_len=max(lens), decode_steps=0)
    cfg = vs.scaled(cfg, ragged=None)
    _say("windowed prompt pass %s d=%d lens=%s w=%d" % (dtype, d, lens, w))
    inp = vs.make_inputs(cfg, seed=61)
    dev = gpu_device
    tdt = cfg.torch_dtype()
    cap = max(lens)
    ctx = vatp.vatp_create(0)
    try:
        p = vatp.Params(len(lens), H, d, tdt, 0, 0, cap, lens, None)
        ws = torch.empty(vatp.vatp_workspace_bytes(ctx, p, vatp.CALL_PREFILL_SCORE_WINDOW), dtype=torch.uint8, device=dev)
        S = torch.full((len(lens), H, cap), -1.0, device=dev)
        nrm = torch.empty(len(lens), H, cap, device=dev)
        hist = torch.full((len(lens), H, w + 1, cap), -2.0, device=dev)
        vatp.vatp_prefill_score_window(ctx, p, inp.Q.to(dev), inp.K.to(dev), inp.V.to(dev), w, S, nrm, hist, ws)
        torch.cuda.synchronize()
        S, hist = S.cpu().double().numpy(), hist.cpu().double().numpy()
    finally:
        vatp.vatp_destroy(ctx)
    rtol = parity.rtol_for(tdt)
    for b, L in enumerate(lens):
        for h in range(H):
            S_or, P_or = parity.orc.prefill_window(inp.Q[b, h, :L].double().numpy(), inp.K[b, h, :L].double().numpy(), w)
            parity.assert_scores_close(S[b, h, :L], S_or, rtol, "windowed S (%d,%d)" % (b, h))
            assert np.all(S[b, h, L:] == -1.0), "scores past the end of the sequence were touched"
            j0 = max(0, L - 1 - w)
            for r in range(P_or.shape[0]):
                j = j0 + r
                parity.assert_scores_close(hist[b, h, r, :j + 1], P_or[r, :j + 1], rtol,
                                           "attention row of query %d unit (%d,%d)" % (j, b, h), atol=1e-35)


# ---------------------------------------------------------------- full sizes, in the launch shapes bench.py times

@pytest.mark.parametrize("name,units,steps,window", [
    ("llama7b_layer", [(0, 0), (0, 13), (0, 31)], 48, None),          # two launches, 16 workgroups per head
    ("llama7b_stack", [(0, 0), (3, 17), (7, 31)], 48, None),          # 256 heads x 820 rows: one launch
    ("ragged16", None, 24, None),                                     # 512 heads of unequal length
    ("llama7b_layer", [(0, 2), (0, 30)], 24, 400),                    # history window, both key ranges of the prompt pass
    ("llama7b_stack", [(1, 5), (6, 20)], 16, 400),
])
def test_fused_route_full_size(gpu_device, name, units, steps, window):
    cfg = vs.CONFIGS[name]
    inp = vs.make_inputs(cfg, seed=0, layer=3 if name == "llama7b_stack" else 0, device=gpu_device)
    if units is None:
        order = np.argsort(inp.lens)
        units = [(int(order[0]), 3), (int(order[-1]), 30), (int(order[8]), 12)]
    _say("fused route full size %s units=%s steps=%d window=%s" % (name, units, steps, window))
    # (the oracle runs the prompt pass of the chosen units itself: the whole triangle, or the window's band)
    rep = parity.run_trajectory(inp, gpu_device, units=units, steps=steps, fused=True, window=window,
                                check_every=4)
    _say("report %r" % rep)
    assert rep.prune_events == len(units) * (steps + 1)
    assert rep.admitted_near_ties <= max(1, rep.prune_events // 50)


def test_long32k_full_size_history_window(gpu_device):
    """Prompt of 32768 with w = 400: 16 key ranges in the row-statistics pass; all heads' scores total w+1."""
    cfg = vs.CONFIGS["long32k"]
    inp = vs.make_inputs(cfg, seed=0, device=gpu_device)
    w = 400
    _say("long32k, history window %d" % w)
    rep = parity.run_trajectory(inp, gpu_device, units=[(0, 1), (0, 26)], steps=12, fused=True, window=w,
                                check_every=3)
    _say("report %r" % rep)
    assert rep.admitted_near_ties <= 1


def test_window_calls_reject_bad_arguments_and_accept_no_history_buffer(gpu_device):
    dev = gpu_device
    b, H, d, L, w = 1, 2, 128, 300, 50
    cfg = vs.scaled(vs.CONFIGS["llama7b_layer"], n_heads=H, prompt_len=L, decode_steps=2, recent=8)
    inp = vs.make_inputs(cfg, seed=9)
    Q, K, V = inp.Q.to(dev), inp.K.to(dev), inp.V.to(dev)
    ctx = vatp.vatp_create(0)
    try:
        p = vatp.Params(b, H, d, torch.bfloat16, 2, 8, L, [L], [150])
        ws = torch.empty(vatp.vatp_workspace_bytes(ctx, p, vatp.CALL_PREFILL_SCORE_WINDOW), dtype=torch.uint8, device=dev)
        S0, S1 = torch.empty(b, H, L, device=dev), torch.empty(b, H, L, device=dev)
        nrm = torch.empty(b, H, L, device=dev)
        hist = torch.empty(b, H, w + 1, L, device=dev)
        vatp.vatp_prefill_score_window(ctx, p, Q, K, V, w, S0, nrm, hist, ws)
        vatp.vatp_prefill_score_window(ctx, p, Q, K, V, w, S1, nrm, None, ws)      # scores only
        torch.cuda.synchronize()
        assert torch.equal(S0, S1)
        with pytest.raises(vatp.VatpError) as e:                                   # workspace of the plain call is too small
            small = torch.empty(vatp.vatp_workspace_bytes(ctx, p, vatp.CALL_PREFILL_SCORE), dtype=torch.uint8, device=dev)
            vatp.vatp_prefill_score_window(ctx, p, Q, K, V, w, S0, nrm, hist, small)
        assert e.value.status == vatp.binding.E_WORKSPACE
        with pytest.raises(vatp.VatpError) as e:
            vatp.vatp_prefill_score_window(ctx, p, Q, K, V, -3, S0, nrm, hist, ws)
        assert e.value.status == vatp.binding.E_SHAPE
    finally:
        vatp.vatp_destroy(ctx)
    c = PrunedKVCache(b, H, d, torch.bfloat16, 2, 8, [150], dev, window=w)
    try:
        c.prefill_score(Q, K, V, [L])
        c.prune_prompt(K, V)
        x = torch.zeros(b, H, d, dtype=torch.bfloat16, device=dev)
        good_hist, good_free = c.hist, c.free
        c.cap_hist = 100                                                            # fewer columns than budget + 1
        with pytest.raises(vatp.VatpError) as e:
            c.decode_prune_step(x, x, x, [L])
        assert e.value.status == vatp.binding.E_BUDGET
        c.cap_hist = c.cap
        c.free = [good_free[0], good_free[0]]                                       # the two count arrays must differ
        with pytest.raises(vatp.VatpError) as e:
            c.decode_prune_step(x, x, x, [L])
        assert e.value.status == vatp.binding.E_SHAPE
        c.free = good_free
        with pytest.raises(vatp.VatpError) as e:                                    # the step index is required
            vatp.vatp_decode_prune_step_window(c.ctx, c._p_dec, x, x, x, c.K[0], c.V[0], c.S[0], c.nrm[0], c.pos[0], c.hid[0],
                                               None, c.K[1], c.V[1], c.S[1], c.nrm[1], c.pos[1], c.hid[1], None,
                                               c.synced[0], c.synced[1], c.free[0], c.free[1], good_hist, c.S_lo[0], c.S_lo[1],
                                               w, c.cap_hist, None, c.ws)
        assert e.value.status == vatp.binding.E_NULL
        c.decode_prune_step(x, x, x, [L])                                           # and the good call still works
        torch.cuda.synchronize()
        assert c.lens == [150]
    finally:
        c.close()
