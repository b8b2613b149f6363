"""GPU parity for the options beyond the paper's default configuration."""
import sys

import numpy as np
import pytest
import torch

import parity
import vatp_synth as vs
from oracle import vatp_oracle as orc
import paper_2406_12335_amd as vatp

pytestmark = pytest.mark.gpu


def _say(msg):
    print("[case] " + msg, flush=True)
    sys.stdout.flush()


@pytest.mark.parametrize("norm_kind", [vatp.NORM_L2, vatp.NORM_LINF, vatp.NORM_NONE])
@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("fp32", 64)])
def test_norm_ablation_trajectories(gpu_device, norm_kind, dtype, d):
    """The l2 and l-infinity value norms of the paper's ablation (Table 2), and the attention-only
    baseline (norm switched off), through a whole trajectory."""
    cfg = vs.scaled(vs.CONFIGS["llama7b_layer"], n_heads=3, head_dim=d, prompt_len=333, dtype=dtype,
                    budget_pct=40, recent=32, decode_steps=12)
    _say("norm kind %d %s d=%d" % (norm_kind, dtype, d))
    rep = parity.run_trajectory(vs.make_inputs(cfg, seed=50 + norm_kind), gpu_device, norm_kind=norm_kind)
    _say("report %r" % rep)


@pytest.mark.parametrize("dtype,d,lens", [("bf16", 128, [700, 64, 257]), ("fp32", 64, [130, 1, 99]), ("bf16", 64, [300, 5, 77])])
def test_prompt_scores_from_given_row_lse(gpu_device, dtype, d, lens):
    """vatp_prefill_score_lse: only the column-sum pass runs; the oracle supplies ln-sum-exp per row."""
    cfg = vs.scaled(vs.CONFIGS["llama7b_layer"], batch=len(lens), n_heads=2, head_dim=d, dtype=dtype,
                    prompt_len=max(lens), decode_steps=0)
    inp = vs.make_inputs(cfg, seed=61)
    inp.lens = lens
    _say("lse-in %s d=%d lens=%s" % (dtype, d, lens))
    cap = max(lens)
    lse = torch.zeros(len(lens), 2, cap)
    want = {}
    for b, L in enumerate(lens):
        for h in range(2):
            Qh, Kh = inp.Q[b, h, :L].double().numpy(), inp.K[b, h, :L].double().numpy()
            l = orc.row_lse(Qh, Kh)
            lse[b, h, :L] = torch.from_numpy(l).float()
            # the GPU is handed the float32-rounded normalisers: so is the oracle
            want[(b, h)] = orc.prefill_scores_given_lse(Qh, Kh, lse[b, h, :L].double().numpy())
    dev = gpu_device
    ctx = vatp.vatp_create(0)
    try:
        p = vatp.Params(len(lens), 2, d, cfg.torch_dtype(), 0, 0, cap, lens, None)
        ws = torch.empty(max(256, vatp.vatp_workspace_bytes(ctx, p, vatp.CALL_PREFILL_SCORE)), dtype=torch.uint8, device=dev)
        S = torch.full((len(lens), 2, cap), -3.0, device=dev)
        nrm = torch.full((len(lens), 2, cap), -3.0, device=dev)
        vatp.vatp_prefill_score_lse(ctx, p, inp.Q.to(dev), inp.K.to(dev), inp.V.to(dev), lse.to(dev), S, nrm, ws)
        torch.cuda.synchronize()
    finally:
        vatp.vatp_destroy(ctx)
    rtol = parity.rtol_for(cfg.torch_dtype())
    for b, L in enumerate(lens):
        for h in range(2):
            parity.assert_scores_close(S[b, h, :L].cpu().numpy(), want[(b, h)], rtol, "S from lse (%d,%d)" % (b, h))
            parity.assert_scores_close(nrm[b, h, :L].cpu().numpy(), orc.l1norm(inp.V[b, h, :L].double().numpy()), rtol, "nrm")
        assert torch.all(S[b, :, L:] == -3.0)


@pytest.mark.parametrize("dtype,d,n0s", [("bf16", 128, [2048, 0, 130]), ("fp32", 64, [300, 127, 128]), ("bf16", 64, [1000, 5, 257]),
                                         ("fp32", 128, [129, 1, 64])])
def test_decode_step_with_attention_output(gpu_device, dtype, d, n0s):
    """vatp_decode_attend_step: same cache update as vatp_decode_step plus out = sum_r a_r V_r (Eq. 1)."""
    H = 2
    tdt = torch.float32 if dtype == "fp32" else torch.bfloat16
    cap = max(n0s) + 1
    g = torch.Generator().manual_seed(71)
    K = (torch.randn(len(n0s), H, cap, d, generator=g) * 1.2).to(tdt)
    V = (torch.randn(len(n0s), H, cap, d, generator=g) * torch.exp(0.5 * torch.randn(len(n0s), H, cap, 1, generator=g))).to(tdt)
    S0 = torch.rand(len(n0s), H, cap, generator=g) + 0.1
    q, k, v = ((torch.randn(len(n0s), H, d, generator=g) * 1.5).to(tdt) for _ in range(3))
    _say("attend %s d=%d n0=%s" % (dtype, d, n0s))
    dev = gpu_device
    ctx = vatp.vatp_create(0)
    try:
        p = vatp.Params(len(n0s), H, d, tdt, 0, 0, cap, n0s, None)
        res = []
        for attend in (False, True):
            Kd, Vd, Sd = K.to(dev).clone(), V.to(dev).clone(), S0.to(dev).clone()
            Nd = torch.zeros(len(n0s), H, cap, device=dev)
            out = torch.full((len(n0s), H, d), 9.0, device=dev)
            call = vatp.CALL_DECODE_ATTEND_STEP if attend else vatp.CALL_DECODE_STEP
            ws = torch.empty(vatp.vatp_workspace_bytes(ctx, p, call), dtype=torch.uint8, device=dev)
            if attend:
                vatp.vatp_decode_attend_step(ctx, p, q.to(dev), k.to(dev), v.to(dev), Kd, Vd, Sd, Nd, None, None, out, ws)
            else:
                vatp.vatp_decode_step(ctx, p, q.to(dev), k.to(dev), v.to(dev), Kd, Vd, Sd, Nd, None, None, ws)
            torch.cuda.synchronize()
            res.append((Kd.cpu(), Vd.cpu(), Sd.cpu(), Nd.cpu(), out.cpu()))
    finally:
        vatp.vatp_destroy(ctx)
    rtol = parity.rtol_for(tdt)
    (Ka, Va, Sa, Na, _), (Kb, Vb, Sb, Nb, out) = res
    for b, n0 in enumerate(n0s):
        n = n0 + 1
        # the cache update is bit-identical to the plain decode step
        assert torch.equal(Ka[b, :, :n], Kb[b, :, :n]) and torch.equal(Va[b, :, :n], Vb[b, :, :n])
        assert torch.equal(Sa[b, :, :n], Sb[b, :, :n]) and torch.equal(Na[b, :, n0], Nb[b, :, n0])
        for h in range(H):
            Kfull = torch.cat([K[b, h, :n0], k[b, h][None]], 0).double().numpy()
            Vfull = torch.cat([V[b, h, :n0], v[b, h][None]], 0).double().numpy()
            want, scale = orc.attention_output(q[b, h].double().numpy(), Kfull, Vfull)
            err = np.abs(out[b, h].double().numpy() - want)
            assert np.all(err <= rtol * scale + 1e-12), "attention output unit (%d,%d): max err %.3g" % (b, h, err.max())


@pytest.mark.parametrize("fused", [False, True])
def test_per_head_budgets_by_passing_heads_as_sequences(gpu_device, fused):
    """Non-uniform budgets across heads (the paper uses uniform ones and names the non-uniform strategy as the
    alternative, Implementation Details): len and budget are per sequence, and a [b, H, cap, d] tensor is the same
    memory as [b*H, 1, cap, d], so every head can be handed over as a sequence of its own with its own budget."""
    H, L = 6, 300
    cfg = vs.scaled(vs.CONFIGS["llama7b_layer"], batch=H, n_heads=1, prompt_len=L, budget_pct=50, recent=8, decode_steps=12)
    inp = vs.make_inputs(cfg, seed=123)
    inp.budgets = [40, 150, 75, 299, 310, 18]          # one per head; 310 > L: that head never prunes during the prompt
    _say("per-head budgets %s fused=%s" % (inp.budgets, fused))
    rep = parity.run_trajectory(inp, gpu_device, fused=fused)
    _say("report %r" % rep)
    assert rep.prune_events == H * 13


@pytest.mark.parametrize("fused,window", [(False, None), (True, None), (True, 20)])
def test_batch_of_256_sequences(gpu_device, fused, window):
    """The per-call limit: 256 sequences of their own lengths and budgets (also what lets a whole layer of
    8 x 32 heads be handed over with one budget per head)."""
    cfg = vs.scaled(vs.CONFIGS["ragged16"], batch=256, n_heads=1, ragged=(1, 300), recent=8, decode_steps=6)
    inp = vs.make_inputs(cfg, seed=31)
    inp.budgets = [max(b, cfg.n_sinks + cfg.recent) for b in inp.budgets]
    _say("256 sequences, fused=%s window=%s, lens %s..." % (fused, window, inp.lens[:6]))
    units = [(b, 0) for b in (0, 1, 63, 64, 65, 128, 200, 255)]
    rep = parity.run_trajectory(inp, gpu_device, units=units, fused=fused, window=window)
    _say("report %r" % rep)
