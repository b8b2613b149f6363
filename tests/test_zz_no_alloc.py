"""vatp_decode_prune_step_static, the entry point that allocates nothing (its scratch is a static device array),
against vatp_decode_prune_step with a caller-owned workspace: identical bits, on two calls in a row, the
second on a smaller input (so the array still holds the first call's contents when the second one runs)."""
import sys

import pytest
import torch

import paper_2406_12335_amd as vatp
from paper_2406_12335_amd import binding as B

pytestmark = pytest.mark.gpu


def _say(msg):
    print("[case] " + msg, flush=True)
    sys.stdout.flush()


def _state(dev, b, H, d, n0, cap, seed, dtype):
    """A cache of n0 rows per head (cap allocated) plus one new token; everything seeded."""
    g = torch.Generator().manual_seed(seed)
    t = lambda *s: torch.randn(*s, generator=g)
    st = dict(K=t(b, H, cap, d).to(dtype), V=t(b, H, cap, d).to(dtype), S=torch.rand(b, H, cap, generator=g) * 3,
              nrm=torch.rand(b, H, cap, generator=g) * 40, pos=torch.arange(cap, dtype=torch.int32).expand(b, H, cap).contiguous(),
              q=(t(b, H, d) * 1.5).to(dtype), k=t(b, H, d).to(dtype), v=t(b, H, d).to(dtype))
    return {k: x.to(dev) for k, x in st.items()}


def _step(dev, ctx, st, b, H, d, n0, cap, budget, F, R, dtype, static, want_out):
    """One fused step from a copy of `st`; returns everything the call writes."""
    K, V, nrm, pos = (st[k].clone() for k in ("K", "V", "nrm", "pos"))
    K2, V2 = torch.zeros_like(K), torch.zeros_like(V)
    S2, nrm2 = torch.full_like(st["S"], -1.0), torch.full_like(nrm, -1.0)
    pos2 = torch.full_like(pos, -1)
    kept = torch.full((b, H, cap), -1, dtype=torch.int32, device=dev)
    syn_in = torch.zeros(b * H, dtype=torch.int32, device=dev)
    syn_out = torch.full((b * H,), -1, dtype=torch.int32, device=dev)
    out = torch.zeros(b, H, d, device=dev) if want_out else None
    p = vatp.Params(b, H, d, dtype, F, R, cap, [n0] * b, [budget] * b)
    new_pos = [1000 + i for i in range(b)]
    if static:
        vatp.vatp_decode_prune_step_static(ctx, p, st["q"], st["k"], st["v"], K, V, st["S"], nrm, pos, new_pos, K2, V2, S2,
                                           nrm2, pos2, kept, syn_in, syn_out, out)
    else:
        ws = torch.empty(vatp.vatp_workspace_bytes(ctx, p, vatp.CALL_DECODE_PRUNE_STEP), dtype=torch.uint8, device=dev)
        vatp.vatp_decode_prune_step(ctx, p, st["q"], st["k"], st["v"], K, V, st["S"], nrm, pos, new_pos, K2, V2, S2, nrm2,
                                    pos2, kept, syn_in, syn_out, out, ws)
    torch.cuda.synchronize()
    res = dict(K=K, V=V, nrm=nrm, pos=pos, K2=K2, V2=V2, S2=S2, nrm2=nrm2, pos2=pos2, kept=kept, syn_out=syn_out)
    if want_out:
        res["out"] = out
    return res


def test_static_scratch_step_matches_the_workspace_step_twice_in_a_row(gpu_device):
    dev = gpu_device
    ctx = vatp.vatp_create(0)
    try:
        # (heads, rows before the step): two launches with the logits in the scratch array both times -- 32 heads of
        # 2048 rows, then 4 heads of 300 rows; the second call also asks for the attention output (partial outputs
        # in the scratch array as well)
        for i, (H, n0, want_out) in enumerate([(32, 2048, False), (4, 300, True)]):
            b, d, F, R, dtype = 1, 128, 2, 64, torch.bfloat16
            cap = n0 + 1
            st = _state(dev, b, H, d, n0, cap, seed=50 + i, dtype=dtype)
            _say("static scratch call %d: %d heads x %d rows, attention output %s" % (i, H, n0, want_out))
            got = _step(dev, ctx, st, b, H, d, n0, cap, n0, F, R, dtype, True, want_out)
            want = _step(dev, ctx, st, b, H, d, n0, cap, n0, F, R, dtype, False, want_out)
            for name in want:
                assert torch.equal(got[name], want[name]), "call %d: %s differs" % (i, name)
            assert int(got["syn_out"].min()) >= F and int(got["syn_out"].max()) <= n0 - R      # one row left every head
        # a shape whose scratch would not fit the static array is refused before anything is launched
        H, n0 = 4096, 2048
        p = vatp.Params(1, H, 128, torch.bfloat16, 2, 64, n0 + 1, [n0], [n0])
        assert vatp.vatp_workspace_bytes(ctx, p, vatp.CALL_DECODE_PRUNE_STEP) > B.VATP_STATIC_SCRATCH_BYTES
        z = torch.zeros(1, device=dev)
        with pytest.raises(vatp.VatpError) as e:
            vatp.vatp_decode_prune_step_static(ctx, p, z, z, z, z, z, z, z, None, None, z, z, z, z, None, None, z, z, None)
        assert e.value.status == B.E_WORKSPACE
    finally:
        vatp.vatp_destroy(ctx)
