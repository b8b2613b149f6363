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


@pytest.mark.parametrize("norm_kind", [vatp.NORM_L2, vatp.NORM_LINF])
@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("fp32", 64)])
def test_norm_ablation_trajectories(gpu_device, norm_kind, dtype, d):
    """The l2 and l-infinity value norms of the paper's ablation (Table 2) through a whole trajectory."""
    cfg = vs.scaled(vs.CONFIGS["llama7b_layer"], n_heads=3, head_dim=d, prompt_len=333, dtype=dtype,
                    budget_pct=40, recent=32, decode_steps=12)
    _say("norm kind %d %s d=%d" % (norm_kind, dtype, d))
    rep = parity.run_trajectory(vs.make_inputs(cfg, seed=50 + norm_kind), gpu_device, norm_kind=norm_kind)
    _say("report %r" % rep)
