"""The library's calls only enqueue kernels on the caller's stream (no allocation, no synchronisation, no
memset), so a sequence of them can be recorded into a HIP graph and replayed."""
import sys

import pytest
import torch

import vatp_synth as vs
from paper_2406_12335_amd.runner import PrunedKVCache

pytestmark = pytest.mark.gpu


def _say(msg):
    print("[case] " + msg, flush=True)
    sys.stdout.flush()


def _sequence(cache, inp, dev_tensors, steps):
    Q, K, V, qd, kd, vd = dev_tensors
    cache.prefill_score(Q, K, V, inp.lens)
    cache.prune_prompt(K, V)
    for t in range(steps):
        cache.decode_prune_step(qd[t], kd[t], vd[t], [L + t for L in inp.lens])


def _state(cache):
    c, n = cache.cur, max(cache.lens)
    return [x[c][:, :, :n].clone() for x in (cache.K, cache.V, cache.S, cache.nrm, cache.pos)] + [cache.kept_idx[:, :, :n].clone()]


@pytest.mark.parametrize("q_per_kv", [1, 4])
def test_prompt_pass_prune_and_fused_steps_replay_from_a_graph(gpu_device, q_per_kv):
    dev = gpu_device
    steps = 6                   # an even number: the cache sets end where they started, so every replay starts alike
    cfg = vs.scaled(vs.CONFIGS["llama7b_layer"], n_heads=4, prompt_len=600, decode_steps=steps, q_per_kv=q_per_kv)
    inp = vs.make_inputs(cfg, seed=9)
    tensors = tuple(t.to(dev) for t in (inp.Q, inp.K, inp.V, inp.qd, inp.kd, inp.vd))
    _say("graph capture, q_per_kv=%d" % q_per_kv)
    cache = PrunedKVCache(1, 4, 128, torch.bfloat16, 2, cfg.recent, inp.budgets, dev, q_per_kv=q_per_kv)
    try:
        # eager run: the reference result (also allocates the prompt-side buffers the runner keeps)
        _sequence(cache, inp, tensors, steps)
        torch.cuda.synchronize()
        want = _state(cache)
        lens_after, cur_after, synced_after = list(cache.lens), cache.cur, cache.synced_cur

        def reset_host_side():
            cache._synced_valid = False
            cache.synced_cur = 0

        reset_host_side()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                _sequence(cache, inp, tensors, steps)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        assert (cache.lens, cache.cur) == (lens_after, cur_after)
        scratch = torch.zeros(1 << 20, device=dev)
        for replay in range(3):
            # spoil the outputs, do some eager work of the program's own, then replay
            for x in (cache.K, cache.V, cache.S, cache.nrm):
                x[0].zero_()
                x[1].zero_()
            scratch.add_(1.0)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            got = _state(cache)
            for a, b in zip(got, want):
                assert torch.equal(a, b), "replay %d differs from the eager run" % replay
    finally:
        cache.close()
