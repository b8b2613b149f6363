"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol
the header declares, and rejects bad arguments before touching a device."""
import os
import re

import pytest
import torch

import paper_2406_12335_amd as vatp
from paper_2406_12335_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "vatp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(vatp_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = vatp.load()
    names = _declared_symbols()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def _params(**kw):
    base = dict(batch=2, n_heads=4, head_dim=128, dtype=vatp.VATP_BF16, n_sink=2, recent=8, cap=64,
                len=[64, 10], budget=[32, 32])
    base.update(kw)
    return vatp.Params(**base)


def test_validate_accepts_good_params():
    for call in (vatp.CALL_PREFILL_SCORE, vatp.CALL_SELECT_COMPACT):
        assert vatp.vatp_validate(_params(), call) == binding.OK
    assert vatp.vatp_validate(_params(len=[63, 10]), vatp.CALL_DECODE_STEP) == binding.OK
    assert vatp.vatp_validate(_params(len=[32, 10]), vatp.CALL_DECODE_PRUNE_STEP) == binding.OK


@pytest.mark.parametrize("kw,call,want", [
    (dict(dtype=7), 0, binding.E_DTYPE),
    (dict(head_dim=96), 0, binding.E_SHAPE),
    (dict(batch=0, len=[], budget=[]), 0, binding.E_SHAPE),
    (dict(batch=257, len=[1] * 257, budget=[32] * 257), 0, binding.E_SHAPE),
    (dict(n_heads=16384), 0, binding.E_SHAPE),
    (dict(len=[65, 1]), 0, binding.E_SHAPE),
    (dict(len=[-1, 1]), 0, binding.E_SHAPE),
    (dict(len=[64, 1]), vatp.CALL_DECODE_STEP, binding.E_SHAPE),          # no room to append
    (dict(budget=[9, 32]), vatp.CALL_SELECT_COMPACT, binding.E_BUDGET),   # B < F + R
    (dict(cap_out=16), vatp.CALL_SELECT_COMPACT, binding.E_BUDGET),       # survivors do not fit
    (dict(budget=None), vatp.CALL_SELECT_COMPACT, binding.E_NULL),
    (dict(len=None), 0, binding.E_NULL),
    (dict(len=[33, 10]), vatp.CALL_DECODE_PRUNE_STEP, binding.E_BUDGET),  # two rows would have to leave
    (dict(len=[64, 10]), vatp.CALL_DECODE_PRUNE_STEP, binding.E_SHAPE),   # no room to append
    (dict(budget=None), vatp.CALL_DECODE_PRUNE_STEP, binding.E_NULL),
    (dict(scale=float("nan")), 0, binding.E_SHAPE),
    (dict(n_sink=-1), 0, binding.E_SHAPE),
])
def test_validate_rejects(kw, call, want):
    assert vatp.vatp_validate(_params(**kw), call) == want


def test_workspace_bytes():
    p = _params()
    units, cap = 8, 64
    assert vatp.vatp_workspace_bytes(None, p, vatp.CALL_PREFILL_SCORE) == units * cap * 4
    dec = vatp.vatp_workspace_bytes(None, _params(len=[10, 10]), vatp.CALL_DECODE_STEP)
    assert dec >= units * cap * 4 and dec % 256 == 0
    assert vatp.vatp_workspace_bytes(None, p, vatp.CALL_SELECT_COMPACT) == 0
    assert vatp.vatp_workspace_bytes(None, _params(dtype=9), vatp.CALL_PREFILL_SCORE) == 0
    # windowed prompt pass: row statistics plus one set of partial statistics per 2048 keys
    assert vatp.vatp_workspace_bytes(None, p, vatp.CALL_PREFILL_SCORE_WINDOW) == 2 * units * cap * 4
    big = _params(cap=5000, len=[5000, 1], budget=[2500, 2500])
    assert vatp.vatp_workspace_bytes(None, big, vatp.CALL_PREFILL_SCORE_WINDOW) == 4 * units * 5000 * 4


def test_entry_points_reject_null_before_any_launch():
    lib = vatp.load()
    p = _params()
    assert lib.vatp_prefill_score(None, p.ref(), None, None, None, None, None, None, 0, None) == binding.E_NULL
    assert lib.vatp_decode_step(None, p.ref(), *([None] * 9), None, 0, None) == binding.E_NULL
    assert lib.vatp_select_compact(None, p.ref(), *([None] * 11), None, 0, None) == binding.E_NULL
    assert lib.vatp_decode_prune_step(None, p.ref(), *([None] * 18), None, 0, None) == binding.E_NULL
    assert lib.vatp_prefill_score_window(None, p.ref(), None, None, None, 4, None, None, None, None, 0, None) == binding.E_NULL
    assert lib.vatp_prefill_score_window(None, p.ref(), None, None, None, -1, None, None, None, None, 0, None) == binding.E_SHAPE
    assert lib.vatp_select_compact_window(None, p.ref(), *([None] * 6), 4, *([None] * 7), 64, None, None, None, None, 0,
                                          None) == binding.E_NULL
    assert lib.vatp_decode_prune_step_window(None, p.ref(), *([None] * 9), None, *([None] * 14), 4, 64, None, None, 0,
                                             None) == binding.E_NULL
    assert "NULL" in vatp.strerror(binding.E_NULL)
    assert vatp.strerror(-99) == "unknown status"


def test_create_without_device_is_an_error_not_a_crash():
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(vatp.VatpError) as e:
        vatp.vatp_create(0)
    assert e.value.status == binding.E_DEVICE
    lib = vatp.load()
    assert lib.vatp_create(None, 0) == binding.E_NULL
    lib.vatp_destroy(None)


def test_validate_rejects_unknown_norm():
    assert vatp.vatp_validate(_params(norm=4), 0) == binding.E_SHAPE
    assert vatp.vatp_validate(_params(norm=-1), 0) == binding.E_SHAPE
    for kind in (vatp.NORM_L1, vatp.NORM_L2, vatp.NORM_LINF, vatp.NORM_NONE):
        assert vatp.vatp_validate(_params(norm=kind), 0) == binding.OK


def test_validate_grouped_queries():
    """q_per_kv: 0 and 1 are plain multi-head attention, up to 16 query heads per K/V head."""
    import torch
    from paper_2406_12335_amd import binding as B
    for g, call, want in [(0, B.CALL_PREFILL_SCORE, B.OK), (1, B.CALL_DECODE_STEP, B.OK), (8, B.CALL_PREFILL_SCORE, B.OK),
                          (16, B.CALL_PREFILL_SCORE, B.OK), (17, B.CALL_PREFILL_SCORE, B.E_SHAPE), (-1, B.CALL_DECODE_STEP, B.E_SHAPE),
                          (2, B.CALL_PREFILL_SCORE_WINDOW, B.OK), (4, B.CALL_DECODE_PRUNE_STEP, B.OK)]:
        p = B.Params(1, 4, 128, torch.bfloat16, 2, 8, 128, [40], [50], q_per_kv=g)
        assert B.vatp_validate(p, call) == want, (g, call)
    # the unit limit counts query heads
    p = B.Params(64, 64, 128, torch.bfloat16, 0, 0, 16, [8] * 64, None, q_per_kv=8)
    assert B.vatp_validate(p, B.CALL_PREFILL_SCORE) == B.E_SHAPE
    # the workspace holds one set of logits / row statistics per query head
    p1 = B.Params(2, 4, 128, torch.bfloat16, 0, 0, 512, [100, 100], None)
    p4 = B.Params(2, 4, 128, torch.bfloat16, 0, 0, 512, [100, 100], None, q_per_kv=4)
    for call in (B.CALL_DECODE_STEP, B.CALL_DECODE_ATTEND_STEP):
        assert B.vatp_workspace_bytes(None, p4, call) == 4 * B.vatp_workspace_bytes(None, p1, call)
    # (the prompt pass also keeps room for partial column sums of a group: as much again)
    assert B.vatp_workspace_bytes(None, p4, B.CALL_PREFILL_SCORE) == 8 * B.vatp_workspace_bytes(None, p1, B.CALL_PREFILL_SCORE)


def test_header_is_plain_c(tmp_path):
    """include/vatp.h compiles as C99 with nothing but the standard headers, and a C caller can take the address
    of every entry point it declares."""
    import os
    import subprocess
    from paper_2406_12335_amd import binding as B
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    src = tmp_path / "use_vatp.c"
    lines = ['#include "vatp.h"', "typedef void (*fn)(void);", "fn table[] = {"]
    lines += ["    (fn)%s," % name for name in B.EXPORTS]
    lines += ["};", "int n_entries(void) { vatp_params p; p.q_per_kv = 0; (void)p; return (int)(sizeof table / sizeof table[0]); }"]
    src.write_text("\n".join(lines) + "\n")
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(root, "include"),
                           "-c", str(src), "-o", str(tmp_path / "use_vatp.o")])


def test_built_library_matches_its_sources():
    """build_library() leaves a digest of sources, headers and flags beside the library; load() rebuilds when it no
    longer matches.  Here: the digest is reproducible, the library that is loaded is current, and a change to any
    source byte changes the digest."""
    import shutil
    from paper_2406_12335_amd import build
    vatp.load()
    assert build.is_current()
    d0 = build.source_digest()
    assert d0 == build.source_digest() and len(d0) == 64
    victim = os.path.join(build.CSRC, "l1norm.hip")
    backup = victim + ".bak_test"
    shutil.copy2(victim, backup)
    try:
        with open(victim, "a") as f:
            f.write("// touched by test_built_library_matches_its_sources\n")
        assert build.source_digest() != d0 and not build.is_current()
    finally:
        shutil.move(backup, victim)
    assert build.source_digest() == d0 and build.is_current()
