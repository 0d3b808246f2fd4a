"""The C-ABI library loads, exports every symbol the header declares, and
rejects bad arguments on the host before anything is launched (no GPU needed)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    from paper_2509_13232_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2509_13232_amd import build
        build.build()
    return binding.lib()


def _declared():
    text = open(os.path.join(ROOT, "include", "spo.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(spo_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(L):
    from paper_2509_13232_amd import binding
    names = _declared()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert getattr(L, n) is not None


def test_status_strings(L):
    from paper_2509_13232_amd import binding
    assert binding.status_string(0) == "ok"
    seen = {binding.status_string(-i) for i in range(1, 7)}
    assert len(seen) == 6 and "unknown status" not in seen


def test_host_side_argument_checks(L):
    from paper_2509_13232_amd.binding import PgDesc
    one = C.c_void_p(256)  # a non-NULL, aligned dummy; never dereferenced on these paths
    # NULL pointers
    tail = (None, None, None, None, 0, None)   # n_obs, v_prev_out, info, ws, ws_bytes, stream
    assert L.spo_tracker_update(None, None, 4, None, None, None, 1, 0.25, 0.875, 0.96, 1, *tail) == -2
    assert L.spo_tracker_update_ema(None, None, 4, None, None, None, 1, 0.25, 0.875, 0.96, 1, *tail) == -2
    assert L.spo_tracker_update_ema(one, one, 4, one, one, one, 1, -1.0, 0.875, 0.96, 1, *tail) == -1
    assert L.spo_advantages(None, None, 4, None, None, 1, 0, 0.0, 1, None, None, None, None, None, 0, None) == -2
    assert L.spo_sample_prompts(None, None, 4, 1, 0.05, 0, 0, 0, 0, None, None, None, 0, None) == -2
    # bad scalars
    assert L.spo_tracker_update(one, one, 4, one, one, one, 1, 0.0, 0.875, 0.96, 1, *tail) == -1
    assert L.spo_tracker_update(one, one, 4, one, one, one, 1, 0.25, 0.97, 0.96, 1, *tail) == -1
    assert L.spo_tracker_update(one, one, 4, one, one, one, 0, 0.25, 0.875, 0.96, 1, *tail) == -1
    assert L.spo_advantages(one, one, 4, one, one, 0, 0, 0.0, 1, None, one, None, None, None, 0, None) == -1
    assert L.spo_advantages(one, one, 4, one, one, 3, 2, 0.0, 1, None, one, None, None, None, 0, None) == -1
    assert L.spo_advantages(one, one, 4, one, one, 3, 0, 0.0, 1, None, one, None, None, one, 8, None) == -4   # workspace too small
    assert L.spo_advantages_workspace_bytes(1 << 20) == 2 * 256 * 8 and L.spo_advantages_workspace_bytes(0) == 0
    # repeated ids need the slot table; a table that is too small or misaligned is refused
    assert L.spo_tracker_update(one, one, 4, one, one, one, 1, 0.25, 0.875, 0.96, 0, *tail) == -4
    assert L.spo_tracker_update(one, one, 1000, one, one, one, 1, 0.25, 0.875, 0.96, 0, None, None, None, one, 256, None) == -4
    assert L.spo_tracker_update(one, one, 4, one, one, one, 1, 0.25, 0.875, 0.96, 1, None, None, None, C.c_void_p(264), 256, None) == -1
    assert L.spo_tracker_update_workspace_bytes(1 << 20) == 4 << 20
    # sampling more prompts than exist without replacement, too many slots, no workspace
    assert L.spo_sample_prompts(one, one, 4, 5, 0.05, 0, 0, 0, 0, one, None, one, 1 << 20, None) == -1
    assert L.spo_sample_prompts(one, one, 1 << 20, 20000, 0.05, 0, 0, 0, 0, one, None, one, 1 << 30, None) == -3
    assert L.spo_sample_prompts(one, one, 4, 2, 0.05, 0, 0, 0, 0, one, None, None, 0, None) == -4
    assert L.spo_sample_prompts(one, one, 4, 2, 0.05, 0, 0, 0, 0, one, None, one, 8, None) == -4
    assert L.spo_sample_prompts_workspace_bytes(1 << 20, 4096) >= 8 << 20
    # loss descriptor
    d = PgDesc()
    assert L.spo_pg_loss_fwd(None, one, one, one, None, one, 0, None) == -2
    assert L.spo_pg_loss_fwd(C.byref(d), one, one, one, None, one, 0, None) == -1      # struct_size
    d.struct_size = C.sizeof(PgDesc)
    d.dtype, d.w_layout, d.T, d.H, d.V, d.B = 1, 0, 512, 128, 1000, 8
    d.eps_low, d.eps_high = 0.2, 0.28
    assert L.spo_pg_loss_fwd(C.byref(d), one, one, one, None, one, 0, None) == -2      # NULL arrays
    for f in ("hidden", "W", "target", "old_logp", "adv_norm", "cu_seqlens"):
        setattr(d, f, 256)
    assert L.spo_pg_loss_fwd_workspace_bytes(C.byref(d)) > 0
    assert L.spo_pg_loss_fwd(C.byref(d), one, one, one, None, None, 0, None) == -4     # no workspace
    assert L.spo_pg_loss_fwd(C.byref(d), one, one, one, None, one, 16, None) == -4     # too small
    d.H = 100
    assert L.spo_pg_loss_fwd(C.byref(d), one, one, one, None, one, 1 << 30, None) == -5  # H % 64
    d.H = 128
    d.eps_low = -0.1
    assert L.spo_pg_loss_fwd(C.byref(d), one, one, one, None, one, 1 << 30, None) == -1
    d.eps_low = 0.2
    assert L.spo_pg_loss_bwd_workspace_bytes(C.byref(d), 0) > 0
    assert L.spo_pg_loss_bwd(C.byref(d), one, one, 1.0, one, 1, one, 1, 1, None, 0, one, 1 << 40, None) == -1  # bf16 accumulate
    assert L.spo_pg_loss_bwd(C.byref(d), one, one, 1.0, one, 7, one, 0, 0, None, 0, one, 1 << 40, None) == -1  # bad dtype
    assert L.spo_pg_loss_bwd(C.byref(d), None, one, 1.0, one, 1, one, 0, 0, None, 0, one, 1 << 40, None) == -2
    # forward and backward in one call: the checks of both
    fb = L.spo_pg_loss_fwd_bwd
    assert L.spo_pg_loss_fwd_bwd_workspace_bytes(C.byref(d), 0) > 0
    assert L.spo_pg_loss_fwd_bwd_workspace_bytes(C.byref(d), -1) == 0
    assert fb(C.byref(d), 1.0, one, one, one, None, one, 1, one, 1, 1, 0, one, 1 << 40, None) == -1   # bf16 accumulate
    assert fb(C.byref(d), 1.0, one, one, one, None, one, 7, one, 0, 0, 0, one, 1 << 40, None) == -1   # bad dtype
    assert fb(C.byref(d), 1.0, None, one, one, None, one, 1, one, 0, 0, 0, one, 1 << 40, None) == -2  # no loss
    assert fb(C.byref(d), 1.0, one, one, one, None, one, 1, one, 0, 0, -3, one, 1 << 40, None) == -1  # chunk < 0
    assert fb(C.byref(d), 1.0, one, one, one, None, one, 1, one, 0, 0, 0, None, 0, None) == -4        # no workspace
    assert fb(C.byref(d), 1.0, one, one, one, None, one, 1, one, 0, 0, 0, one, 16, None) == -4        # too small
    d.logits = 256
    assert fb(C.byref(d), 1.0, one, one, one, None, one, 1, one, 0, 0, 0, one, 1 << 40, None) == -5   # logits-in form
    assert L.spo_pg_loss_fwd_bwd_workspace_bytes(C.byref(d), 0) == 0
    d.logits = None
    d.hidden = None
    assert L.spo_pg_loss_fwd(C.byref(d), one, one, one, None, one, 1 << 30, None) == -2
    d.hidden = 256
    # the backward workspace grows with the chunk and is bounded by it
    small = L.spo_pg_loss_bwd_workspace_bytes(C.byref(d), 256)
    d.T = 1 << 20
    d.V, d.H = 151936, 4096
    big8k = L.spo_pg_loss_bwd_workspace_bytes(C.byref(d), 8192)
    big32k = L.spo_pg_loss_bwd_workspace_bytes(C.byref(d), 32768)
    assert small < big8k < big32k < 40 << 30
    # one call: a piece's stored logits and its logit gradients, each within 8 GiB by default
    fb0 = L.spo_pg_loss_fwd_bwd_workspace_bytes(C.byref(d), 0)
    fb8k = L.spo_pg_loss_fwd_bwd_workspace_bytes(C.byref(d), 8192)
    assert fb8k < fb0 < 24 << 30 and fb8k > big8k
