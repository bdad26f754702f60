"""CPU-only checks of the C boundary: the library loads, exports every declared symbol, and
its host-side logic (configuration checks, parameter count, schedule replay) is right.
No GPU call is made here."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import workloads
from oracle.lsam_oracle import PeriodSchedule
from paper_2509_03110_amd import lsam

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "lsam.h")).read()
    declared = set(re.findall(r"\b(lsam_[a-z_]+)\s*\(", header))
    declared -= {"lsam_ctx", "lsam_config"}
    assert declared == set(lsam.EXPORTS)
    L = lsam.lib()
    for name in declared:
        assert hasattr(L, name), name


@pytest.mark.parametrize("name", list(workloads.WORKLOADS))
def test_param_count_matches_workload(name):
    w = workloads.WORKLOADS[name]
    cfg, keep = lsam.config_from_workload(w)
    assert lsam.lsam_num_params(cfg) == w.d
    assert lsam.lsam_workspace_bytes(cfg) > 4 * w.K * w.d * 3


def test_bad_configs_are_rejected_with_a_message():
    w = workloads.WORKLOADS["cfg1"]
    for field, value in [("K", 0), ("K", 65), ("batch", 0), ("gemm_dtype", 7), ("rho", -1.0),
                         ("momentum", 1.0), ("sched_mode", 3), ("lr", 0.0), ("algorithm", 2)]:
        cfg, keep = lsam.config_from_workload(w)
        setattr(cfg, field, value)
        assert lsam.lsam_workspace_bytes(cfg) == 0
        assert lsam.last_error()
    cfg, keep = lsam.config_from_workload(w, tau=None, tau_min=3, tau_max=2)
    assert lsam.lsam_num_params(cfg) == -1
    cfg, keep = lsam.config_from_workload(w, tau=(4, 0))
    assert lsam.lsam_num_params(cfg) == -1
    # null arguments never reach the GPU
    cfg, keep = lsam.config_from_workload(w)
    h = C.c_void_p()
    assert lsam.lib().lsam_init(C.byref(cfg), None, 0, None, 0, None, C.byref(h)) == lsam.EINVAL
    assert lsam.lib().lsam_step(None, None, None, None) == lsam.EINVAL
    assert lsam.lib().lsam_sync(None) == lsam.EINVAL


def test_convolutional_configs_are_checked_on_the_host():
    base = workloads.Workload("c", K=2, dims=(3, 8, 16, 24, 5), batch=6, n_conv=2, img_h=8, img_w=8,
                              pool_mask=0b11, n_classes=5)
    cfg, keep = lsam.config_from_workload(base)
    assert lsam.lsam_num_params(cfg) == base.d == 27 * 8 + 8 + 72 * 16 + 16 + 64 * 24 + 24 + 24 * 5 + 5
    bn = base.scaled(bn_mask=0b10)
    cfg, keep = lsam.config_from_workload(bn)
    assert lsam.lsam_num_params(cfg) == bn.d == base.d + 2 * 16
    for over, msg in ((dict(dims=(3, 8, 12, 24, 5)), "multiples of 8"),
                      (dict(img_h=6, img_w=6), "even image sides"),
                      (dict(n_conv=4), "at least one dense layer"),
                      (dict(img_h=0), "img_h"),
                      (dict(bn_mask=0b100), "no convolution"),
                      (dict(bn_mask=0b1, bn_eps=0.0), "bn_eps"),
                      (dict(batch=1 << 22, img_h=64, img_w=64), "too large")):
        cfg, keep = lsam.config_from_workload(base.scaled(**over))
        assert lsam.lsam_workspace_bytes(cfg) == 0, over
        assert msg in lsam.last_error(), (over, lsam.last_error())
    # a dense model must not name normalised layers
    cfg, keep = lsam.config_from_workload(workloads.WORKLOADS["cfg1"].scaled(bn_mask=1))
    assert lsam.lsam_workspace_bytes(cfg) == 0 and "bn_mask" in lsam.last_error()


@pytest.mark.parametrize("mode", [lsam.SCHED_FIXED, lsam.SCHED_REDRAW])
@pytest.mark.parametrize("seed,lo,hi,K", [(0, 2, 8, 4), (5, 4, 16, 16), (123456789, 1, 3, 7)])
def test_schedule_replay_is_bit_exact_with_oracle(mode, seed, lo, hi, K):
    cfg, keep = lsam.make_config(K=K, d_raw=8, tau_min=lo, tau_max=hi, sched_seed=seed,
                                 sched_mode=mode)
    ticks = 200
    due, tau = lsam.lsam_schedule_replay(cfg, ticks)
    s = PeriodSchedule(K, tau_min=lo, tau_max=hi, seed=seed, mode=mode)
    for t in range(ticks):
        assert tau[t].tolist() == s.tau
        s.tick()
        d = s.due()
        assert np.flatnonzero(due[t]).tolist() == d
        if d:
            s.served(d)


def test_schedule_replay_explicit_periods():
    cfg, keep = lsam.make_config(K=3, d_raw=8, tau=(2, 3, 4))
    due, tau = lsam.lsam_schedule_replay(cfg, 12)
    expected = {2: [0], 3: [1], 4: [0, 2], 6: [0, 1], 8: [0, 2], 9: [1], 10: [0], 12: [0, 1, 2]}
    for t in range(12):
        assert np.flatnonzero(due[t]).tolist() == expected.get(t + 1, [])


def test_static_entry_checks_its_arguments_before_touching_the_gpu():
    # limits and null pointers are refused on the host; no device call is reached
    u = lsam.lsam_update_desc()
    lam = (C.c_float * 65)()
    u.K, u.d, u.stride, u.g_stride = 65, 64, 64, 64
    u.lambda_ = C.cast(lam, C.POINTER(C.c_float))
    fake = 4096                                   # never dereferenced: the checks fail first
    call = lsam.lib().lsam_step_grads_static
    assert call(C.byref(u), fake, fake, fake, fake, fake, fake, fake, None, None) == lsam.EINVAL
    assert "K outside" in lsam.last_error()
    u.K, u.d = 4, lsam.STATIC_MAX_D + 1
    u.stride = u.g_stride = u.d
    assert call(C.byref(u), fake, fake, fake, fake, fake, fake, fake, None, None) == lsam.EINVAL
    assert "d outside" in lsam.last_error()
    u.d, u.stride, u.g_stride = 100, 64, 100
    assert call(C.byref(u), fake, fake, fake, fake, fake, fake, fake, None, None) == lsam.EINVAL
    assert "strides" in lsam.last_error()
    assert call(C.byref(u), None, fake, fake, fake, fake, fake, fake, None, None) == lsam.EINVAL
