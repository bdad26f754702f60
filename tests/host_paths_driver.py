"""Runs every host-only path of the library (no GPU call): layout of all workloads, configurations
that must be rejected, schedule replay, argument checks of the entry point that allocates nothing.
Started by test_host_sanitizers.py in a process that preloads the sanitizer runtime, with the
library to load named in LSAM_LIB."""
import ctypes
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
from paper_2509_03110_amd import lsam  # noqa: E402

lsam.LIB_PATH = os.environ["LSAM_LIB"]
import workloads  # noqa: E402

L = lsam.lib()
n = 0
for name, w in sorted(workloads.WORKLOADS.items()):
    cfg, keep = lsam.config_from_workload(w)
    d, ws = L.lsam_num_params(ctypes.byref(cfg)), L.lsam_workspace_bytes(ctypes.byref(cfg))
    assert d == w.d and ws > 0, (name, d, w.d, ws, lsam.last_error())
    n += 1
for over in (dict(K=0), dict(K=65), dict(batch=0), dict(rho=-1.0), dict(momentum=1.0), dict(tau=(0, 1)),
             dict(gemm_dtype=3), dict(dims=(784,) + (16,) * 40 + (10,))):
    cfg, keep = lsam.config_from_workload(workloads.WORKLOADS["cfg1"].scaled(**over))
    assert L.lsam_workspace_bytes(ctypes.byref(cfg)) == 0 and lsam.last_error(), over
for name in ("resnet18", "wrn16x10", "resnet20", "vgg16"):
    base = workloads.WORKLOADS[name]
    for over in (dict(skip_mask=0b10), dict(proj_mask=1 << 1), dict(stride_mask=1 << 40), dict(preact=1, bn_mask=1),
                 dict(img_h=7), dict(pool_mask=1 << 45), dict(dims=base.dims[:-2] + (12, 10)), dict(n_conv=len(base.dims))):
        cfg, keep = lsam.config_from_workload(base.scaled(**over))
        L.lsam_workspace_bytes(ctypes.byref(cfg))       # accepted or rejected: either way without a fault
w = workloads.WORKLOADS["cfg3"]
cfg, keep = lsam.config_from_workload(w.scaled(sched_mode=lsam.SCHED_REDRAW, tau=None))
due = np.zeros((300, w.K), dtype=np.int32)
tau = np.zeros((300, w.K), dtype=np.int32)
assert L.lsam_schedule_replay(ctypes.byref(cfg), 300, due.ctypes.data, tau.ctypes.data) == 0 and due.sum() > 0
u = lsam.lsam_update_desc()
assert L.lsam_step_grads_static(ctypes.byref(u), None, None, None, None, None, None, None, None, None) < 0
assert L.lsam_init(None, None, 0, None, 0, None, None) < 0
print("host paths clean: %d workloads laid out" % n)
