"""Glue shared by the test files: build an oracle / a GPU context from a Workload."""
import numpy as np

from oracle.lsam_oracle import LsamOracle


def oracle_from(w, init, **over):
    kw = dict(K=w.K, init_params=init, dims=w.dims, d_raw=w.d_raw, batch=w.batch,
              gemm_dtype=w.gemm_dtype, rho=w.rho, gamma=w.gamma, lr=w.lr,
              lr_center=w.lr_center, momentum=w.momentum, beta=w.beta, lambda0=w.lambda0,
              lambda_abs=w.lambda_abs, nesterov=w.nesterov, tau=w.tau, tau_min=w.tau_min,
              tau_max=w.tau_max, sched_seed=w.sched_seed, sched_mode=w.sched_mode)
    kw.update(over)
    return LsamOracle(**kw)


def rel_l2(a, b):
    a = np.asarray(a, dtype=np.float64).ravel()
    b = np.asarray(b, dtype=np.float64).ravel()
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def rel_max(a, b):
    a = np.asarray(a, dtype=np.float64).ravel()
    b = np.asarray(b, dtype=np.float64).ravel()
    return float(np.max(np.abs(a - b)) / max(np.max(np.abs(b)), 1e-300))
