"""Glue shared by the test files: build an oracle / a GPU context from a Workload."""
import numpy as np

from oracle.lsam_oracle import LsamOracle


def oracle_from(w, init, **over):
    kw = dict(K=w.K, init_params=init, dims=w.dims, d_raw=w.d_raw, batch=w.batch,
              gemm_dtype=w.gemm_dtype, rho=w.rho, gamma=w.gamma, lr=w.lr,
              lr_center=w.lr_center, momentum=w.momentum, beta=w.beta, lambda0=w.lambda0,
              lambda_abs=w.lambda_abs, nesterov=w.nesterov, tau=w.tau, tau_min=w.tau_min,
              tau_max=w.tau_max, sched_seed=w.sched_seed, sched_mode=w.sched_mode,
              algorithm=w.algorithm, noise_scale=w.noise_scale, noise_seed=w.noise_seed,
              n_conv=w.n_conv, img_h=w.img_h, img_w=w.img_w, pool_mask=w.pool_mask,
              bn_mask=w.bn_mask, bn_eps=w.bn_eps, stride_mask=w.stride_mask,
              skip_mask=w.skip_mask, global_avg_pool=w.global_avg_pool, proj_mask=w.proj_mask, preact=w.preact)
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


def outlier_fraction(a, b, tol):
    """Fraction of elements whose error exceeds tol * max|b|."""
    a = np.asarray(a, dtype=np.float64).ravel()
    b = np.asarray(b, dtype=np.float64).ravel()
    return float(np.mean(np.abs(a - b) > tol * max(np.max(np.abs(b)), 1e-300)))


def close_enough(a, b, tol, what):
    """The parity criterion for floating-point vectors.

    Relative L2 error <= tol.  Element-wise, |a-b| <= tol * max|b| must hold for all but a
    fraction 2e-3 of the elements, and no element may be off by more than 100 tol * max|b|.
    The allowance exists because the ReLU mask is a decision taken on a rounded value: a
    pre-activation within rounding distance of zero can fall on different sides in fp32 and in
    the float64 oracle, which switches one sample's contribution to one weight row on or off
    (a change of order 1/B of that row's gradient) without either side being wrong."""
    l2, mx, fr = rel_l2(a, b), rel_max(a, b), outlier_fraction(a, b, tol)
    assert l2 <= tol, "%s: relative L2 error %.3e > %.1e" % (what, l2, tol)
    assert fr <= 2e-3, "%s: %.2e of the elements are off by more than %.1e (max %.3e)" % (what, fr, tol, mx)
    assert mx <= 100 * tol, "%s: worst element off by %.3e" % (what, mx)
    return max(l2, mx if fr == 0.0 else l2)


def bn_away_from_zero(w, init):
    """Every normalised layer gets gamma = 0.25 and beta = +1.5 (even channels) or -1.5 (odd
    channels): normalised values lie within about four standard deviations, so a channel is
    either positive everywhere (its ReLU passes everything; shortcuts only add non-negative
    values to it) or negative everywhere (dead, and the shortcut into it comes from a dead
    channel as well), and almost no ReLU decision is taken near zero."""
    init = init.copy()
    model = oracle_from(w.scaled(K=1, tau=(1,)), init).model
    for l, (b0, b1, b2) in model.bn_offsets.items():
        init[b0:b1] = 0.25
        init[b1:b2] = np.where(np.arange(b1 - b0) % 2 == 0, 1.5, -1.5)
    # a normalised projection shortcut adds its own values: same sign per channel as the main branch
    for l, (p0, p1, p2, p3, p4) in model.proj_offsets.items():
        init[p2:p3] = 0.25
        init[p3:p4] = np.where(np.arange(p4 - p3) % 2 == 0, 1.5, -1.5)
    return init
