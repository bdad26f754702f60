"""The entry point that allocates nothing (lsam_step_grads_static) against lsam_step_grads.

Same kernels on the same values: every output must be equal bit for bit.  Two calls in a row,
the second on a smaller problem, so that anything the first call left in the library's fixed
scratch array would show."""
import numpy as np
import pytest
import torch

import workloads
from paper_2509_03110_amd import lsam

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _one_call(K, d, seed, nesterov, rho):
    w = workloads.WORKLOADS["cfg4"].scaled(K=K, d_raw=d, tau=(3,) * K, nesterov=nesterov, rho=rho,
                                           data_seed=seed, momentum=0.8, lr=0.05)
    rng = np.random.default_rng(seed)
    init = rng.standard_normal((K + 1) * d).astype(np.float32)       # distinct x_i and y
    cfg, keep = lsam.config_from_workload(w)
    eng = lsam.Lsam(cfg, init, device=DEV, keep=keep)
    g1, g2 = workloads.raw_grads(w, 0)
    g1d, g2d = torch.from_numpy(g1).to(DEV), torch.from_numpy(g2).to(DEV)
    # one earlier step so that v and S are not zero when the compared step starts
    eng.lsam_step_grads(g2d, g1d)
    x0 = np.stack([eng.lsam_get_params(i) for i in range(K)])
    v0 = np.stack([eng.lsam_get_buffer(lsam.BUF_VELOCITY, i) for i in range(K)])
    S0 = np.stack([eng.lsam_get_buffer(lsam.BUF_ITER_SUM, i) for i in range(K)])
    y0 = eng.lsam_get_params(-1)
    eng.lsam_step_grads(g1d, g2d)
    want = {"x": np.stack([eng.lsam_get_params(i) for i in range(K)]),
            "v": np.stack([eng.lsam_get_buffer(lsam.BUF_VELOCITY, i) for i in range(K)]),
            "S": np.stack([eng.lsam_get_buffer(lsam.BUF_ITER_SUM, i) for i in range(K)]),
            "xt": np.stack([eng.lsam_get_buffer(lsam.BUF_PERTURBED, i) for i in range(K)]),
            "norms": eng.lsam_get_norms()}
    eng.close()

    pad = (d + 63) // 64 * 64                # the row stride the context uses for its own state
    def dev(a):
        t = torch.zeros(K, pad, device=DEV)
        t[:, :d] = torch.from_numpy(a).to(DEV)
        return t
    x, v, S = dev(x0), dev(v0), dev(S0)
    xt = torch.full((K, pad), 7.0, device=DEV)
    y = torch.from_numpy(y0).to(DEV)
    norms = torch.zeros(K, device=DEV)
    lam = [w.lambda0 / (np.float64(np.float32(w.lr)) * 3)] * K       # lambda0 / (eta tau_i)
    lsam.lsam_step_grads_static(x, v, S, y, g1d, g2d, xt if rho else None, norms, lam, rho=w.rho,
                                gamma=w.gamma, lr=w.lr, momentum=w.momentum, nesterov=nesterov, d=d)
    torch.cuda.synchronize()
    assert np.array_equal(norms.cpu().numpy(), want["norms"])
    assert np.array_equal(x.cpu().numpy()[:, :d], want["x"])
    assert np.array_equal(v.cpu().numpy()[:, :d], want["v"])
    assert np.array_equal(S.cpu().numpy()[:, :d], want["S"])
    if rho:
        assert np.array_equal(xt.cpu().numpy()[:, :d], want["xt"])
        assert np.all(xt.cpu().numpy()[:, d:] == 7.0)                # nothing written past d
    assert np.all(x.cpu().numpy()[:, d:] == 0.0)


def test_static_entry_matches_the_context_call_twice_in_a_row():
    _one_call(K=5, d=65536 * 3 + 40, seed=21, nesterov=1, rho=0.05)   # several partial sums per replica
    _one_call(K=2, d=1000, seed=22, nesterov=0, rho=0.05)             # smaller: one partial sum
    _one_call(K=3, d=4099, seed=23, nesterov=1, rho=0.0)              # rho = 0: no x~ written


def test_static_entry_rejects_what_is_beyond_its_limits():
    z = torch.zeros(4, 64, device=DEV)
    with pytest.raises(lsam.LsamError) as e:
        lsam.lsam_step_grads_static(torch.zeros(65, 64, device=DEV), z, z, z[0], z, z, z, None,
                                    [0.0] * 65, rho=0.1, gamma=0.0, lr=0.1, momentum=0.9, nesterov=1)
    assert e.value.code == lsam.EINVAL and "K outside" in str(e.value)
    with pytest.raises(lsam.LsamError):
        lsam.lsam_step_grads_static(z, z, z, z[0], z, z, z, None, [0.0] * 4, rho=0.1, gamma=0.0, lr=0.1,
                                    momentum=0.9, nesterov=1, d=lsam.STATIC_MAX_D + 1)
