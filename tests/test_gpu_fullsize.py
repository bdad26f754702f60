"""GPU parity at the full sizes the benchmark runs, in the benchmark's launch configuration.

A float64 oracle of every replica at these sizes would take many minutes, so each test checks
what the oracle can reach in seconds and covers the rest by properties that hold at any size:

  * update-only path (K=8, d=1e8): the update is coordinate-wise once the per-replica norm is
    known, so the oracle runs on a sample of 200 000 coordinates plus one extra coordinate
    that carries the norm of all the others (||g1|| is then exactly the full-vector norm);
    the GPU's norms are also compared with the float64 norm of the whole vector.
  * bf16 MLP shapes (cfg3: K=8, width 4096, B=256; cfg5: K=16, width 8192, B=512): the oracle
    computes one whole replica; several other replicas get the same batch and must reproduce
    that replica's loss and gradients bit for bit (the kernels are deterministic and
    replica-independent), the remaining ones are checked for finite, plausible output.
"""
import numpy as np
import pytest
import torch

import workloads
from paper_2509_03110_amd import lsam
from util import bn_away_from_zero, close_enough, oracle_from, rel_max

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def test_update_path_full_size_sampled():
    w = workloads.WORKLOADS["cfg4"]
    K, d = w.K, w.d_raw
    rng = np.random.default_rng(44)
    J = np.sort(rng.choice(d, size=200_000, replace=False))
    init = workloads.init_params(w)                       # y = x_i ~ N(0,1) [1e8]
    g1 = np.empty((K, d), dtype=np.float32)
    g2 = np.empty((K, d), dtype=np.float32)
    gen = np.random.default_rng([w.data_seed, 77])
    for k in range(K):                                    # fixed gradient buffers ~ N(0, 1e-2^2)
        g1[k] = gen.standard_normal(d, dtype=np.float32) * np.float32(w.grad_std)
        g2[k] = gen.standard_normal(d, dtype=np.float32) * np.float32(w.grad_std)
    full_norm = np.array([np.sqrt(np.sum(np.square(g1[k], dtype=np.float64))) for k in range(K)])
    rest = np.sqrt(np.maximum(full_norm ** 2 - np.sum(np.square(g1[:, J], dtype=np.float64), axis=1), 0))
    g1s = np.concatenate([g1[:, J].astype(np.float64), rest[:, None]], axis=1)
    g2s = np.concatenate([g2[:, J].astype(np.float64), np.zeros((K, 1))], axis=1)
    ws = w.scaled(d_raw=J.size + 1)
    ora = oracle_from(ws, np.concatenate([init[J].astype(np.float64), [0.0]]))

    cfg, keep = lsam.config_from_workload(w)
    eng = lsam.Lsam(cfg, init, device=DEV, keep=keep)
    g1d, g2d = torch.from_numpy(g1).to(DEV), torch.from_numpy(g2).to(DEV)
    del g1, g2
    for t in range(8):
        eng.lsam_step_grads(g1d, g2d)
        ora.step_grads(g1s, g2s)
        assert np.allclose(eng.lsam_get_norms(), full_norm, rtol=1e-6)
        assert np.allclose(ora.last_norm, full_norm, rtol=1e-12)
        assert eng.lsam_sync() == ora.sync()
        assert eng.lsam_get_schedule() == ora.get_schedule()
    for i in list(range(K)) + [-1]:
        close_enough(eng.lsam_get_params(i)[J], ora.get_params(i)[:-1], 1e-4, "x of replica %d" % i)
    for i in (0, K - 1):
        close_enough(eng.lsam_get_buffer(lsam.BUF_VELOCITY, i)[J], ora.v[i][:-1], 1e-4, "v %d" % i)
        close_enough(eng.lsam_get_buffer(lsam.BUF_ITER_SUM, i)[J], ora.S[i][:-1], 1e-4, "S %d" % i)
        xt = eng.lsam_get_buffer(lsam.BUF_PERTURBED, i)[J]
        assert rel_max(xt, ora.last_perturbed[i][:-1]) < 1e-5
    eng.close()


def _full_shape_one_replica(name, twins):
    w = workloads.WORKLOADS[name]
    init = workloads.init_params(w)
    cfg, keep = lsam.config_from_workload(w)
    eng = lsam.Lsam(cfg, init, device=DEV, keep=keep)
    tau0 = eng.lsam_get_schedule()[0][0]
    X, lab = workloads.batch(w, 0)
    for k in twins:                      # replicas that see replica 0's batch
        X[k], lab[k] = X[0], lab[0]
    loss = torch.zeros(w.K, device=DEV)
    eng.lsam_step(torch.from_numpy(X).to(DEV).to(torch.bfloat16).contiguous(),
                  torch.from_numpy(lab).to(DEV), loss)
    gl = loss.cpu().numpy()
    ora = oracle_from(w.scaled(K=1, tau=(tau0,)), init)
    ol = ora.step(X[:1], lab[:1])
    assert abs(gl[0] - ol[0]) <= 2e-2 * abs(ol[0])
    assert abs(eng.lsam_get_norms()[0] - ora.last_norm[0]) <= 5e-2 * ora.last_norm[0]
    # these configurations run fused (as bench.py times them): the weight matrices' gradients are
    # never stored -- the first pass's goes into the norm and, recomputed, into the perturbed
    # operand copy; the second pass's straight into the sampler step -- so they are checked through
    # the norm above, the perturbed copy, v and x; the bias gradients are stored as always
    assert eng.lsam_set_fused_step(True) == 1
    g2 = eng.lsam_get_buffer(lsam.BUF_GRAD, 0)
    for l, (o0, o1, o2) in enumerate(ora.model.offsets):
        # (the first layers' bias gradients are the smallest and noisiest part of g2: seven layers of
        # bf16 operand rounding and of ReLU decisions above them; 1.1e-1 measured for b1 of config 5)
        close_enough(g2[o1:o2], ora.last_g2[0][o1:o2], 2e-1, "%s full shape: g2 of b%d, replica 0" % (name, l + 1))
    close_enough(eng.lsam_get_params(0), ora.get_params(0), 2e-2, "%s full shape: x of replica 0" % name)
    close_enough(eng.lsam_get_buffer(lsam.BUF_VELOCITY, 0), ora.v[0], 1e-1, "%s full shape: v" % name)
    for k in twins:
        assert gl[k] == gl[0]
        assert np.array_equal(eng.lsam_get_buffer(lsam.BUF_GRAD, k), g2), "replica %d differs" % k
    norms = eng.lsam_get_norms()
    assert np.all(np.isfinite(gl)) and np.all(np.isfinite(norms)) and np.all(norms > 0)
    assert np.all(np.abs(gl - np.log(w.n_classes)) < 0.5)     # near-uniform predictions at init
    eng.close()


def test_cfg3_full_shape_one_replica():
    _full_shape_one_replica("cfg3", twins=(3, 7))


def test_cfg5_full_shape_one_replica():
    _full_shape_one_replica("cfg5", twins=(6, 15))


def test_fp32_large_tile_variants_one_replica():
    """fp32 shapes large enough for the 256x128 (forward) and 256x256 (weight-gradient) tile
    variants of the fp32 GEMM, which the small parity cases never reach.  The oracle computes
    replica 0 from a margin initialisation (no ReLU decision near zero, so the tight fp32
    bound applies to every buffer); twin replicas must reproduce it bit for bit."""
    w = workloads.Workload("fp32big", K=16, dims=(256, 2048, 2048, 24), batch=512, rho=0.05,
                           lr=0.01, tau=(3,) * 16, n_classes=24, data_seed=21)
    init = workloads.init_params_margin(w)
    cfg, keep = lsam.config_from_workload(w)
    eng = lsam.Lsam(cfg, init, device=DEV, keep=keep)
    X, lab = workloads.batch(w, 0)
    twins = (5, 15)
    for k in twins:
        X[k], lab[k] = X[0], lab[0]
    loss = torch.zeros(w.K, device=DEV)
    eng.lsam_step(torch.from_numpy(X).to(DEV), torch.from_numpy(lab).to(DEV), loss)
    gl = loss.cpu().numpy()
    ora = oracle_from(w.scaled(K=1, tau=(3,)), init)
    ol = ora.step(X[:1], lab[:1])
    assert ora.model.last_margin > 1e-3
    assert abs(gl[0] - ol[0]) <= 1e-5 * abs(ol[0])
    assert abs(eng.lsam_get_norms()[0] - ora.last_norm[0]) <= 1e-5 * ora.last_norm[0]
    g2 = eng.lsam_get_buffer(lsam.BUF_GRAD, 0)
    for l, (o0, o1, o2) in enumerate(ora.model.offsets):
        close_enough(g2[o0:o1], ora.last_g2[0][o0:o1], 1e-4, "dW%d" % (l + 1))
        close_enough(g2[o1:o2], ora.last_g2[0][o1:o2], 1e-4, "db%d" % (l + 1))
    close_enough(eng.lsam_get_params(0), ora.get_params(0), 1e-4, "x of replica 0")
    close_enough(eng.lsam_get_buffer(lsam.BUF_VELOCITY, 0), ora.v[0], 1e-4, "v of replica 0")
    for k in twins:
        assert gl[k] == gl[0]
        assert np.array_equal(eng.lsam_get_buffer(lsam.BUF_GRAD, k), g2), "replica %d differs" % k
    assert np.all(np.isfinite(gl)) and np.all(np.isfinite(eng.lsam_get_norms()))
    eng.close()


@pytest.mark.parametrize("name", ["cnn5", "cnn5bn"])
def test_cnn5_full_size_two_steps_all_replicas(name):
    # the paper's own shape (4 workers, batch 128, 32x32x3 images): the oracle still reaches
    # every replica in seconds, so the whole state is compared.  A replica takes about 5e6 ReLU
    # and 1.3e6 pooling decisions per pass; a pre-activation (or two values of a pooling
    # window) within fp32 rounding distance can fall differently in float64, and one such
    # decision moves one of the 1.3e5 terms of a first-layer weight-gradient row.  Gradients
    # are therefore held to the looser bound, layer by layer, parameters to the tight one
    # (tests/test_gpu_parity.py holds the gradients to 1e-5 where every decision is exact).
    w = workloads.WORKLOADS[name].scaled(tau=(2, 2, 2, 2))
    init = workloads.init_params(w)
    cfg, keep = lsam.config_from_workload(w)
    eng = lsam.Lsam(cfg, init, device=DEV, keep=keep)
    ora = oracle_from(w, init)
    loss = torch.zeros(w.K, dtype=torch.float32, device=DEV)
    for t in range(2):
        X, lab = workloads.batch(w, t)
        eng.lsam_step(torch.from_numpy(X).to(DEV), torch.from_numpy(lab).to(DEV), loss)
        ol = ora.step(X, lab)
        assert np.allclose(loss.cpu().numpy(), ol, rtol=1e-5)
        assert np.allclose(eng.lsam_get_norms(), ora.last_norm, rtol=1e-3)
        if t == 0:
            for i in range(w.K):
                g2 = eng.lsam_get_buffer(lsam.BUF_GRAD, i)
                for l, (o0, o1, o2) in enumerate(ora.model.offsets):
                    close_enough(g2[o0:o1], ora.last_g2[i][o0:o1], 2e-2, "dW%d of replica %d" % (l + 1, i))
                    if l in ora.model.bn_offsets:
                        # the bias below a normalisation has a gradient of exactly zero; what
                        # either side computes for it is rounding noise
                        assert np.max(np.abs(g2[o1:o2])) < 1e-3 * np.max(np.abs(g2[o0:o1]))
                        b0, b1, b2 = ora.model.bn_offsets[l]
                        close_enough(g2[b0:b1], ora.last_g2[i][b0:b1], 2e-2, "dgamma%d of replica %d" % (l + 1, i))
                        close_enough(g2[b1:b2], ora.last_g2[i][b1:b2], 2e-2, "dbeta%d of replica %d" % (l + 1, i))
                    else:
                        close_enough(g2[o1:o2], ora.last_g2[i][o1:o2], 2e-2, "db%d of replica %d" % (l + 1, i))
        assert eng.lsam_sync() == ora.sync()
        for i in list(range(w.K)) + [-1]:
            close_enough(eng.lsam_get_params(i), ora.get_params(i), 1e-4 if t == 0 else 1e-3,
                         "x of replica %d after step %d" % (i, t + 1))
    assert eng.lsam_get_schedule() == ora.get_schedule()
    eng.close()


@pytest.mark.parametrize("name,tol", [("vgg16", 1e-4), ("vgg16bf", 2e-2)])
def test_vgg16_reduced_batch_against_oracle_and_full_batch_properties(name, tol):
    # Sixteen weight layers, thirteen of them batch-normalised convolutions.  The float64 oracle
    # needs two minutes for one replica at batch 128, and batch normalisation ties the samples of
    # a batch together, so no subset of a batch can be checked on its own: the oracle comparison
    # runs one replica at batch 8 (same layers, same kernels, other grid sizes), and the full
    # shape is checked for what must hold at any size: replicas that are given the same batch
    # reproduce each other bit for bit (kernels are deterministic and replica-independent), the
    # loss at the initial point is near log(10), the schedule is exact.
    full = workloads.WORKLOADS[name]
    w = full.scaled(K=1, batch=8, tau=(2,))
    init = workloads.init_params(w)
    cfg, keep = lsam.config_from_workload(w)
    eng = lsam.Lsam(cfg, init, device=DEV, keep=keep)
    ora = oracle_from(w, init)
    loss = torch.zeros(w.K, dtype=torch.float32, device=DEV)
    X, lab = workloads.batch(w, 0)
    eng.lsam_step(torch.from_numpy(X).to(DEV), torch.from_numpy(lab).to(DEV), loss)
    ol = ora.step(X, lab)
    assert np.allclose(loss.cpu().numpy(), ol, rtol=max(tol, 1e-4))
    assert np.allclose(eng.lsam_get_norms(), ora.last_norm, rtol=max(tol, 5e-3))
    if name == "vgg16":
        close_enough(eng.lsam_get_buffer(lsam.BUF_GRAD, 0), ora.last_g2[0], 5e-2, "g2")
    # With bf16 products the gradient of this network is not a well-conditioned function of its
    # inputs at batch 8: in the oracle alone, relative noise of 3e-8 on the operands before they
    # are rounded (the difference between fp32 and float64 activations) moves operands across
    # bf16 rounding boundaries and, thirteen normalised layers and their ReLU and pooling
    # decisions later, changes the gradient by 30 % (1 % in the last layer).  An element-wise
    # gradient comparison would test that noise, not the kernels; the bf16 kernels are held to
    # the oracle element-wise on the small and medium shapes of tests/test_gpu_parity.py; here
    # the loss and the gradient norm have to stay within the bf16 tolerance.
    if name == "vgg16":
        close_enough(eng.lsam_get_params(0), ora.get_params(0), tol, "x after one step")
    eng.close()

    w = full.scaled(tau=(2, 2, 2, 2))
    cfg, keep = lsam.config_from_workload(w)
    eng = lsam.Lsam(cfg, init, device=DEV, keep=keep)
    loss = torch.zeros(w.K, dtype=torch.float32, device=DEV)
    X, lab = workloads.batch(w, 0)
    X[2], lab[2] = X[0], lab[0]                    # replicas 0 and 2 see the same batch
    for t in range(2):
        eng.lsam_step(torch.from_numpy(X).to(DEV), torch.from_numpy(lab).to(DEV), loss)
        lg = loss.cpu().numpy()
        assert np.all(np.isfinite(lg)) and lg[0] == lg[2]
        if t == 0:
            assert np.all(np.abs(lg - np.log(10.0)) < 0.5), lg
        # before the first center update the two replicas are the same computation
        assert np.array_equal(eng.lsam_get_buffer(lsam.BUF_GRAD, 0), eng.lsam_get_buffer(lsam.BUF_GRAD, 2))
        if t == 0:
            assert np.array_equal(eng.lsam_get_params(0), eng.lsam_get_params(2))
            assert not np.array_equal(eng.lsam_get_params(0), eng.lsam_get_params(1))
    assert eng.lsam_sync() == 4
    assert eng.lsam_get_schedule() == ([2, 2, 2, 2], [0, 0, 0, 0], 1)
    eng.close()


_bn_away_from_zero = bn_away_from_zero


@pytest.mark.parametrize("natural", [False, True])
def test_resnet20_full_size_one_step_against_the_oracle(natural):
    # ResNet-20 at the paper's shape (4 workers, batch 128, 32x32x3 images, 19 batch-normalised
    # convolutions in 9 residual blocks, global average pooling).  The GPU steps all four
    # replicas; the oracle, at 18 s per replica, follows the last one (replicas are independent
    # until the first center update).
    # natural = False: normalisation parameters that keep the ReLU decisions away from zero.
    # Then the gradient of the pass at the perturbed point must agree layer by layer to 2e-3
    # (measured: 1e-6 in the first two stages, up to 6e-4 in the third, whose sums run over
    # 8192 positions only) and the parameters after the step to 1e-6.
    # natural = True: the workload's own initialisation.  Each of the 19 layers takes 0.5 to
    # 2 million ReLU decisions per pass on values the normalisation has centred at zero; those
    # within fp32 rounding of zero fall differently in float64, and each one moves one of the
    # B H W terms of a weight-gradient row, so the gradients agree to a few percent only
    # (measured 1e-2 at the top to 3e-2 at the stem) while loss and norm agree to 1e-5 / 1e-3.
    w = workloads.WORKLOADS["resnet20"]
    init = workloads.init_params(w)
    if not natural:
        init = _bn_away_from_zero(w, init)
    cfg, keep = lsam.config_from_workload(w)
    eng = lsam.Lsam(cfg, init, device=DEV, keep=keep)
    loss = torch.zeros(w.K, dtype=torch.float32, device=DEV)
    X, lab = workloads.batch(w, 0)
    eng.lsam_step(torch.from_numpy(X).to(DEV), torch.from_numpy(lab).to(DEV), loss)
    gl, norms = loss.cpu().numpy(), eng.lsam_get_norms()
    i = w.K - 1
    ora = oracle_from(w.scaled(K=1, tau=(w.tau[i],)), init)
    ol = ora.step(X[i:i + 1], lab[i:i + 1])
    tol_g, tol_x = (1e-1, 2e-3) if natural else (2e-3, 1e-6)
    assert abs(gl[i] - ol[0]) <= 1e-5 * abs(ol[0])
    assert abs(norms[i] - ora.last_norm[0]) <= 1e-3 * ora.last_norm[0]
    g2 = eng.lsam_get_buffer(lsam.BUF_GRAD, i)
    worst = 0.0
    for l, (o0, o1, o2) in enumerate(ora.model.offsets):
        worst = max(worst, close_enough(g2[o0:o1], ora.last_g2[0][o0:o1], tol_g, "dW%d" % (l + 1)))
        if l in ora.model.bn_offsets:
            b0, b1, b2 = ora.model.bn_offsets[l]
            close_enough(g2[b0:b1], ora.last_g2[0][b0:b1], tol_g, "dgamma%d" % (l + 1))
            close_enough(g2[b1:b2], ora.last_g2[0][b1:b2], tol_g, "dbeta%d" % (l + 1))
        else:
            close_enough(g2[o1:o2], ora.last_g2[0][o1:o2], tol_g, "db%d" % (l + 1))
    ex = close_enough(eng.lsam_get_params(i), ora.get_params(0), tol_x, "x after one step")
    print("resnet20 full size, natural=%s: worst weight-gradient error %.2e, parameters %.2e" % (natural, worst, ex))
    assert eng.lsam_sync() == 0
    eng.close()


@pytest.mark.parametrize("name,batch", [("resnet18", 16), ("resnet34", 8), ("wrn16x10", 4), ("wrn40x10", 2)])
def test_resnet18_and_34_full_model_one_step_against_the_oracle(name, batch):
    # ResNet-18 / ResNet-34 with every layer at its real shape (32x32x3 images, stages of 64 to
    # 512 channels, projection shortcuts where a stage begins, 4 workers) at a batch the oracle
    # finishes in half a minute for one replica (it needs 1.7 s per sample and pass here).  The
    # GPU steps all four replicas, the oracle follows the last one.  Normalisation parameters
    # that keep ReLU decisions away from zero, as in the ResNet-20 test above, so that gradients
    # can be held to 2e-3 group by group, the projection's own included.
    # The wide residual networks WRN-16x10 and WRN-40x10 (pre-activation blocks, 160 to 640
    # channels, 14 resp. 38 weight layers) the same way at batch 4 resp. 2: 10 s per sample and
    # pass in the oracle.  (WRN-28x10 lies between the two and has no shape of its own.)
    w = workloads.WORKLOADS[name].scaled(batch=batch)
    init = _bn_away_from_zero(w, workloads.init_params(w))
    cfg, keep = lsam.config_from_workload(w)
    eng = lsam.Lsam(cfg, init, device=DEV, keep=keep)
    loss = torch.zeros(w.K, dtype=torch.float32, device=DEV)
    X, lab = workloads.batch(w, 0)
    eng.lsam_step(torch.from_numpy(X).to(DEV), torch.from_numpy(lab).to(DEV), loss)
    gl, norms = loss.cpu().numpy(), eng.lsam_get_norms()
    i = w.K - 1
    ora = oracle_from(w.scaled(K=1, tau=(w.tau[i],)), init)
    ol = ora.step(X[i:i + 1], lab[i:i + 1])
    assert abs(gl[i] - ol[0]) <= 1e-5 * abs(ol[0])
    assert abs(norms[i] - ora.last_norm[0]) <= 1e-3 * ora.last_norm[0]
    g2 = eng.lsam_get_buffer(lsam.BUF_GRAD, i)
    worst = 0.0
    for l, (o0, o1, o2) in enumerate(ora.model.offsets):
        worst = max(worst, close_enough(g2[o0:o1], ora.last_g2[0][o0:o1], 2e-3, "dW%d" % (l + 1)))
        if l in ora.model.bn_offsets:
            b0, b1, b2 = ora.model.bn_offsets[l]
            close_enough(g2[b0:b2], ora.last_g2[0][b0:b2], 2e-3, "dgamma, dbeta %d" % (l + 1))
        if l in ora.model.proj_offsets:
            p0, p1, p2, p3, p4 = ora.model.proj_offsets[l]
            worst = max(worst, close_enough(g2[p0:p1], ora.last_g2[0][p0:p1], 2e-3, "dW_p %d" % (l + 1)))
            if p4 > p2:      # (a pre-activation projection has no normalisation)
                close_enough(g2[p2:p4], ora.last_g2[0][p2:p4], 2e-3, "dgamma_p, dbeta_p %d" % (l + 1))
    ex = close_enough(eng.lsam_get_params(i), ora.get_params(0), 1e-5, "x after one step")
    print("%s, batch %d: worst weight-gradient error %.2e, parameters %.2e" % (name, batch, worst, ex))
    assert eng.lsam_sync() == 0
    eng.close()
