"""Workload table and seeded synthetic input generators.

This module holds data only: hyper-parameter tables for the five workloads and
seeded numpy generators for initial parameters, input batches, labels and raw
gradient vectors.  It contains none of the method's arithmetic (no model, no
schedule generator, no rounding rules), so both the CPU oracle's tests and the
GPU path's tests/benchmarks can draw identical inputs from it without sharing
any computation.

The shapes mirror the paper's image-classification set-up (Experiments,
"Experiment Setup": n = 4 workers, per-worker batch 128; CIFAR-shaped
3x32x32 = 3072-dim inputs, 10/100 classes), with dense MLPs standing in for
the paper's convolutional models, plus a small convolutional classifier on
32x32x3 inputs (the paper's SVHN model is a five-layer convolutional network
whose layers it does not list).
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Optional, Tuple

import numpy as np

SCHED_FIXED = 0   # periods drawn once at start
SCHED_REDRAW = 1  # a replica's period is redrawn at each of its syncs


@dataclass(frozen=True)
class Workload:
    name: str
    K: int                                  # replicas (the paper's n workers)
    dims: Tuple[int, ...] = ()              # in_0, out_1, ..., out_L; () => raw-vector mode
    d_raw: int = 0                          # parameters per replica in raw-vector mode
    batch: int = 0                          # B per replica
    gemm_dtype: int = 0                     # 0 = fp32, 1 = bf16 operands / fp32 accumulate
    rho: float = 0.05
    gamma: float = 1e-12
    lr: float = 0.1
    lr_center: float = 1.0
    momentum: float = 0.9
    beta: float = 0.9
    lambda0: float = 0.5
    lambda_abs: float = -1.0                # >= 0 overrides lambda0/(lr*tau)
    nesterov: int = 1
    tau: Optional[Tuple[int, ...]] = None   # explicit periods, else drawn
    tau_min: int = 1
    tau_max: int = 1
    sched_seed: int = 0
    sched_mode: int = SCHED_FIXED
    algorithm: int = 0                      # 0 = LSAM, 1 = synchronous data-parallel baseline
    noise_scale: float = 0.0                # sigma of the Langevin sampler, 0 = noise-free
    noise_seed: int = 0
    n_conv: int = 0                         # leading 3x3 convolution layers (0: dense model);
    img_h: int = 0                          # then dims = (C_0..C_n_conv, F_1.., classes) and the
    img_w: int = 0                          # input is [K, B, img_h, img_w, C_0]
    pool_mask: int = 0                      # bit l: 2x2 max-pool after convolution l
    bn_mask: int = 0                        # bit l: batch normalisation in convolution l
    bn_eps: float = 1e-5
    stride_mask: int = 0                    # bit l: convolution l has stride 2
    skip_mask: int = 0                      # bit l: the input of convolution l-1 is added to the
                                            # output of convolution l before its ReLU (basic block)
    proj_mask: int = 0                      # bit l (with skip_mask): that shortcut is a 1x1 convolution
                                            # with batch normalisation (projection), C_{l-1} -> C_{l+1}
    preact: int = 0                         # 1: pre-activation blocks (sums before the normalisations;
                                            # a projection is a bare 1x1 convolution of the rectified input)
    global_avg_pool: int = 0                # 1: the dense layers read the per-channel mean of the last image
    steps: int = 20
    data_seed: int = 0
    n_classes: int = field(default=0)
    grad_std: float = 1e-2                  # raw mode: std of the synthetic gradients
    batch_pool: int = 0                     # 0 => fresh batch each step, else pool size cycled

    @property
    def layer_shapes(self):
        """(fan_in, out) per layer: a 3x3 filter bank counts 9 C_in inputs, the first dense
        layer after the convolutions reads the whole (pooled) image."""
        h, w = self.img_h, self.img_w
        out = []
        for l in range(len(self.dims) - 1):
            fan_in = self.dims[l]
            if l < self.n_conv:
                fan_in = 9 * self.dims[l]
                if (self.stride_mask >> l) & 1:
                    h, w = h // 2, w // 2
                if (self.pool_mask >> l) & 1:
                    h, w = h // 2, w // 2
            elif self.n_conv and l == self.n_conv:
                fan_in = self.dims[l] if self.global_avg_pool else h * w * self.dims[l]
            out.append((fan_in, self.dims[l + 1]))
        return out

    @property
    def input_shape(self):
        return (self.img_h, self.img_w, self.dims[0]) if self.n_conv else (self.dims[0],)

    @property
    def d(self) -> int:
        if not self.dims:
            return self.d_raw
        return sum(fi * fo + fo + (2 * fo if (self.bn_mask >> l) & 1 and l < self.n_conv else 0) +
                   (fo * self.dims[l - 1] + (1 if self.preact else 3) * fo if (self.proj_mask >> l) & 1 else 0)
                   for l, (fi, fo) in enumerate(self.layer_shapes))

    def scaled(self, **kw) -> "Workload":
        return replace(self, **kw)


def _mlp(inp, width, hidden, classes):
    return (inp,) + (width,) * hidden + (classes,)


WORKLOADS = {
    # K=2, MLP 784-128-10 fp32, B=32, rho .05, lr .1, momentum .9, period 4, 20 steps
    "cfg1": Workload("cfg1", K=2, dims=(784, 128, 10), batch=32, rho=0.05,
                     tau=(4, 4), steps=20, data_seed=0, n_classes=10),
    # K=4, MLP 3072-1024-1024-10 fp32, B=128, periods from {2..8} seeded, 50 steps
    "cfg2": Workload("cfg2", K=4, dims=(3072, 1024, 1024, 10), batch=128, rho=0.05,
                     tau_min=2, tau_max=8, sched_seed=2, steps=50, data_seed=2,
                     n_classes=10),
    # K=8, 4 hidden layers of width 4096, 100 classes, bf16 operands, B=256
    "cfg3": Workload("cfg3", K=8, dims=_mlp(3072, 4096, 4, 100), batch=256, gemm_dtype=1,
                     rho=0.1, tau_min=2, tau_max=8, sched_seed=3, steps=20, data_seed=3,
                     n_classes=100, batch_pool=8),
    # update-only bandwidth path: K=8 x d=1e8 raw vectors, 100 iterations
    "cfg4": Workload("cfg4", K=8, d_raw=100_000_000, rho=0.05, tau_min=2, tau_max=8,
                     sched_seed=4, steps=100, data_seed=4),
    # K=16, 6 hidden layers of width 8192, 1000 classes, bf16 operands, B=512
    "cfg5": Workload("cfg5", K=16, dims=_mlp(3072, 8192, 6, 1000), batch=512, gemm_dtype=1,
                     rho=0.1, tau_min=4, tau_max=16, sched_seed=5, steps=20, data_seed=5,
                     n_classes=1000, batch_pool=4),
    # the paper's own set-up (Experiments, "Experiment Setup": n = 4 workers, batch 128 each,
    # communication interval 16, learning rate 0.02 for the small CNN, rho = 0.1) on
    # SVHN-shaped 32x32x3 inputs: three 3x3 convolutions, each followed by a 2x2 max-pool,
    # and two dense layers (five weight layers; the paper does not list its CNN-5's layers)
    "cnn5": Workload("cnn5", K=4, dims=(3, 32, 64, 128, 256, 10), batch=128, n_conv=3, img_h=32,
                     img_w=32, pool_mask=0b111, rho=0.1, lr=0.02, tau=(16, 16, 16, 16),
                     steps=20, data_seed=6, n_classes=10, batch_pool=4),
    # the same network with every convolution batch-normalised (the paper's deeper models
    # normalise every layer and keep the statistics per worker, Appendix "Batch Normalization")
    "cnn5bn": Workload("cnn5bn", K=4, dims=(3, 32, 64, 128, 256, 10), batch=128, n_conv=3, img_h=32,
                       img_w=32, pool_mask=0b111, bn_mask=0b111, rho=0.1, lr=0.02,
                       tau=(16, 16, 16, 16), steps=20, data_seed=7, n_classes=10, batch_pool=4),
    # VGG-16 as the paper trains it on CIFAR-10 (Experiments: VGG-16, 4 workers, batch 128,
    # learning rate 0.2): thirteen 3x3 convolutions in five groups, each group closed by a 2x2
    # max-pool, every convolution batch-normalised, then dense 512-512-512-10 (sixteen weight
    # layers).  The paper does not say which VGG-16 variant it uses; this is the usual CIFAR one.
    "vgg16": Workload("vgg16", K=4, dims=(3, 64, 64, 128, 128, 256, 256, 256, 512, 512, 512, 512,
                                          512, 512, 512, 512, 10),
                      batch=128, n_conv=13, img_h=32, img_w=32,
                      pool_mask=(1 << 1) | (1 << 3) | (1 << 6) | (1 << 9) | (1 << 12),
                      bn_mask=(1 << 13) - 1, rho=0.1, lr=0.2, tau=(16, 16, 16, 16), steps=20,
                      data_seed=8, n_classes=10, batch_pool=2),
}
# ResNet-20 as the paper trains it on CIFAR-10 (Experiments: ResNet-20, 4 workers, batch 128,
# learning rate 0.2, rho 0.1, communication interval 16), in the CIFAR form of He et al.: a 3x3
# stem of 16 channels, three stages of three basic blocks (two batch-normalised 3x3 convolutions
# each) with 16, 32 and 64 channels, the first convolution of stages two and three with stride 2,
# parameter-free shortcuts, global average pooling and one dense layer (twenty weight layers,
# 0.27 M parameters).
WORKLOADS["resnet20"] = Workload(
    "resnet20", K=4, dims=(3, 16) + (16,) * 6 + (32,) * 6 + (64,) * 6 + (10,), batch=128, n_conv=19,
    img_h=32, img_w=32, bn_mask=(1 << 19) - 1, stride_mask=(1 << 7) | (1 << 13),
    skip_mask=sum(1 << l for l in range(2, 19, 2)), global_avg_pool=1, rho=0.1, lr=0.2,
    tau=(16, 16, 16, 16), steps=20, data_seed=10, n_classes=10, batch_pool=2)


def _basic_block_net(name, blocks, widths, classes, **kw):
    """A 3x3 stem of widths[0] channels, then stage s of blocks[s] basic blocks at widths[s]
    channels; the first block of every stage but the first halves the image and changes the
    channel count through a projection shortcut.  Every convolution batch-normalised, global
    average pooling, one dense layer."""
    dims, stride, skip, proj = [3, widths[0]], 0, 0, 0
    l = 1
    for s, (n, c) in enumerate(zip(blocks, widths)):
        for b in range(n):
            if s > 0 and b == 0:
                stride |= 1 << l
                proj |= 1 << (l + 1)
            skip |= 1 << (l + 1)
            dims += [c, c]
            l += 2
    return Workload(name, K=4, dims=tuple(dims) + (classes,), batch=128, n_conv=l, img_h=32, img_w=32,
                    bn_mask=(1 << l) - 1, stride_mask=stride, skip_mask=skip, proj_mask=proj,
                    global_avg_pool=1, rho=0.1, lr=0.2, tau=(16, 16, 16, 16), steps=20, n_classes=classes,
                    batch_pool=2, **kw)


# ResNet-18 (Experiments: SVHN) and ResNet-34 (CIFAR-100) of He et al., four stages of 64, 128,
# 256 and 512 channels with (2, 2, 2, 2) resp. (3, 4, 6, 3) basic blocks and projection
# shortcuts where a stage begins; on 32x32 images the stem is one 3x3 convolution without the
# ImageNet models' 7x7 stride-2 convolution and max-pool (the usual form for images of this
# size; the paper does not say which it uses).  4 workers, batch 128, communication interval 16,
# learning rate 0.2 and rho 0.1 (Appendix "Hyperparameter Selection").
WORKLOADS["resnet18"] = _basic_block_net("resnet18", (2, 2, 2, 2), (64, 128, 256, 512), 10, data_seed=12)
WORKLOADS["resnet34"] = _basic_block_net("resnet34", (3, 4, 6, 3), (64, 128, 256, 512), 100, data_seed=13)


def _wide_resnet(name, depth, k, classes, **kw):
    """WRN-depth x k of Zagoruyko and Komodakis: a 3x3 stem of 16 channels, three stages of
    (depth - 4) / 6 pre-activation basic blocks with 16 k, 32 k and 64 k channels, stages two and
    three starting with stride 2; a 1x1 convolution as the shortcut where a block changes
    shape (the first block of every stage); normalisation, ReLU, global average pooling and
    one dense layer at the end.  No dropout."""
    n = (depth - 4) // 6
    dims, stride, skip, proj = [3, 16], 0, 0, 0
    l = 1
    for s, c in enumerate((16 * k, 32 * k, 64 * k)):
        for b in range(n):
            if b == 0:
                proj |= 1 << (l + 1)
                if s > 0:
                    stride |= 1 << l
            skip |= 1 << (l + 1)
            dims += [c, c]
            l += 2
    return Workload(name, K=4, dims=tuple(dims) + (classes,), batch=128, n_conv=l, img_h=32, img_w=32,
                    bn_mask=(1 << l) - 1, stride_mask=stride, skip_mask=skip, proj_mask=proj, preact=1,
                    global_avg_pool=1, rho=0.1, lr=0.2, tau=(16, 16, 16, 16), steps=20, n_classes=classes,
                    batch_pool=2, **kw)


# The wide residual networks of the Experiments section: WRN-16x10 (CIFAR-10), WRN-28x10 and
# WRN-40x10 (CIFAR-100); 4 workers, batch 128, communication interval 16, learning rate 0.2, rho 0.1.
WORKLOADS["wrn16x10"] = _wide_resnet("wrn16x10", 16, 10, 10, data_seed=14)
WORKLOADS["wrn28x10"] = _wide_resnet("wrn28x10", 28, 10, 100, data_seed=15)
WORKLOADS["wrn40x10"] = _wide_resnet("wrn40x10", 40, 10, 100, data_seed=16)
# the same model with bf16 matrix products (tensors stay fp32; see the boundary's gemm_dtype)
WORKLOADS["vgg16bf"] = replace(WORKLOADS["vgg16"], name="vgg16bf", gemm_dtype=1)
WORKLOADS["resnet18bf"] = replace(WORKLOADS["resnet18"], name="resnet18bf", gemm_dtype=1)
WORKLOADS["wrn16x10bf"] = replace(WORKLOADS["wrn16x10"], name="wrn16x10bf", gemm_dtype=1)


def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.default_rng([int(seed), int(stream)])


def init_params(w: Workload, seed: Optional[int] = None) -> np.ndarray:
    """One flat fp32 parameter vector [d]: per layer W [out,in] row-major then b [out],
    each drawn U(-1/sqrt(in), 1/sqrt(in)), then gamma ~ U(0.9, 1.1) and beta ~ U(-0.1, 0.1) for a
    batch-normalised layer, then W_p, b_p, gamma_p, beta_p of a projection shortcut drawn the
    same way (fan-in C_{l-1}); raw mode: N(0,1)."""
    rng = _rng(w.data_seed if seed is None else seed, 1)
    if not w.dims:
        return rng.standard_normal(w.d_raw, dtype=np.float32)
    parts = []
    for l, (fan_in, out) in enumerate(w.layer_shapes):
        bound = np.float32(1.0 / np.sqrt(fan_in))
        parts.append((rng.random(out * fan_in, dtype=np.float32) * 2 - 1) * bound)
        parts.append((rng.random(out, dtype=np.float32) * 2 - 1) * bound)
        if l < w.n_conv and (w.bn_mask >> l) & 1:
            # gamma around 1, beta around 0 (not exactly, so that tests see both)
            parts.append(1 + (rng.random(out, dtype=np.float32) - np.float32(0.5)) * np.float32(0.2))
            parts.append((rng.random(out, dtype=np.float32) - np.float32(0.5)) * np.float32(0.2))
        if (w.proj_mask >> l) & 1:
            cs = w.dims[l - 1]
            bound = np.float32(1.0 / np.sqrt(cs))
            parts.append((rng.random(out * cs, dtype=np.float32) * 2 - 1) * bound)
            parts.append((rng.random(out, dtype=np.float32) * 2 - 1) * bound)
            if not w.preact:
                parts.append(1 + (rng.random(out, dtype=np.float32) - np.float32(0.5)) * np.float32(0.2))
                parts.append((rng.random(out, dtype=np.float32) - np.float32(0.5)) * np.float32(0.2))
    return np.concatenate(parts).astype(np.float32)


def init_params_margin(w: Workload, seed: Optional[int] = None, ratio: float = 8.0) -> np.ndarray:
    """Like init_params, but every hidden unit is pushed away from the ReLU kink: hidden
    unit j of a layer of width n gets bias +c (j even) or -c (j odd) with c = 2/sqrt(n), and
    the weights feeding hidden units are scaled down so that the data-dependent part of
    every hidden pre-activation has a standard deviation near c/ratio.  The activation vectors
    keep a norm of order one, so training stays as stable as from init_params.
    Used where a comparison must not depend on which side of zero a rounded value falls."""
    p = init_params(w, seed).copy()
    off = 0
    L = len(w.dims) - 1
    c_prev = None
    for l, (fan_in, out) in enumerate(w.layer_shapes):
        if l < L - 1:
            c = 2.0 / np.sqrt(out)
            natural_std = 0.577 if l == 0 else 0.408 * c_prev
            p[off:off + out * fan_in] *= np.float32((c / ratio) / natural_std)
            p[off + out * fan_in: off + out * fan_in + out] = np.where(
                np.arange(out) % 2 == 0, c, -c).astype(np.float32)
            c_prev = c
        off += out * fan_in + out
        if l < w.n_conv and (w.bn_mask >> l) & 1:
            off += 2 * out
        if (w.proj_mask >> l) & 1:
            off += out * w.dims[l - 1] + (1 if w.preact else 3) * out
    return p


def batch(w: Workload, step: int):
    """Inputs X [K,B,in_0] (convolutional workloads: [K,B,H,W,C_0]) fp32 ~ N(0,1) and labels
    [K,B] int32 uniform over the classes
    for tick `step` (a pool index when the workload cycles a fixed pool).  For bf16
    workloads the low 16 mantissa bits are cleared so every value is exactly
    representable in bf16 and no rounding rule enters the data."""
    idx = step % w.batch_pool if w.batch_pool else step
    rng = _rng(w.data_seed, 1000 + idx)
    X = rng.standard_normal((w.K, w.batch) + w.input_shape, dtype=np.float32)
    if w.gemm_dtype == 1:
        X = (X.view(np.uint32) & np.uint32(0xFFFF0000)).view(np.float32)
    labels = rng.integers(0, w.n_classes, size=(w.K, w.batch), dtype=np.int32)
    return X, labels


def raw_grads(w: Workload, step: int, d: Optional[int] = None):
    """Raw-vector mode: two gradient sets g1, g2 [K,d] fp32 ~ N(0, grad_std^2)."""
    d = w.d_raw if d is None else d
    rng = _rng(w.data_seed, 5000 + step)
    g1 = rng.standard_normal((w.K, d), dtype=np.float32) * np.float32(w.grad_std)
    g2 = rng.standard_normal((w.K, d), dtype=np.float32) * np.float32(w.grad_std)
    return g1, g2
