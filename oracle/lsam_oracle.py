"""Plain CPU oracle of the K-replica LSAM step.  TEST INFRASTRUCTURE ONLY.

This file is the correctness reference the HIP path is compared against.  It is
imported only by the tests, the smoke check and the benchmark's CPU-baseline
leg; the product path never calls it and shares no code with it.

Everything is float64 numpy, one replica after another, no blocking, fusion or
reordering beyond what the paper's formulas state.  `numpy.matmul` is the only
library primitive used as a step (the dense layers, and the nine taps of a
3x3 convolution, each a matrix product over the channels).

What follows the paper, by passage:
  * loss f(x; xi): empirical mean over the minibatch (Introduction, problem
    statement).
  * first-order SAM point  x~ = x + rho * grad f(x) / (||grad f(x)|| + gamma)
    (Formulation, definition of f_SAM; Appendix, look-back map T_{rho,gamma}).
  * SAM gradient g_t = grad f(x~; xi_t), same minibatch in both passes, no
    Jacobian of the map (Theorem "Convergence of G_t with Constant
    Perturbation", definition of g_t).
  * local update  x <- x - eta (g_t + lambda (x - y))  (Algorithm 1, x-update),
    driven through a Nesterov-momentum sampler (Section "Distributed Training").
  * center direction g' = (1/(n tau)) sum_i sum_s x_s^(i) - y, look-ahead
    g = g' + beta (g' - g'_prev), y <- Optimizer(y, g, eta'), counters reset
    (Algorithm 2, synchronous optimization step; Section "Acceleration
    Techniques for Optimization").
  * lambda = lambda0 / (eta tau) (Appendix "Hyperparameter Search").

Readings where the paper is silent (each also listed in the design notes):
  gamma default 1e-12; y <- y + eta' g (ascent on the log-density score, which
  makes beta = 0, eta' = 1 give the plain mean of the samples and agrees with
  Algorithm 1's y-update); no look-ahead term at the first sync; Nesterov form
  v <- mu v + G, x <- x - eta (G + mu v); per-replica trigger c_i >= tau_i with
  the mean taken over the due replicas' samples (equals Algorithm 2 when all
  periods are equal); the iterate sum S_i collects post-update iterates;
  ReLU'(0) = 0; reported loss is the first-pass loss.

Parity status: the paper prints no iterate, loss value or worked example, so
agreement with the authors' own implementation is "parity unpinned".  Every
function here is pinned instead by finite differences, closed forms, reduction
to Algorithm 1 / Algorithm 2 special cases, brute-force bookkeeping and an
autograd/`torch.optim.SGD` witness in tests/test_oracle_pins.py (the
convolutional model: torch's own convolution and pooling routines under
autograd, finite differences, and hand-worked impulse and tie cases).
"""
from __future__ import annotations

import numpy as np

SCHED_FIXED = 0
SCHED_REDRAW = 1

_LCG_A = 6364136223846793005
_LCG_C = 1442695040888963407
_MASK64 = (1 << 64) - 1


class PeriodSchedule:
    """Seeded per-replica communication periods (integer only).

    State s_0 = seed; s_{j+1} = (A s_j + C) mod 2^64; draw_j = (s_{j+1} >> 33)
    mod (tau_max - tau_min + 1) + tau_min.  The first K draws give tau_0..tau_{K-1};
    in redraw mode every replica that syncs takes the next draw, lower index first.
    """

    def __init__(self, K, tau=None, tau_min=1, tau_max=1, seed=0, mode=SCHED_FIXED):
        self.K = int(K)
        self.tau_min, self.tau_max = int(tau_min), int(tau_max)
        self.mode = int(mode)
        self.state = int(seed) & _MASK64
        if tau is not None:
            self.tau = [int(t) for t in tau]
            self.explicit = True
        else:
            self.explicit = False
            self.tau = [self.draw() for _ in range(self.K)]
        if len(self.tau) != self.K or min(self.tau) < 1:
            raise ValueError("need K periods >= 1")
        self.count = [0] * self.K   # c_i: local iterations since replica i last synced
        self.t_y = 0                # number of center updates so far

    def draw(self):
        self.state = (_LCG_A * self.state + _LCG_C) & _MASK64
        return (self.state >> 33) % (self.tau_max - self.tau_min + 1) + self.tau_min

    def tick(self):
        for i in range(self.K):
            self.count[i] += 1

    def due(self):
        return [i for i in range(self.K) if self.count[i] >= self.tau[i]]

    def served(self, due):
        for i in due:
            self.count[i] = 0
            if self.mode == SCHED_REDRAW and not self.explicit:
                self.tau[i] = self.draw()
        self.t_y += 1


def bf16_round(a):
    """Round-to-nearest-even to bfloat16, taken from the float32 value (the precision
    the rounded tensors have on the device), returned as float64."""
    f = np.ascontiguousarray(a, dtype=np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).astype(np.float64).reshape(np.shape(a))


def _identity(a):
    return np.asarray(a, dtype=np.float64)


class Mlp:
    """Dense ReLU classifier on a flat parameter vector: per layer W_l [out,in]
    row-major then b_l [out]; Z_l = A_{l-1} W_l^T + b_l, A_l = ReLU(Z_l) for l < L,
    logits = Z_L; loss = mean_b [logsumexp(logits_b) - logits_b[label_b]]."""

    def __init__(self, dims, gemm_dtype=0):
        self.dims = tuple(int(v) for v in dims)
        self.L = len(self.dims) - 1
        self.q = bf16_round if gemm_dtype == 1 else _identity
        self.offsets = []
        off = 0
        for l in range(self.L):
            fi, fo = self.dims[l], self.dims[l + 1]
            self.offsets.append((off, off + fo * fi, off + fo * fi + fo))
            off += fo * fi + fo
        self.d = off
        self.last_margin = np.inf   # diagnostic: smallest |hidden pre-activation| seen last call
        # diagnostic, filled when keep_hidden is set: per hidden layer (Z, |A||W|^T + |b|) of the
        # last call -- the pre-activations and the magnitude their rounding error scales with
        self.keep_hidden = False
        self.last_hidden = []

    def unpack(self, x):
        out = []
        for l, (o0, o1, o2) in enumerate(self.offsets):
            out.append((x[o0:o1].reshape(self.dims[l + 1], self.dims[l]), x[o1:o2]))
        return out

    def loss_and_grad(self, x, X, labels):
        """Returns (loss, grad [d]).  With bf16 operands, exactly the tensors fed to the
        matrix units are rounded: W, the input X, hidden activations and every dZ (the
        bias gradient sums the same rounded dZ); all accumulation, the softmax and the
        results stay in float64."""
        q = self.q
        layers = self.unpack(np.asarray(x, dtype=np.float64))
        B = X.shape[0]
        acts = [q(X)]
        self.last_margin = np.inf
        self.last_hidden = []
        for l, (W, b) in enumerate(layers):
            Z = acts[l] @ q(W).T + b
            if l < self.L - 1:
                self.last_margin = min(self.last_margin, float(np.min(np.abs(Z))))
                if self.keep_hidden:
                    self.last_hidden.append((Z, np.abs(acts[l]) @ np.abs(q(W)).T + np.abs(b)))
            acts.append(q(np.maximum(Z, 0.0)) if l < self.L - 1 else Z)
        logits = acts[-1]
        zmax = logits.max(axis=1, keepdims=True)
        e = np.exp(logits - zmax)
        se = e.sum(axis=1, keepdims=True)
        lse = np.log(se) + zmax
        rows = np.arange(B)
        loss = float(np.mean(lse[:, 0] - logits[rows, labels]))
        dZ = e / se
        dZ[rows, labels] -= 1.0
        dZ /= B
        grad = np.zeros(self.d)
        for l in range(self.L - 1, -1, -1):
            W, _ = layers[l]
            o0, o1, o2 = self.offsets[l]
            dZq = q(dZ)
            grad[o0:o1] = (dZq.T @ acts[l]).ravel()
            grad[o1:o2] = dZq.sum(axis=0)
            if l > 0:
                dA = dZq @ q(W)
                dZ = dA * (acts[l] > 0.0)
        return loss, grad


def conv_layer_shapes(dims, n_conv, img_h, img_w, pool_mask, stride_mask=0, global_avg_pool=0):
    """(fan_in, out) of every layer of the convolutional model described at `Cnn`, plus the
    image size after the convolution stack."""
    h, w = int(img_h), int(img_w)
    shapes = []
    for l in range(len(dims) - 1):
        if l < n_conv:
            shapes.append((9 * dims[l], dims[l + 1]))
            if (stride_mask >> l) & 1:
                if h % 2 or w % 2:
                    raise ValueError("a stride-2 convolution needs even image sides")
                h, w = h // 2, w // 2
            if (pool_mask >> l) & 1:
                if h % 2 or w % 2:
                    raise ValueError("2x2 pooling needs even image sides")
                h, w = h // 2, w // 2
        elif l == n_conv:
            shapes.append(((1 if global_avg_pool else h * w) * dims[l], dims[l + 1]))
        else:
            shapes.append((dims[l], dims[l + 1]))
    return shapes, (h, w)


class Cnn:
    """Small convolutional ReLU classifier (the paper's experiments train convolutional
    networks on 32x32x3 images; Section "Experiments" names a five-layer one without giving
    its layers, so the shape is a parameter here).

    Layers l < n_conv: 3x3 convolution, stride 1, zero padding 1, C_l -> C_{l+1} channels,
    bias, [batch normalisation if bit l of bn_mask is set,] ReLU, then a 2x2/stride-2 max-pool
    if bit l of pool_mask is set.  The remaining
    layers are dense as in `Mlp`, the first of them reading the image flattened in (row,
    column, channel) order.  dims = (C_0, ..., C_{n_conv}, F_1, ..., classes).
    Tensors are [B, H, W, C].  Flat parameters per layer: W_l [out, 3, 3, C_l] (dense:
    [out, in]) row-major, then b_l [out], then, for a batch-normalised layer, gamma_l [out] and
    beta_l [out].

    Batch normalisation is the training-mode one (Appendix "Batch Normalization": every worker
    normalises with the statistics of its own minibatch, nothing is synchronised): per channel,
    over the B H W positions of the replica's batch,
      mu = mean Z, var = mean (Z - mu)^2, Xh = (Z - mu) / sqrt(var + eps), Y = gamma Xh + beta,
    and its backward pass carries the dependence of mu and var on Z:
      dbeta = sum dY, dgamma = sum dY Xh, dZ = gamma / sqrt(var + eps) (dY - dbeta/N - Xh dgamma/N).
    Running averages for inference are not part of a training step and are not kept.

    Residual networks (the ResNet models of Section "Experiments"; He et al., "Deep Residual
    Learning for Image Recognition", CIFAR variant): bit l of stride_mask gives convolution l
    stride 2 (output [H/2, W/2]); bit l of skip_mask closes a basic block of the two
    convolutions l-1 and l: the block's input, i.e. the image convolution l-1 read, is added
    to the (normalised) output of convolution l before its ReLU.  Where the two differ in shape
    the shortcut is that paper's parameter-free one: every second pixel of the block input in
    both directions, channels padded with zeros.  Bit l of proj_mask (with bit l of skip_mask)
    replaces that shortcut by that paper's projection: a 1x1 convolution of the block input with
    the block's stride, C_{l-1} -> C_{l+1} channels, with bias and its own batch normalisation
    (no ReLU); its parameters W_p [C_{l+1}, C_{l-1}], b_p, gamma_p, beta_p follow those of
    convolution l in the flat vector.  global_avg_pool: the dense layers read the
    mean of the last image over its positions, one value per channel.

    preact = 1 gives the pre-activation blocks of wide residual networks (Zagoruyko and
    Komodakis, "Wide Residual Networks"; the Experiments section trains WRN-16/28/40 x 10): the
    sum of a block is taken on the convolutions' outputs before any normalisation, and the
    normalisation and ReLU of convolution l act on that sum, u_l = conv_l(a_{l-1}) + b_l
    [+ shortcut], a_l = relu(bn_l(u_l)).  The shortcut of a block closed by convolution l is
    u_{l-2}, the sum two convolutions below (shapes must agree), or, with bit l of proj_mask, a
    1x1 convolution (block stride, bias, no normalisation) of a_{l-2}, the normalised and
    rectified block input, as that paper's networks use where a block changes shape; its
    parameters are W_p [C_{l+1}, C_{l-1}] and b_p only.  Read this way the network's first
    normalisation is the stem's, each block's two normalisations are those of the convolution
    below its first and of its first convolution, and the last convolution's is the one in
    front of the pooling.

      Z[b,i,j,o] = b[o] + sum_{u,v,c} Xpad[b,s i+u,s j+v,c] W[o,u,v,c]     (Xpad: X with a zero rim, s: stride)
      P[b,i,j,c] = max_{u,v in {0,1}} A[b,2i+u,2j+v,c]
    The pool's gradient goes to the first maximal element of each window in (u, v) order."""

    def __init__(self, dims, n_conv, img_h, img_w, pool_mask, bn_mask=0, bn_eps=1e-5, gemm_dtype=0,
                 stride_mask=0, skip_mask=0, global_avg_pool=0, proj_mask=0, preact=0):
        self.preact = int(preact)
        self.bn_mask, self.bn_eps = int(bn_mask), float(bn_eps)
        self.stride_mask, self.skip_mask = int(stride_mask), int(skip_mask)
        self.proj_mask = int(proj_mask)
        if self.proj_mask & ~self.skip_mask:
            raise ValueError("a projection belongs to a shortcut")
        self.gap = int(global_avg_pool)
        if self.skip_mask & 0b11:
            raise ValueError("a block needs two convolutions below its closing one")
        # gemm_dtype 1: every matrix product (each tap of a convolution, each dense layer, and
        # their dW and dX) takes its two operands rounded to bfloat16 and accumulates exactly;
        # everything stored -- activations, gradients, biases, normalisation -- stays unrounded
        # (the bias gradients therefore sum the unrounded dZ)
        self.q = bf16_round if gemm_dtype == 1 else _identity
        self.dims = tuple(int(v) for v in dims)
        self.L = len(self.dims) - 1
        self.n_conv = int(n_conv)
        self.H, self.W = int(img_h), int(img_w)
        self.pool_mask = int(pool_mask)
        self.shapes, self.final_hw = conv_layer_shapes(self.dims, self.n_conv, self.H, self.W,
                                                       self.pool_mask, self.stride_mask, self.gap)
        self.offsets = []
        self.bn_offsets = {}        # layer -> (start of gamma, start of beta, end)
        self.proj_offsets = {}      # layer -> (start of W_p, of b_p, of gamma_p, of beta_p, end)
        off = 0
        for l, (fi, fo) in enumerate(self.shapes):
            self.offsets.append((off, off + fo * fi, off + fo * fi + fo))
            off += fo * fi + fo
            if l < self.n_conv and (self.bn_mask >> l) & 1:
                self.bn_offsets[l] = (off, off + fo, off + 2 * fo)
                off += 2 * fo
            if l < self.n_conv and (self.proj_mask >> l) & 1:
                cs = self.dims[l - 1]
                nb = 0 if self.preact else fo        # a pre-activation projection has no normalisation
                self.proj_offsets[l] = (off, off + fo * cs, off + fo * cs + fo, off + fo * cs + fo + nb,
                                        off + fo * cs + fo + 2 * nb)
                off += fo * cs + fo + 2 * nb
        self.d = off
        self.last_margin = np.inf

    @staticmethod
    def _shortcut(src, shape):
        """The block input `src` [B, H, W, C] brought to `shape` [B, H', W', C']: every second
        pixel when the block halved the image, zero channels appended when it widened it."""
        s = src
        if s.shape[1] != shape[1]:
            s = s[:, ::2, ::2, :]
        if s.shape[1:3] != tuple(shape[1:3]) or s.shape[3] > shape[3]:
            raise ValueError("shortcut and block output do not fit")
        out = np.zeros(shape)
        out[..., :s.shape[3]] = s
        return out

    @staticmethod
    def _shortcut_adjoint(g, shape):
        """Adjoint of `_shortcut`: the gradient of the block output `g`, sent back to the shape
        of the block input."""
        out = np.zeros(shape)
        part = g[..., :shape[3]]
        if shape[1] != g.shape[1]:
            out[:, ::2, ::2, :] = part
        else:
            out[...] = part
        return out

    def loss_and_grad(self, x, X, labels):
        x = np.asarray(x, dtype=np.float64)
        X = np.asarray(X, dtype=np.float64)
        q = self.q
        bn_saved = {}
        proj_saved = {}
        B = X.shape[0]
        self.last_margin = np.inf
        # ---- forward ----
        conv_in, conv_act, pooled_from, conv_src, raw = [], [], [], [], []
        A = X
        for l in range(self.n_conv):
            o0, o1, o2 = self.offsets[l]
            cin, cout = self.dims[l], self.dims[l + 1]
            st = 2 if (self.stride_mask >> l) & 1 else 1
            Wl = x[o0:o1].reshape(cout, 3, 3, cin)
            hin, win = A.shape[1], A.shape[2]
            h, w = hin // st, win // st
            Ap = np.zeros((B, hin + 2, win + 2, cin))
            Ap[:, 1:hin + 1, 1:win + 1, :] = A
            Z = np.zeros((B, h, w, cout)) + x[o1:o2]
            Apq, Wq = q(Ap), q(Wl)
            for u in range(3):
                for v in range(3):
                    Z += Apq[:, u:u + st * h:st, v:v + st * w:st, :] @ Wq[:, u, v, :].T
            if self.preact and (self.skip_mask >> l) & 1:
                if l in self.proj_offsets:
                    p0, p1, p2, _, _ = self.proj_offsets[l]
                    S = conv_src[l - 1]
                    if S.shape[1] != h:
                        S = S[:, ::2, ::2, :]
                    proj_saved[l] = (S,)
                    Z = Z + q(S) @ q(x[p0:p1].reshape(cout, S.shape[3])).T + x[p1:p2]
                else:
                    if raw[l - 2].shape != Z.shape:
                        raise ValueError("shortcut and block output do not fit")
                    Z = Z + raw[l - 2]
            raw.append(Z)
            if l in self.bn_offsets:
                g0, g1, g2 = self.bn_offsets[l]
                mu = Z.mean(axis=(0, 1, 2))
                var = ((Z - mu) ** 2).mean(axis=(0, 1, 2))
                inv = 1.0 / np.sqrt(var + self.bn_eps)
                Xh = (Z - mu) * inv
                bn_saved[l] = (Xh, inv)
                Z = x[g0:g1] * Xh + x[g1:g2]
            if self.preact:
                pass
            elif l in self.proj_offsets:
                p0, p1, p2, p3, p4 = self.proj_offsets[l]
                S = conv_src[l - 1]
                if S.shape[1] != h:
                    S = S[:, ::2, ::2, :]
                Wp = x[p0:p1].reshape(cout, S.shape[3])
                Zp = q(S) @ q(Wp).T + x[p1:p2]
                mup = Zp.mean(axis=(0, 1, 2))
                invp = 1.0 / np.sqrt(((Zp - mup) ** 2).mean(axis=(0, 1, 2)) + self.bn_eps)
                Xhp = (Zp - mup) * invp
                proj_saved[l] = (S, Xhp, invp)
                Z = Z + x[p2:p3] * Xhp + x[p3:p4]
            elif (self.skip_mask >> l) & 1:
                Z = Z + self._shortcut(conv_src[l - 1], Z.shape)
            self.last_margin = min(self.last_margin, float(np.min(np.abs(Z))))
            R = np.maximum(Z, 0.0)
            conv_src.append(A)
            conv_in.append(Ap)
            conv_act.append(R)
            if (self.pool_mask >> l) & 1:
                win_ = R.reshape(B, h // 2, 2, w // 2, 2, cout).transpose(0, 1, 3, 5, 2, 4)
                win_ = win_.reshape(B, h // 2, w // 2, cout, 4)     # window order (u, v)
                pooled_from.append(np.argmax(win_, axis=-1))         # first maximum
                A = win_.max(axis=-1)
            else:
                pooled_from.append(None)
                A = R
        final_image = A
        if self.gap:
            A = A.mean(axis=(1, 2))
        acts = [A.reshape(B, -1)]
        for l in range(self.n_conv, self.L):
            o0, o1, o2 = self.offsets[l]
            fi, fo = self.shapes[l]
            Z = q(acts[-1]) @ q(x[o0:o1].reshape(fo, fi)).T + x[o1:o2]
            if l < self.L - 1:
                self.last_margin = min(self.last_margin, float(np.min(np.abs(Z))))
                acts.append(np.maximum(Z, 0.0))
            else:
                acts.append(Z)
        logits = acts[-1]
        zmax = logits.max(axis=1, keepdims=True)
        e = np.exp(logits - zmax)
        se = e.sum(axis=1, keepdims=True)
        rows = np.arange(B)
        loss = float(np.mean((np.log(se) + zmax)[:, 0] - logits[rows, labels]))
        # ---- backward ----
        dZ = e / se
        dZ[rows, labels] -= 1.0
        dZ /= B
        grad = np.zeros(self.d)
        dA = None
        for l in range(self.L - 1, self.n_conv - 1, -1):
            o0, o1, o2 = self.offsets[l]
            fi, fo = self.shapes[l]
            a_in = acts[l - self.n_conv]
            grad[o0:o1] = (q(dZ).T @ q(a_in)).ravel()
            grad[o1:o2] = dZ.sum(axis=0)
            dA = q(dZ) @ q(x[o0:o1].reshape(fo, fi))
            if l > self.n_conv:
                dZ = dA * (a_in > 0.0)
        if self.gap and self.n_conv:
            bh, bw = final_image.shape[1], final_image.shape[2]
            dA = np.broadcast_to(dA[:, None, None, :] / (bh * bw), final_image.shape)
        skip_grad = {}       # layer whose input receives it -> gradient of the shortcut
        raw_grad = {}        # pre-activation blocks: layer whose sum u_l receives it -> gradient
        for l in range(self.n_conv - 1, -1, -1):
            o0, o1, o2 = self.offsets[l]
            cin, cout = self.dims[l], self.dims[l + 1]
            st = 2 if (self.stride_mask >> l) & 1 else 1
            R = conv_act[l]
            h, w = R.shape[1], R.shape[2]
            if pooled_from[l] is not None:
                dP = dA.reshape(B, h // 2, w // 2, cout)
                dwin = np.zeros((B, h // 2, w // 2, cout, 4))
                np.put_along_axis(dwin, pooled_from[l][..., None], dP[..., None], axis=-1)
                dR = dwin.reshape(B, h // 2, w // 2, cout, 2, 2).transpose(0, 1, 4, 2, 5, 3)
                dR = dR.reshape(B, h, w, cout)
            else:
                dR = dA.reshape(B, h, w, cout)
            dZc = dR * (R > 0.0)
            if self.preact:
                pass
            elif l in self.proj_offsets:
                # through the projection's normalisation and 1x1 convolution, back to the block input
                p0, p1, p2, p3, p4 = self.proj_offsets[l]
                S, Xhp, invp = proj_saved[l]
                n = B * h * w
                dbp = dZc.sum(axis=(0, 1, 2))
                dgp = (dZc * Xhp).sum(axis=(0, 1, 2))
                grad[p2:p3] = dgp
                grad[p3:p4] = dbp
                dZp = x[p2:p3] * invp * (dZc - dbp / n - Xhp * dgp / n)
                Wp = x[p0:p1].reshape(cout, S.shape[3])
                flatp = dZp.reshape(-1, cout)
                grad[p0:p1] = (q(flatp).T @ q(S.reshape(-1, S.shape[3]))).ravel()
                grad[p1:p2] = flatp.sum(axis=0)
                dS = q(dZp) @ q(Wp)
                full = np.zeros(conv_src[l - 1].shape)
                if full.shape[1] != h:
                    full[:, ::2, ::2, :] = dS
                else:
                    full[...] = dS
                skip_grad[l - 1] = ("full", full)
            elif (self.skip_mask >> l) & 1:
                skip_grad[l - 1] = ("out", dZc)   # the sum's gradient reaches both of its terms
            if l in self.bn_offsets:
                g0, g1, g2 = self.bn_offsets[l]
                Xh, inv = bn_saved[l]
                n = B * h * w
                dbeta = dZc.sum(axis=(0, 1, 2))
                dgamma = (dZc * Xh).sum(axis=(0, 1, 2))
                grad[g0:g1] = dgamma
                grad[g1:g2] = dbeta
                dZc = x[g0:g1] * inv * (dZc - dbeta / n - Xh * dgamma / n)
            if self.preact:
                # dZc is the gradient of the sum u_l: add what the block above sent down its
                # identity shortcut, then hand this block's own shortcut its share
                if l in raw_grad:
                    dZc = dZc + raw_grad.pop(l)
                if l in self.proj_offsets:
                    p0, p1, p2, _, _ = self.proj_offsets[l]
                    (S,) = proj_saved[l]
                    du = dZc.reshape(-1, cout)
                    grad[p0:p1] = (q(du).T @ q(S.reshape(-1, S.shape[3]))).ravel()
                    grad[p1:p2] = du.sum(axis=0)
                    dSu = q(dZc) @ q(x[p0:p1].reshape(cout, S.shape[3]))
                    spread = np.zeros(conv_src[l - 1].shape)
                    if spread.shape[1] != h:
                        spread[:, ::2, ::2, :] = dSu
                    else:
                        spread[...] = dSu
                    skip_grad[l - 1] = ("full", spread)
                elif (self.skip_mask >> l) & 1:
                    raw_grad[l - 2] = dZc
            Wl = x[o0:o1].reshape(cout, 3, 3, cin)
            Ap = conv_in[l]
            hin, win = Ap.shape[1] - 2, Ap.shape[2] - 2
            dW = np.zeros((cout, 3, 3, cin))
            dAp = np.zeros_like(Ap)
            flat = dZc.reshape(-1, cout)
            flatq, dZq, Apq, Wq = q(flat), q(dZc), q(Ap), q(Wl)
            for u in range(3):
                for v in range(3):
                    dW[:, u, v, :] = flatq.T @ Apq[:, u:u + st * h:st, v:v + st * w:st, :].reshape(-1, cin)
                    dAp[:, u:u + st * h:st, v:v + st * w:st, :] += dZq @ Wq[:, u, v, :]
            grad[o0:o1] = dW.ravel()
            grad[o1:o2] = flat.sum(axis=0)
            dA = dAp[:, 1:hin + 1, 1:win + 1, :]
            if l in skip_grad:
                kind, gsk = skip_grad.pop(l)
                dA = dA + (gsk if kind == "full" else self._shortcut_adjoint(gsk, dA.shape))
        return loss, grad


# ---- Langevin noise of the sampler ----------------------------------------------------------------
# Section "Langevin Dynamics for Sampling" names SGLD as the Sampler of Algorithm 2; the
# experiments run it noise-free.  With noise_scale = sigma > 0 the sampler step becomes
#   x <- x - eta (G + mu v) + sigma sqrt(2 eta) xi,   xi ~ N(0, I),
# the Euler-Maruyama step of dx = grad log q dt + sqrt(2) dW at sigma = 1, mu = 0.
# xi comes from the counter-based generator Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel
# random numbers: as easy as 1, 2, 3", SC'11), so that any element of any step can be produced
# on its own.  One call yields the four normals of four neighbouring columns:
#   counter = (column // 4, row, (8 * layer + piece) | replica << 16, step)     [MLP]
#             piece: 0 W, 1 b, 2 gamma, 3 beta, 4..7 the same of the layer's projection shortcut
#   counter = (j // 4 mod 2^32, j // 4 >> 32, replica << 16, step)               [raw vector]
#   key     = (seed mod 2^32, seed >> 32)
#   u_i = ((r_i >> 8) + 1/2) / 2^24;  z0, z1 = sqrt(-2 ln u0) (cos, sin)(2 pi u1);  z2, z3 from u2, u3
# (a bias vector counts as one row; `step` is the number of sampler steps taken before).
PHILOX_M0, PHILOX_M1 = 0xD2511F53, 0xCD9E8D57
PHILOX_W0, PHILOX_W1 = 0x9E3779B9, 0xBB67AE85


def philox4x32_10(counter, key):
    """counter: four arrays of 32-bit values, key: two 32-bit values -> four uint64 arrays
    holding the 32-bit outputs."""
    m32 = np.uint64(0xFFFFFFFF)
    c = [np.asarray(x, dtype=np.uint64) & m32 for x in np.broadcast_arrays(*counter)]
    k0, k1 = np.uint64(key[0]) & m32, np.uint64(key[1]) & m32
    for _ in range(10):
        p0 = np.uint64(PHILOX_M0) * c[0]
        p1 = np.uint64(PHILOX_M1) * c[2]
        c = [(p1 >> np.uint64(32)) ^ c[1] ^ k0, p1 & m32, (p0 >> np.uint64(32)) ^ c[3] ^ k1, p0 & m32]
        k0 = (k0 + np.uint64(PHILOX_W0)) & m32
        k1 = (k1 + np.uint64(PHILOX_W1)) & m32
    return c


def normals_from_counters(counter, key):
    """[..., 4] standard normals, one Philox call per leading index (Box-Muller)."""
    r = philox4x32_10(counter, key)
    u = [((x >> np.uint64(8)).astype(np.float64) + 0.5) / 16777216.0 for x in r]
    out = np.empty(u[0].shape + (4,))
    for pair in range(2):
        rad = np.sqrt(-2.0 * np.log(u[2 * pair]))
        ang = 2.0 * np.pi * u[2 * pair + 1]
        out[..., 2 * pair] = rad * np.cos(ang)
        out[..., 2 * pair + 1] = rad * np.sin(ang)
    return out


def langevin_noise(dims, d_raw, replica, step, seed, shapes=None, bn_mask=0, proj_mask=0, preact=0):
    """xi for one replica and step, in the flat parameter layout.  `shapes`: (fan_in, out) per
    layer when they are not the consecutive pairs of `dims` (convolutional layers: a filter
    bank [out, 3, 3, C] is the matrix [out, 9 C]).  The pieces of layer l carry the codes
    8 l + 0 (W), 1 (b), 2 (gamma), 3 (beta), 4..7 (the same four of its projection shortcut);
    vectors count as one-row matrices."""
    key = (seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)
    if not len(dims):
        groups = np.arange((d_raw + 3) // 4, dtype=np.uint64)
        z = normals_from_counters((groups & np.uint64(0xFFFFFFFF), groups >> np.uint64(32),
                                   np.uint64(replica << 16), np.uint64(step)), key)
        return z.reshape(-1)[:d_raw]
    parts = []
    if shapes is None:
        shapes = [(dims[l], dims[l + 1]) for l in range(len(dims) - 1)]
    for l, (fi, fo) in enumerate(shapes):
        pieces = [(8 * l, fo, fi), (8 * l + 1, 1, fo)]
        if (bn_mask >> l) & 1:
            pieces += [(8 * l + 2, 1, fo), (8 * l + 3, 1, fo)]
        if (proj_mask >> l) & 1:
            pieces += [(8 * l + 4, fo, dims[l - 1]), (8 * l + 5, 1, fo)]
            if not preact:
                pieces += [(8 * l + 6, 1, fo), (8 * l + 7, 1, fo)]
        for which, rows, cols in pieces:
            cg = np.arange((cols + 3) // 4, dtype=np.uint64)[None, :]
            rr = np.arange(rows, dtype=np.uint64)[:, None]
            code = np.uint64(which | (replica << 16))
            z = normals_from_counters((cg, rr, code, np.uint64(step)), key)
            parts.append(z.reshape(rows, -1)[:, :cols].ravel())
    return np.concatenate(parts)


# Which method the K replicas run.  ALG_LSAM is Algorithm 2.  ALG_DATA_PARALLEL is the
# synchronous baseline of the experiments section (DP-SAM; DP-SGD when rho = 0): every
# iteration the workers' gradients are averaged, at the first pass and again at the perturbed
# point, every replica takes the same momentum step on the averaged gradient, and there is
# neither coupling nor a center update (communication interval 1, nothing left to average).
ALG_LSAM = 0
ALG_DATA_PARALLEL = 1


class LsamOracle:
    """K replicas x_i, velocities v_i, iterate sums S_i, one center y."""

    def __init__(self, K, init_params, dims=(), d_raw=0, batch=0, gemm_dtype=0,
                 rho=0.05, gamma=1e-12, lr=0.1, lr_center=1.0, momentum=0.9, beta=0.9,
                 lambda0=0.5, lambda_abs=-1.0, nesterov=1, tau=None, tau_min=1, tau_max=1,
                 sched_seed=0, sched_mode=SCHED_FIXED, algorithm=ALG_LSAM, noise_scale=0.0,
                 noise_seed=0, n_conv=0, img_h=0, img_w=0, pool_mask=0, bn_mask=0, bn_eps=1e-5,
                 stride_mask=0, skip_mask=0, global_avg_pool=0, proj_mask=0, preact=0):
        self.K = int(K)
        self.algorithm = int(algorithm)
        self.noise_scale, self.noise_seed = float(noise_scale), int(noise_seed)
        self.dims = tuple(dims)
        self.t = 0                      # sampler steps taken so far
        if n_conv:
            self.model = Cnn(dims, n_conv, img_h, img_w, pool_mask, bn_mask, bn_eps, gemm_dtype,
                             stride_mask, skip_mask, global_avg_pool, proj_mask, preact)
        else:
            self.model = Mlp(dims, gemm_dtype) if len(dims) else None
        self.shapes = self.model.shapes if n_conv else None
        self.bn_mask = int(bn_mask) if n_conv else 0
        self.proj_mask = int(proj_mask) if n_conv else 0
        self.preact = int(preact) if n_conv else 0
        self.d = self.model.d if self.model else int(d_raw)
        self.batch = int(batch)
        self.rho, self.gamma = float(rho), float(gamma)
        self.lr, self.lr_center = float(lr), float(lr_center)
        self.mu, self.beta = float(momentum), float(beta)
        self.lambda0, self.lambda_abs = float(lambda0), float(lambda_abs)
        self.nesterov = bool(nesterov)
        self.sched = PeriodSchedule(K, tau, tau_min, tau_max, sched_seed, sched_mode)
        p = np.asarray(init_params, dtype=np.float64).ravel()
        if p.size == self.d:
            self.x = np.tile(p, (self.K, 1))
            self.y = p.copy()
        elif p.size == (self.K + 1) * self.d:
            self.x = p[: self.K * self.d].reshape(self.K, self.d).copy()
            self.y = p[self.K * self.d:].copy()
        else:
            raise ValueError("init_params must hold d or (K+1)*d values")
        self.v = np.zeros((self.K, self.d))
        self.S = np.zeros((self.K, self.d))
        self.gprev = None
        # kept for inspection by tests
        self.last_norm = np.zeros(self.K)
        self.last_perturbed = np.zeros((self.K, self.d))
        self.last_g1 = np.zeros((self.K, self.d))
        self.last_g2 = np.zeros((self.K, self.d))
        # per replica: the dense model's `last_hidden` diagnostic of the first and second pass
        self.last_hidden = [None] * self.K

    # -- hyper-parameters -------------------------------------------------------------
    def set_scalars(self, lr, rho):
        self.lr, self.rho = float(lr), float(rho)

    def coupling(self, i):
        """lambda_i = lambda0 / (eta tau_i) unless a fixed lambda is given."""
        if self.algorithm == ALG_DATA_PARALLEL:
            return 0.0
        if self.lambda_abs >= 0.0:
            return self.lambda_abs
        return self.lambda0 / (self.lr * self.sched.tau[i])

    # -- the sampler step --------------------------------------------------------------
    def _ascend(self, i, g1):
        n = float(np.sqrt(np.sum(g1 * g1)))
        self.last_norm[i] = n
        xt = self.x[i] + self.rho * g1 / (n + self.gamma)
        self.last_perturbed[i] = xt
        return xt

    def _descend(self, i, g2):
        G = g2 + self.coupling(i) * (self.x[i] - self.y)
        self.v[i] = self.mu * self.v[i] + G
        if self.nesterov:
            self.x[i] = self.x[i] - self.lr * (G + self.mu * self.v[i])
        else:
            self.x[i] = self.x[i] - self.lr * self.v[i]
        if self.noise_scale != 0.0:
            xi = langevin_noise(self.dims, self.d, i, self.t, self.noise_seed, self.shapes, self.bn_mask,
                                self.proj_mask, self.preact)
            self.x[i] = self.x[i] + self.noise_scale * np.sqrt(2.0 * self.lr) * xi
        self.S[i] += self.x[i]

    def step(self, X, labels):
        """One local iteration of every replica on its own minibatch; returns the K
        first-pass losses."""
        losses = np.zeros(self.K)
        if self.algorithm == ALG_DATA_PARALLEL:
            data = [(np.asarray(X[i], dtype=np.float64), np.asarray(labels[i]).astype(np.int64))
                    for i in range(self.K)]
            g1 = np.zeros((self.K, self.d))
            for i, (Xi, li) in enumerate(data):
                losses[i], g1[i] = self.model.loss_and_grad(self.x[i], Xi, li)
            xt = self._ascend_mean(g1)
            g2 = np.zeros((self.K, self.d))
            for i, (Xi, li) in enumerate(data):
                _, g2[i] = self.model.loss_and_grad(xt[i], Xi, li)
            self._descend_mean(g2)
            self.sched.tick()
            self.t += 1
            return losses
        for i in range(self.K):
            Xi = np.asarray(X[i], dtype=np.float64)
            li = np.asarray(labels[i]).astype(np.int64)
            losses[i], g1 = self.model.loss_and_grad(self.x[i], Xi, li)
            hidden1 = getattr(self.model, "last_hidden", None)
            xt = self._ascend(i, g1)
            _, g2 = self.model.loss_and_grad(xt, Xi, li)
            self.last_g1[i], self.last_g2[i] = g1, g2
            self.last_hidden[i] = (hidden1, getattr(self.model, "last_hidden", None))
            self._descend(i, g2)
        self.sched.tick()
        self.t += 1
        return losses

    def _ascend_mean(self, g1):
        """Data-parallel ascent: one perturbation, from the average of the K gradients."""
        gbar = np.mean(g1, axis=0)
        self.last_g1[:] = gbar
        return np.stack([self._ascend(i, gbar) for i in range(self.K)])

    def _descend_mean(self, g2):
        gbar = np.mean(g2, axis=0)
        self.last_g2[:] = gbar
        for i in range(self.K):
            self._descend(i, gbar)

    def step_grads(self, g1, g2):
        """Raw-vector mode: the two gradients are handed in instead of computed."""
        if self.algorithm == ALG_DATA_PARALLEL:
            self._ascend_mean(np.asarray(g1, dtype=np.float64))
            self._descend_mean(np.asarray(g2, dtype=np.float64))
            self.sched.tick()
            self.t += 1
            return
        for i in range(self.K):
            a = np.asarray(g1[i], dtype=np.float64)
            self._ascend(i, a)
            self._descend(i, np.asarray(g2[i], dtype=np.float64))
        self.sched.tick()
        self.t += 1

    # -- the center step ---------------------------------------------------------------
    def sync(self):
        if self.algorithm == ALG_DATA_PARALLEL:
            return 0
        due = self.sched.due()
        if not due:
            return 0
        m = sum(self.sched.count[i] for i in due)
        total = np.zeros(self.d)
        for i in due:
            total += self.S[i]
        gp = total / m - self.y
        g = gp if self.gprev is None else gp + self.beta * (gp - self.gprev)
        self.y = self.y + self.lr_center * g
        self.gprev = gp
        for i in due:
            self.S[i] = 0.0
        self.sched.served(due)
        return len(due)

    # -- read-out ----------------------------------------------------------------------
    def get_params(self, replica):
        return (self.y if replica < 0 else self.x[replica]).copy()

    def get_schedule(self):
        return list(self.sched.tau), list(self.sched.count), self.sched.t_y
