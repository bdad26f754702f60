#!/usr/bin/env python3
"""Throughput of the K-replica LSAM hot path on one MI355X.

One "step" is one pass of the whole path over one batch of synthetic input: `lsam_step`
(forward/backward, gradient norm, ascent perturbation, second forward/backward, descent +
coupling for all K replicas) followed by `lsam_sync` (schedule test and, when replicas are
due, the center update).  Inputs are resident in HBM before the timed region starts.

Prints ONE JSON line: replica-samples/s plus a `roofline` object for the dominant kernel
class (HIP-event durations measured inside the library on its own stream over a second run
of the same steps) and a `cpu_baseline` object (the CPU oracle timed on a bounded sample).
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import workloads  # noqa: E402

PEAK_HBM_GBS = 8000.0
PEAK_TFLOPS = {0: 157.3, 1: 2500.0}   # dense MFMA: fp32, bf16


# HBM bytes per launch of each kernel class, from two `rocprofv3 --pmc` runs of this script
# (FETCH_SIZE, then WRITE_SIZE; KiB per dispatch scaled by what the same counter reads for a plain
# 1 GiB device copy: x2.0 and x1.0), summed over the dispatches of a class and divided by its
# launches (a split-K GEMM and its reduce count as one launch).  The figures belong to the
# kernel sources whose digest is TRAFFIC_SOURCES; with any other sources `traffic` is null.
TRAFFIC_SOURCES = "184631bf3fbaf3a4"
TRAFFIC = {
    "cfg2": {"bias_grad": 2148523, "center": 84162976, "descent": 538499328, "gemm_dw": 43632755,
             "gemm_dx": 42127701, "gemm_fwd": 62107669, "perturb": 201932160},
    "cfg3": {"bias_grad": 13690112, "center": 1393525408, "descent": 877295, "gemm_dw_ascend":
             732954300, "gemm_dw_norm": 17543979, "gemm_dw_step": 2905857877, "gemm_dx":
             250149963, "gemm_fwd": 144075458, "softmax_ce": 1429696},
    "cfg4": {"center": 2400049184, "descent": 25600058581, "perturb": 9600045269,
             "sumsq_partials": 3416877589},
    "cfg5": {"bias_grad": 117981832, "descent": 3481941, "gemm_dw_ascend": 6219425829,
             "gemm_dw_norm": 152019669, "gemm_dw_step": 27294712777, "gemm_dx": 2581714869,
             "gemm_fwd": 1161916226, "softmax_ce": 96450869},
    "cnn5": {"bias_grad": 17354844, "conv_first": 80453440, "descent": 79486763, "gemm_dw":
             67376004, "gemm_dx": 34787669, "gemm_fwd": 38345732, "perturb": 29800448, "pool":
             68586073},
    "cnn5bn": {"batchnorm": 157826080, "bias_grad": 562773, "conv_first": 80449835, "descent":
             79552597, "gemm_dw": 67362485, "gemm_dx": 34787669, "gemm_fwd": 38344209, "perturb":
             29825024, "pool": 68585845},
    "resnet18": {"batchnorm": 259997189, "conv_first": 155183819, "descent": 1431000491,
             "gemm_dw": 308601196, "gemm_dx": 178777639, "gemm_fwd": 230439253, "perturb":
             536618624, "pool": 183890665, "unfold_fold": 218021649},
    "resnet18bf": {"batchnorm": 259998289, "bias_grad": 50432, "conv_first": 155182635, "descent":
             1431003904, "gemm_dw": 268401223, "gemm_dx": 145274408, "gemm_fwd": 274711036,
             "perturb": 536618453, "pool": 183890643, "softmax_ce": 124587, "unfold_fold":
             218021620},
    "resnet20": {"batchnorm": 86666182, "descent": 34874283, "gemm_dw": 212806394, "gemm_dx":
             269469124, "gemm_fwd": 100369632, "perturb": 13073408, "pool": 64194118,
             "unfold_fold": 328611381},
    "resnet34": {"batchnorm": 244145097, "bias_grad": 347008, "conv_first": 155250368, "descent":
             2731215403, "gemm_dw": 264940556, "gemm_dx": 153711067, "gemm_fwd": 215734746,
             "perturb": 1024204416, "pool": 195406042, "softmax_ce": 485291, "unfold_fold":
             218021544},
    "vgg16": {"batchnorm": 175729217, "bias_grad": 1091675, "conv_first": 155189792, "descent":
             1952575829, "gemm_dw": 140527392, "gemm_dx": 16961707, "gemm_fwd": 137751684,
             "perturb": 732209579, "pool": 89627452},
    "vgg16bf": {"batchnorm": 175695851, "bias_grad": 1011170, "conv_first": 155195029, "descent":
             1952580053, "gemm_dw": 113747526, "gemm_dx": 12092075, "gemm_fwd": 169044908,
             "perturb": 732209749, "pool": 89627526, "softmax_ce": 124587},
    "wrn16x10": {"batchnorm": 736315405, "descent": 2191812864, "gemm_dw": 1854432135, "gemm_dx":
             549450901, "gemm_fwd": 1184345296, "perturb": 821921621, "pool": 441879842,
             "unfold_fold": 629743101},
    "wrn16x10bf": {"batchnorm": 736315944, "bias_grad": 50048, "descent": 2191814955, "gemm_dw":
             1114631144, "gemm_dx": 496001376, "gemm_fwd": 1400264620, "perturb": 821921707,
             "pool": 441879842, "softmax_ce": 124587, "unfold_fold": 629743085},
    "wrn28x10": {"batchnorm": 760367501, "bias_grad": 346880, "descent": 4678217856, "gemm_dw":
             1943620653, "gemm_dx": 458547460, "gemm_fwd": 1271969861, "perturb": 1754327680,
             "pool": 508961023, "softmax_ce": 485035, "unfold_fold": 629743043},
    "wrn40x10": {"batchnorm": 768818096, "bias_grad": 346880, "descent": 7157244245, "gemm_dw":
             2026127685, "gemm_dx": 458552949, "gemm_fwd": 1321328546, "perturb": 2683965739,
             "pool": 533675103, "softmax_ce": 485376, "unfold_fold": 629742957},
}


def kernel_sources_digest():
    import glob
    import hashlib
    h = hashlib.sha256()
    # the files that hold device code (the host engine, lsam_api.hip and engine.h, launches
    # these kernels but does not change what one launch of them moves)
    files = sorted(glob.glob(os.path.join(ROOT, "paper_2509_03110_amd", "csrc", "kernels_*.hip")) +
                   [os.path.join(ROOT, "paper_2509_03110_amd", "csrc", h) for h in ("b32s.h", "langevin.h")])
    for f in files:
        with open(f, "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def layer_table(eng, w):
    """What the library reports about each layer (`lsam_layer_info`): which kernels serve it, the
    rows of its matrix products, whether its gradients are stored."""
    return [eng.lsam_layer_info(l) for l in range(len(w.dims) - 1)]


def gemm_flops(w, layers):
    """Per all-replica step (both passes): flops of the forward, dX and dW GEMM classes and of
    the first convolution layer's own kernels.  On the fused path (bf16 dense model) the
    weight-gradient product is formed for the perturbed operand copy and, at the perturbed
    point, for the sampler step; the norm of the first-pass gradient comes from the Gram
    matrices of the product's factors, 2 B^2 (out + in) flops, or from a product whose result
    is only summed."""
    from paper_2509_03110_amd import lsam
    K = w.K
    per = [float(rows) * fi * fo if kind not in (lsam.LAYER_HEAD, lsam.LAYER_CONV_FIRST) else 0.0
           for kind, _, _, rows, fi, fo, _, _ in layers]
    first = sum(float(rows) * fi * fo for kind, _, _, rows, fi, fo, _, _ in layers if kind == lsam.LAYER_CONV_FIRST)
    proj = sum(float(rows) * pc * fo for _, _, _, rows, _, fo, pc, _ in layers)    # 1x1 projections
    sw, sw_dx = sum(per) + proj, sum(per[1:]) + proj
    out = {"gemm_fwd": 2 * 2.0 * sw * K, "gemm_dx": 2 * 2.0 * sw_dx * K}
    if first:
        out["conv_first"] = 2 * 2 * 2.0 * first * K      # forward and weight gradient
    if any(r[2] for r in layers):
        out["gemm_dw_ascend"] = out["gemm_dw_step"] = 2.0 * sw * K
        out["gemm_dw_norm"] = K * sum(2.0 * rows * rows * (fi + fo) if route == 2 else 2.0 * rows * fi * fo
                                      for _, _, route, rows, fi, fo, _, _ in layers)
    else:
        out["gemm_dw"] = 2 * 2.0 * sw * K
    return out


def conv_bytes(w, layers):
    """Algorithmic bytes per all-replica step (both passes) of the kernels around the
    convolution GEMMs: where an unfolded image is stored it is written once (plus the image
    read), where its gradient is stored that is read once (plus the image gradient written);
    the pool reads its input and writes a quarter of it, its backward pass reads both and
    writes the full-size gradient."""
    from paper_2509_03110_amd import lsam
    unfold = pool = bn = 0.0
    for l in range(w.n_conv):
        kind, dx_stored, _, rows, _, _, proj_c, proj_step = layers[l]
        cin, cout = w.dims[l], w.dims[l + 1]
        st2 = 4 if (w.stride_mask >> l) & 1 else 1    # pixels of the image read per output pixel
        if kind == lsam.LAYER_CONV_STORED:
            unfold += rows * (st2 * cin + 9 * cin) * 4.0
        if dx_stored:
            unfold += rows * (9 * cin + st2 * cin) * 4.0
        if proj_c:
            # projection: its normalisation costs what the layer's own does (below), and its
            # output is read once more where the two branches meet; the gather for a strided
            # one reads and writes the pixels it keeps; backward, the gradient of those pixels
            # is added to the block input's gradient under that input's mask (3 reads, 1 write)
            # (a pre-activation block's bare projection is added to the convolution's output
            # instead: two reads and a write)
            if w.preact:
                pool += rows * cout * 4.0 * 3
            else:
                bn += rows * cout * 4.0 * (1 + 1 + 2 + 3)
            if proj_step == 2:
                unfold += rows * proj_c * 4.0 * 2
            pool += rows * proj_c * 4.0 * 4
        elif (w.skip_mask >> l) & 1 and w.preact:
            # identity shortcut of a pre-activation block: the sum two convolutions below is added
            # to this one's (forward), this one's gradient to that one's (backward)
            pool += rows * cout * 4.0 * (3 + 3)
        elif (w.skip_mask >> l) & 1:
            # shortcut: read with the normalisation (forward); backward reads dY, the mask and the
            # block input's gradient and writes the latter
            pool += rows * w.dims[l - 1] * 4.0 * (1 + 4)
        if (w.pool_mask >> l) & 1:
            pool += rows * cout * 4.0 * (1.25 + 2.25)
        if (w.bn_mask >> l) & 1:
            # statistics read Z; normalise+ReLU reads Z, writes the activation; the backward
            # sums read Z and dY; the backward apply reads Z and dY and writes dZ
            bn += rows * cout * 4.0 * (1 + 2 + 2 + 3)
    out = {}
    if bn:
        out["batchnorm"] = 2 * bn * w.K
    if unfold:
        out["unfold_fold"] = 2 * unfold * w.K
    if pool:
        out["pool"] = 2 * pool * w.K
    return out


def stream_bytes(w, fused_step=False, restarts=0.0):
    """Algorithmic bytes per all-replica step of the update-path kernels (reads + writes
    the method itself requires; y is shared by the K replicas): descent reads x, g2, v, S
    (16 B per parameter) and writes x, v, S (12 B), plus the bf16 operand copy (2 B) in bf16
    mode, plus y once for all replicas.  `restarts`: replicas per step, on average, whose sum
    of iterates starts again from zero (served by the center update one tick before): their S
    is written but not read."""
    n = float(w.K) * w.d
    bf = w.gemm_dtype == 1 and not w.n_conv
    out = {"sumsq_partials": 4 * n,
           "perturb": (10 if bf else 12) * n,
           "descent": (30 if bf else 28) * n + 4.0 * w.d - 4.0 * restarts * w.d}
    if fused_step:
        # the weight matrices take their step where the second-pass gradient is produced: that
        # kernel reads x, v, S (12 B per parameter) and y once, writes x, v, S (12 B) and the
        # bf16 operand copy (2 B), and neither writes nor reads g2; the separate kernel is left
        # with the bias vectors
        nw = sum(a * b for a, b in w.layer_shapes)
        nb = w.d - nw
        out["gemm_dw_step"] = 26.0 * w.K * nw + 4.0 * nw - 4.0 * restarts * nw
        out["descent"] = 28.0 * w.K * nb + 4.0 * nb - 4.0 * restarts * nb
        # the ascent GEMMs read x and write the bf16 copy of x~; no perturbation kernel runs
        out["gemm_dw_ascend"] = 6.0 * w.K * nw
        del out["perturb"]
    return out


def make_inputs(w, torch, dev, n_sets):
    sets = []
    if w.dims:
        for s in range(n_sets):
            X, lab = workloads.batch(w, s)
            Xd = torch.from_numpy(X).to(dev)
            if w.gemm_dtype == 1 and not w.n_conv:
                Xd = Xd.to(torch.bfloat16)
            sets.append((Xd.contiguous(), torch.from_numpy(lab).to(dev)))
    else:
        # raw-vector mode: fixed gradient buffers ~ N(0, grad_std^2), generated on the device
        gen = torch.Generator(device=dev)
        gen.manual_seed(w.data_seed)
        g1 = torch.randn(w.K, w.d_raw, device=dev, generator=gen) * w.grad_std
        g2 = torch.randn(w.K, w.d_raw, device=dev, generator=gen) * w.grad_std
        sets.append((g1, g2))
    return sets


def cpu_baseline(w, budget_s=20.0):
    """Times the oracle, single-threaded, on a bounded sample of the workload."""
    from threadpoolctl import threadpool_limits
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    from util import oracle_from
    with threadpool_limits(limits=1):
        if w.dims:
            # one replica; shrink the batch for the two largest workloads
            frac = {"cfg5": 8, "cfg3": 2, "vgg16": 16, "vgg16bf": 16, "resnet20": 4}.get(w.name, 1)
            ws = w.scaled(K=1, batch=max(w.batch // frac, 1), tau=(10 ** 6,))
            o = oracle_from(ws, workloads.init_params(ws))
            X, lab = workloads.batch(ws, 0)
            n, t0 = 0, time.perf_counter()
            while True:
                o.step(X, lab)
                n += 1
                if time.perf_counter() - t0 > budget_s / 2 or n >= 20:
                    break
            dt = time.perf_counter() - t0
            value = n * ws.batch / dt
            sample = ("%d step(s) of 1 replica at batch %d (of K=%d, B=%d); samples/s of that bounded "
                      "sample, taken as the rate of the whole workload (work per sample is the same: "
                      "extrapolated)" % (n, ws.batch, w.K, w.batch))
            unit = "replica-samples/s"
        else:
            d = min(w.d_raw, 10_000_000)
            ws = w.scaled(K=1, d_raw=d, tau=(4,))
            o = oracle_from(ws, workloads.init_params(ws))
            g1, g2 = workloads.raw_grads(ws, 0)
            n, t0 = 0, time.perf_counter()
            while True:
                o.step_grads(g1, g2)
                o.sync()
                n += 1
                if time.perf_counter() - t0 > budget_s / 2 or n >= 20:
                    break
            dt = time.perf_counter() - t0
            value = n * d / dt
            sample = ("%d iteration(s) of 1 replica at d=%d (of K=%d, d=%d); extrapolated as above"
                      % (n, d, w.K, w.d_raw))
            unit = "replica-params/s"
    model = "unknown"
    try:
        with open("/proc/cpuinfo") as fh:
            for line in fh:
                if line.startswith("model name"):
                    model = line.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    return {"value": value, "unit": unit, "cores": 1, "kind": "oracle", "sample": sample,
            "host_cpu": model, "host_cores": os.cpu_count()}


def default_steps(w):
    return {"cfg1": 200, "cfg2": 200, "cnn5": 100, "cnn5bn": 100}.get(w.name, 20)


def run_workload(w, steps, warmup, kernel_timing=True):
    """Times `steps` steps of workload `w` after `warmup` untimed ones; returns the fields of
    the JSON line that belong to this workload."""
    import torch
    from paper_2509_03110_amd import lsam
    dev = torch.device("cuda:0")
    cfg, keep = lsam.config_from_workload(w)
    eng = lsam.Lsam(cfg, workloads.init_params(w), device=dev, keep=keep)
    sets = make_inputs(w, torch, dev, w.batch_pool or 8)
    loss = torch.zeros(w.K, device=dev)

    def one(i):
        a, b = sets[i % len(sets)]
        if w.dims:
            eng.lsam_step(a, b, loss)
        else:
            eng.lsam_step_grads(a, b)
        eng.lsam_sync()

    for i in range(warmup):
        one(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        one(i)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms = dt / steps * 1e3

    if w.dims:
        value, unit, metric = w.K * w.batch / (dt / steps), "replica-samples/s", \
            "replica-samples/sec per LSAM step"
    else:
        value, unit, metric = w.K * w.d_raw / (dt / steps), "replica-params/s", \
            "replica-params/sec per LSAM update iteration"

    roof, kernels = None, {}
    if kernel_timing:
        eng.lsam_timing_enable(True)
        for i in range(steps):
            one(i)
        stats = eng.lsam_timing_read()
        eng.lsam_timing_enable(False)
        layers = layer_table(eng, w) if w.dims else []
        fused_step = any(r[2] for r in layers)
        flops = gemm_flops(w, layers) if w.dims else {}
        # center update: 4 B/param per due replica (S read; starting it again from zero costs
        # no write, the next step simply does not read it) + 16 B/param (y and g'_prev read and
        # written), summed over the ticks of this run that had a sync
        first = warmup + steps
        due, _ = lsam.lsam_schedule_replay(cfg, first + steps)
        nd = due[first:].sum(axis=1)
        restarts = float(due[first - 1:-1].sum()) / steps     # served one tick earlier
        nbytes = stream_bytes(w, fused_step, restarts)
        nbytes.update(conv_bytes(w, layers))
        nbytes["center"] = float(np.sum((4.0 * nd + 16.0) * (nd > 0))) * w.d / steps
        traffic = TRAFFIC.get(w.name, {}) if kernel_sources_digest() == TRAFFIC_SOURCES else {}
        for name, (cnt, tot) in stats.items():
            if cnt == 0:
                continue
            k = {"launches_per_step": cnt / steps, "ms_per_step": tot / steps,
                 "avg_launch_ms": tot / cnt}
            if name in ("gemm_dw_step", "gemm_dw_ascend") and name in nbytes and tot > 0:
                # a contraction whose epilogue streams the sampler state: priced against the
                # roof that binds it (HBM), with its matrix-unit rate beside it
                k.update(bound="hbm", achieved=nbytes[name] * steps / (tot * 1e-3) / 1e9,
                         peak=PEAK_HBM_GBS, unit="GB/s",
                         algorithmic_bytes_per_launch=nbytes[name] * steps / cnt,
                         mfma_tflops=flops[name] * steps / (tot * 1e-3) / 1e12)
            elif name in flops and tot > 0:
                k.update(bound="mfma", achieved=flops[name] * steps / (tot * 1e-3) / 1e12,
                         peak=PEAK_TFLOPS[w.gemm_dtype], unit="TFLOP/s",
                         algorithmic_flops_per_launch=flops[name] * steps / cnt)
            elif name in nbytes and tot > 0:
                k.update(bound="hbm", achieved=nbytes[name] * steps / (tot * 1e-3) / 1e9,
                         peak=PEAK_HBM_GBS, unit="GB/s",
                         algorithmic_bytes_per_launch=nbytes[name] * steps / cnt)
            if "achieved" in k:
                k["frac"] = k["achieved"] / k["peak"]
            k["traffic"] = traffic.get(name)
            kernels[name] = k
        ranked = [n for n in sorted(kernels, key=lambda n: -kernels[n]["ms_per_step"])
                  if "achieved" in kernels[n]]
        if ranked:
            top = kernels[ranked[0]]
            roof = {"kernel": ranked[0], "bound": top["bound"], "achieved": top["achieved"],
                    "peak": top["peak"], "unit": top["unit"], "frac": top["frac"],
                    "traffic": top["traffic"], "avg_launch_ms": top["avg_launch_ms"]}

    out = {
        "metric": metric, "value": value, "unit": unit, "n_gpus": 1, "steps": steps,
        "warmup": warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32" if (w.gemm_dtype == 0) else "bf16 operands, f32 accumulate and master weights",
        "data": "synthetic",
        "config": {"workload": w.name, "K": w.K, "dims": list(w.dims), "n_conv": w.n_conv,
                   "image": [w.img_h, w.img_w], "pool_mask": w.pool_mask, "bn_mask": w.bn_mask,
                   "d": w.d, "batch": w.batch,
                   "rho": w.rho, "lr": w.lr, "momentum": w.momentum, "algorithm": w.algorithm,
                   "noise_scale": w.noise_scale,
                   "periods": eng.lsam_get_schedule()[0]},
        "roofline": roof, "kernels": kernels,
    }
    eng.close()
    del eng, sets
    torch.cuda.empty_cache()
    return out


def add_measured_fractions(out, w, peaks):
    """The same fractions against what the simplest kernels reach on this very device."""
    copy_gbs, bf16_tf, f32_tf = peaks
    mfma_meas = bf16_tf if w.gemm_dtype == 1 else f32_tf
    for k in list(out["kernels"].values()) + ([out["roofline"]] if out["roofline"] else []):
        if k.get("bound") == "mfma":
            k["frac_of_measured"] = k["achieved"] / mfma_meas
        elif k.get("bound") == "hbm":
            k["frac_of_measured"] = k["achieved"] / copy_gbs


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="cfg5", choices=sorted(workloads.WORKLOADS),
                    help="the timed workload (default: the largest configuration that fits one GPU)")
    ap.add_argument("--also", default=None,
                    help="comma-separated workloads reported in short form under `other_workloads` "
                         "(default: cfg2,cfg3,cfg4 when the workload is cfg5; 'none' for none)")
    ap.add_argument("--algorithm", type=int, default=0, choices=[0, 1],
                    help="0 = LSAM (default), 1 = synchronous data-parallel baseline")
    ap.add_argument("--noise-scale", type=float, default=0.0,
                    help="sigma of the Langevin sampler (0 = noise-free, the default)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-timing", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: the path holds all K replicas on a single MI355X and "
              "uses no collectives, so --gpus %d is not supported." % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2509_03110_amd import lsam
    if not torch.cuda.is_available():
        print("no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = torch.device("cuda:0")
    w = workloads.WORKLOADS[args.workload]
    if args.algorithm or args.noise_scale:
        w = w.scaled(algorithm=args.algorithm, noise_scale=args.noise_scale, noise_seed=1)
    steps = args.steps if args.steps is not None else default_steps(w)
    timing = not args.no_kernel_timing

    out = run_workload(w, steps, args.warmup, timing)
    also = args.also if args.also is not None else ("cfg2,cfg3,cfg4" if w.name == "cfg5" else "none")
    others = {}
    for name in [n for n in also.split(",") if n and n != "none" and n != w.name]:
        wo = workloads.WORKLOADS[name]
        others[name] = (wo, run_workload(wo, min(default_steps(wo), 50), args.warmup, timing))
    if timing:
        scratch = torch.empty(1 << 28, dtype=torch.float32, device=dev)          # 1 GiB
        peaks = lsam.lsam_probe_peaks(scratch)
        del scratch
        out["measured_peaks"] = {"copy_GBps": peaks[0], "mfma_bf16_TFLOPs": peaks[1],
                                 "mfma_f32_TFLOPs": peaks[2]}
        add_measured_fractions(out, w, peaks)
        for wo, r in others.values():
            add_measured_fractions(r, wo, peaks)
    if others:
        keep = ("bound", "achieved", "peak", "unit", "frac", "frac_of_measured", "ms_per_step",
                "avg_launch_ms", "launches_per_step")
        out["other_workloads"] = {
            name: {"value": r["value"], "unit": r["unit"], "ms_per_step": r["ms_per_step"],
                   "steps": r["steps"], "dtype": r["dtype"],
                   "kernels": {k: {f: v[f] for f in keep if f in v} for k, v in r["kernels"].items()
                               if "achieved" in v}}
            for name, (wo, r) in others.items()}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
