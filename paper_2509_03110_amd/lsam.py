"""ctypes binding of liblsam.so: the same entry points as include/lsam.h, argument
marshalling only.  PyTorch appears here solely as the owner of device memory and of the
HIP stream; every step of the method runs in the library's kernels.

The library must have been built (python -m paper_2509_03110_amd.build); loading fails
loudly otherwise -- there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblsam.so")

OK, EINVAL, ENOMEM, EHIP, ESTATE = 0, -1, -2, -3, -4
GEMM_FP32, GEMM_BF16 = 0, 1
SCHED_FIXED, SCHED_REDRAW = 0, 1
ALG_LSAM, ALG_DATA_PARALLEL = 0, 1
STATIC_MAX_D = 1 << 34
LAYER_DENSE, LAYER_HEAD, LAYER_CONV_FIRST, LAYER_CONV_DIRECT, LAYER_CONV_STORED = range(5)
BUF_PARAMS, BUF_VELOCITY, BUF_ITER_SUM, BUF_GRAD, BUF_PERTURBED, BUF_CENTER_DIR = range(6)

EXPORTS = [
    "lsam_workspace_bytes", "lsam_init", "lsam_step", "lsam_step_grads", "lsam_sync",
    "lsam_get_params", "lsam_get_buffer", "lsam_set_buffer", "lsam_get_norms", "lsam_get_schedule",
    "lsam_set_scalars", "lsam_num_params", "lsam_schedule_replay", "lsam_timing_enable",
    "lsam_timing_read", "lsam_probe_peaks", "lsam_destroy", "lsam_last_error",
    "lsam_get_counters", "lsam_set_counters", "lsam_get_activation", "lsam_step_grads_static", "lsam_note_replay", "lsam_set_fused_step", "lsam_layer_info",
]


class lsam_config(C.Structure):
    _fields_ = [
        ("K", C.c_int32), ("n_layers", C.c_int32), ("dims", C.POINTER(C.c_int32)),
        ("d_raw", C.c_int64), ("batch", C.c_int32), ("gemm_dtype", C.c_int32),
        ("rho", C.c_float), ("gamma", C.c_float), ("lr", C.c_float), ("lr_center", C.c_float),
        ("momentum", C.c_float), ("beta", C.c_float), ("lambda0", C.c_float),
        ("lambda_abs", C.c_float), ("nesterov", C.c_int32), ("tau", C.POINTER(C.c_int32)),
        ("tau_min", C.c_int32), ("tau_max", C.c_int32), ("sched_seed", C.c_uint64),
        ("sched_mode", C.c_int32), ("algorithm", C.c_int32),
        ("noise_scale", C.c_float), ("noise_seed", C.c_uint64),
        ("n_conv", C.c_int32), ("img_h", C.c_int32), ("img_w", C.c_int32),
        ("bn_eps", C.c_float), ("pool_mask", C.c_uint64), ("bn_mask", C.c_uint64),
        ("stride_mask", C.c_uint64), ("skip_mask", C.c_uint64), ("proj_mask", C.c_uint64),
        ("global_avg_pool", C.c_int32), ("preact", C.c_int32),
    ]


class lsam_update_desc(C.Structure):
    _fields_ = [
        ("K", C.c_int32), ("d", C.c_int64), ("stride", C.c_int64), ("g_stride", C.c_int64),
        ("rho", C.c_float), ("gamma", C.c_float), ("lr", C.c_float), ("momentum", C.c_float),
        ("nesterov", C.c_int32), ("lambda_", C.POINTER(C.c_float)),
    ]


class LsamError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("lsam error %d: %s" % (code, msg))
        self.code = code


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("%s is missing: run `python -m paper_2509_03110_amd.build`" % LIB_PATH)
        L = C.CDLL(LIB_PATH)
        vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
        cfgp = C.POINTER(lsam_config)
        L.lsam_workspace_bytes.restype = C.c_size_t
        L.lsam_workspace_bytes.argtypes = [cfgp]
        L.lsam_num_params.restype = i64
        L.lsam_num_params.argtypes = [cfgp]
        L.lsam_init.restype = C.c_int
        L.lsam_init.argtypes = [cfgp, vp, i64, vp, C.c_size_t, vp, C.POINTER(vp)]
        L.lsam_step.restype = C.c_int
        L.lsam_step.argtypes = [vp, vp, vp, vp]
        L.lsam_step_grads.restype = C.c_int
        L.lsam_step_grads.argtypes = [vp, vp, vp]
        L.lsam_sync.restype = C.c_int
        L.lsam_sync.argtypes = [vp]
        L.lsam_get_params.restype = C.c_int
        L.lsam_get_params.argtypes = [vp, i32, vp, i64]
        L.lsam_get_buffer.restype = C.c_int
        L.lsam_get_buffer.argtypes = [vp, i32, i32, vp, i64]
        L.lsam_set_buffer.restype = C.c_int
        L.lsam_set_buffer.argtypes = [vp, i32, i32, vp, i64]
        L.lsam_get_norms.restype = C.c_int
        L.lsam_get_norms.argtypes = [vp, vp]
        L.lsam_get_schedule.restype = C.c_int
        L.lsam_get_schedule.argtypes = [vp, vp, vp, vp]
        L.lsam_set_scalars.restype = C.c_int
        L.lsam_set_scalars.argtypes = [vp, C.c_float, C.c_float]
        L.lsam_layer_info.restype = C.c_int
        L.lsam_layer_info.argtypes = [vp, i32, vp, i32]
        L.lsam_set_fused_step.restype = C.c_int
        L.lsam_set_fused_step.argtypes = [vp, i32]
        L.lsam_note_replay.restype = C.c_int
        L.lsam_note_replay.argtypes = [vp]
        L.lsam_get_counters.restype = C.c_int
        L.lsam_get_counters.argtypes = [vp, vp, i64]
        L.lsam_set_counters.restype = C.c_int
        L.lsam_set_counters.argtypes = [vp, vp, i64]
        L.lsam_get_activation.restype = C.c_int
        L.lsam_get_activation.argtypes = [vp, i32, i32, vp, i64]
        L.lsam_step_grads_static.restype = C.c_int
        L.lsam_step_grads_static.argtypes = [C.POINTER(lsam_update_desc)] + [vp] * 9
        L.lsam_schedule_replay.restype = C.c_int
        L.lsam_schedule_replay.argtypes = [cfgp, i32, vp, vp]
        L.lsam_timing_enable.restype = C.c_int
        L.lsam_timing_enable.argtypes = [vp, i32]
        L.lsam_timing_read.restype = C.c_int
        L.lsam_timing_read.argtypes = [vp, i32, vp, vp, vp]
        L.lsam_probe_peaks.restype = C.c_int
        L.lsam_probe_peaks.argtypes = [vp, C.c_size_t, vp, vp, vp, vp]
        L.lsam_destroy.restype = None
        L.lsam_destroy.argtypes = [vp]
        L.lsam_last_error.restype = C.c_char_p
        L.lsam_last_error.argtypes = []
        _lib = L
    return _lib


def last_error() -> str:
    return lib().lsam_last_error().decode()


def _check(rc):
    if rc < 0:
        raise LsamError(rc, last_error())
    return rc


def make_config(K, dims=(), d_raw=0, batch=0, gemm_dtype=GEMM_FP32, rho=0.05, gamma=1e-12,
                lr=0.1, lr_center=1.0, momentum=0.9, beta=0.9, lambda0=0.5, lambda_abs=-1.0,
                nesterov=1, tau=None, tau_min=1, tau_max=1, sched_seed=0,
                sched_mode=SCHED_FIXED, algorithm=ALG_LSAM, noise_scale=0.0, noise_seed=0,
                n_conv=0, img_h=0, img_w=0, pool_mask=0, bn_mask=0, bn_eps=1e-5, stride_mask=0,
                skip_mask=0, global_avg_pool=0, proj_mask=0, preact=0):
    """Fills an lsam_config; returns (config, keepalive) -- keep `keepalive` referenced while
    the config is in use (it owns the dims / tau arrays the struct points to)."""
    cfg = lsam_config()
    keep = []
    cfg.K = K
    cfg.n_layers = max(len(dims) - 1, 0)
    if len(dims):
        arr = (C.c_int32 * len(dims))(*dims)
        keep.append(arr)
        cfg.dims = C.cast(arr, C.POINTER(C.c_int32))
    cfg.d_raw = d_raw
    cfg.batch = batch
    cfg.gemm_dtype = gemm_dtype
    cfg.rho, cfg.gamma, cfg.lr, cfg.lr_center = rho, gamma, lr, lr_center
    cfg.momentum, cfg.beta, cfg.lambda0, cfg.lambda_abs = momentum, beta, lambda0, lambda_abs
    cfg.nesterov = nesterov
    if tau is not None:
        t = (C.c_int32 * len(tau))(*tau)
        keep.append(t)
        cfg.tau = C.cast(t, C.POINTER(C.c_int32))
    cfg.tau_min, cfg.tau_max = tau_min, tau_max
    cfg.sched_seed, cfg.sched_mode = sched_seed, sched_mode
    cfg.algorithm = algorithm
    cfg.noise_scale, cfg.noise_seed = noise_scale, noise_seed
    cfg.n_conv, cfg.img_h, cfg.img_w, cfg.pool_mask = n_conv, img_h, img_w, pool_mask
    cfg.bn_mask, cfg.bn_eps = bn_mask, bn_eps
    cfg.stride_mask, cfg.skip_mask, cfg.global_avg_pool = stride_mask, skip_mask, global_avg_pool
    cfg.proj_mask, cfg.preact = proj_mask, preact
    return cfg, keep


def config_from_workload(w, **over):
    kw = dict(K=w.K, dims=w.dims, d_raw=w.d_raw, batch=w.batch, gemm_dtype=w.gemm_dtype,
              rho=w.rho, gamma=w.gamma, lr=w.lr, lr_center=w.lr_center, momentum=w.momentum,
              beta=w.beta, lambda0=w.lambda0, lambda_abs=w.lambda_abs, nesterov=w.nesterov,
              tau=w.tau, tau_min=w.tau_min, tau_max=w.tau_max, sched_seed=w.sched_seed,
              sched_mode=w.sched_mode, algorithm=w.algorithm, noise_scale=w.noise_scale,
              noise_seed=w.noise_seed, n_conv=w.n_conv, img_h=w.img_h, img_w=w.img_w,
              pool_mask=w.pool_mask, bn_mask=w.bn_mask, bn_eps=w.bn_eps,
              stride_mask=w.stride_mask, skip_mask=w.skip_mask, global_avg_pool=w.global_avg_pool,
              proj_mask=w.proj_mask, preact=w.preact)
    kw.update(over)
    return make_config(**kw)


def lsam_probe_peaks(scratch, stream=None):
    """scratch: a contiguous device tensor (overwritten).  Returns (copy GB/s, bf16 MFMA TFLOP/s,
    fp32 MFMA TFLOP/s) measured on its device."""
    import torch
    out = (C.c_double * 3)()
    st = torch.cuda.current_stream(scratch.device).cuda_stream if stream is None else stream
    _check(lib().lsam_probe_peaks(scratch.data_ptr(), scratch.numel() * scratch.element_size(), st,
                                  C.addressof(out), C.addressof(out) + 8, C.addressof(out) + 16))
    return out[0], out[1], out[2]


def lsam_step_grads_static(x, v, S, y, g1, g2, xt, norms, lam, rho, gamma, lr, momentum, nesterov,
                           d=None, stream=None):
    """x, v, S, xt: device tensors [K, stride]; g1, g2: [K, g_stride]; y: [>= d]; norms: [K] or
    None; lam: K host floats.  d defaults to the row length of x."""
    import torch
    K = x.shape[0]
    u = lsam_update_desc()
    u.K, u.d = K, (x.shape[1] if d is None else d)
    u.stride, u.g_stride = x.stride(0), g1.stride(0)
    u.rho, u.gamma, u.lr, u.momentum, u.nesterov = rho, gamma, lr, momentum, nesterov
    arr = (C.c_float * K)(*[float(a) for a in lam])
    u.lambda_ = C.cast(arr, C.POINTER(C.c_float))
    st = torch.cuda.current_stream(x.device).cuda_stream if stream is None else stream
    ptr = lambda t: None if t is None else t.data_ptr()
    return _check(lib().lsam_step_grads_static(C.byref(u), ptr(x), ptr(v), ptr(S), ptr(y), ptr(g1),
                                               ptr(g2), ptr(xt), ptr(norms), st))


def lsam_workspace_bytes(cfg) -> int:
    return lib().lsam_workspace_bytes(C.byref(cfg))


def lsam_num_params(cfg) -> int:
    return lib().lsam_num_params(C.byref(cfg))


def lsam_schedule_replay(cfg, n_ticks):
    due = np.zeros((n_ticks, cfg.K), dtype=np.int32)
    tau = np.zeros((n_ticks, cfg.K), dtype=np.int32)
    _check(lib().lsam_schedule_replay(C.byref(cfg), n_ticks, due.ctypes.data, tau.ctypes.data))
    return due, tau


class Lsam:
    """Owns one lsam_ctx plus the torch tensor that backs its workspace."""

    def __init__(self, cfg, init_params, device="cuda:0", stream=None, keep=None):
        import torch
        self._keep = keep
        self.cfg = cfg
        self.K = cfg.K
        self.d = lsam_num_params(cfg)
        nbytes = lsam_workspace_bytes(cfg)
        if nbytes == 0:
            raise LsamError(EINVAL, last_error())
        self.device = torch.device(device)
        self.workspace = torch.empty(nbytes + 256, dtype=torch.uint8, device=self.device)
        base = self.workspace.data_ptr()
        self._ws_ptr = (base + 255) // 256 * 256
        self.stream = stream if stream is not None else torch.cuda.current_stream(self.device)
        init = np.ascontiguousarray(init_params, dtype=np.float32).ravel()
        h = C.c_void_p()
        with torch.cuda.device(self.device):
            _check(lib().lsam_init(C.byref(cfg), init.ctypes.data, init.size, self._ws_ptr, nbytes,
                                   self.stream.cuda_stream, C.byref(h)))
        self._h = h

    def lsam_step(self, X, labels, loss=None):
        return _check(lib().lsam_step(self._h, X.data_ptr(), labels.data_ptr(),
                                      None if loss is None else loss.data_ptr()))

    def lsam_step_grads(self, g1, g2):
        return _check(lib().lsam_step_grads(self._h, g1.data_ptr(), g2.data_ptr()))

    def lsam_sync(self):
        return _check(lib().lsam_sync(self._h))

    def lsam_get_params(self, replica):
        out = np.empty(self.d, dtype=np.float32)
        _check(lib().lsam_get_params(self._h, replica, out.ctypes.data, out.size))
        return out

    def lsam_get_buffer(self, which, replica):
        out = np.empty(self.d, dtype=np.float32)
        _check(lib().lsam_get_buffer(self._h, which, replica, out.ctypes.data, out.size))
        return out

    def lsam_set_buffer(self, which, replica, src):
        a = np.ascontiguousarray(src, dtype=np.float32).ravel()
        return _check(lib().lsam_set_buffer(self._h, which, replica, a.ctypes.data, a.size))

    def lsam_get_norms(self):
        out = np.empty(self.K, dtype=np.float32)
        _check(lib().lsam_get_norms(self._h, out.ctypes.data))
        return out

    def lsam_get_schedule(self):
        tau = np.zeros(self.K, dtype=np.int32)
        cnt = np.zeros(self.K, dtype=np.int32)
        ty = C.c_int64(0)
        _check(lib().lsam_get_schedule(self._h, tau.ctypes.data, cnt.ctypes.data, C.byref(ty)))
        return tau.tolist(), cnt.tolist(), ty.value

    def lsam_layer_info(self, layer):
        """(kind, dx_stored, norm_route, rows, fan_in, out, projection channels, projection step)
        of layer `layer`; see include/lsam.h."""
        out = np.zeros(8, dtype=np.int32)
        _check(lib().lsam_layer_info(self._h, layer, out.ctypes.data, out.size))
        return tuple(int(v) for v in out)

    def lsam_set_fused_step(self, on):
        return _check(lib().lsam_set_fused_step(self._h, 1 if on else 0))

    def lsam_note_replay(self):
        return _check(lib().lsam_note_replay(self._h))

    def lsam_get_counters(self):
        out = np.zeros(2 * self.K + 3, dtype=np.int64)
        _check(lib().lsam_get_counters(self._h, out.ctypes.data, out.size))
        return out

    def lsam_set_counters(self, state):
        a = np.ascontiguousarray(state, dtype=np.int64).ravel()
        return _check(lib().lsam_set_counters(self._h, a.ctypes.data, a.size))

    def lsam_get_activation(self, layer, replica):
        width, batch = self.cfg.dims[layer], self.cfg.batch
        out = np.empty((batch, width), dtype=np.float32)
        _check(lib().lsam_get_activation(self._h, layer, replica, out.ctypes.data, out.size))
        return out

    def lsam_set_scalars(self, lr, rho):
        return _check(lib().lsam_set_scalars(self._h, lr, rho))

    def lsam_timing_enable(self, on):
        return _check(lib().lsam_timing_enable(self._h, 1 if on else 0))

    def lsam_timing_read(self):
        cap = 32
        names = (C.c_char_p * cap)()
        counts = (C.c_int64 * cap)()
        ms = (C.c_double * cap)()
        n = _check(lib().lsam_timing_read(self._h, cap, names, counts, ms))
        return {names[i].decode(): (counts[i], ms[i]) for i in range(n)}

    def close(self):
        if getattr(self, "_h", None):
            lib().lsam_destroy(self._h)
            self._h = None
            self.workspace = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
