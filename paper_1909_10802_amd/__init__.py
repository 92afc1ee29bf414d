"""Python binding of libga (include/ga.h): argument marshalling only.

Every function below has the name and the argument order of the C entry point
it calls; tensors are passed as torch CUDA tensors (PyTorch is used for device
memory and streams only) and turned into raw device pointers here.  All
arithmetic of the master update runs in the HIP kernels of libga.so.  There is
no CPU fallback: if the library has not been built, importing a function that
needs it raises.
"""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libga.so")

GA_MODE_ASGD, GA_MODE_SA, GA_MODE_SA_STEP, GA_MODE_GA, GA_MODE_GA_HINGE = range(5)
GA_FAMILY_MOMENTUM, GA_FAMILY_DANA, GA_FAMILY_ADAM = range(3)
GA_ARR_THETA, GA_ARR_V, GA_ARR_M, GA_ARR_SNAPSHOT, GA_ARR_WORKER_V, GA_ARR_ADAM_V2 = range(6)
GA_GAP_PARAMETER, GA_GAP_LAYER, GA_GAP_GLOBAL = range(3)
GA_F32, GA_BF16 = 0, 1
GA_OK, GA_ERR_ARG, GA_ERR_WORKER, GA_ERR_ALIGN, GA_ERR_STATE, GA_ERR_HIP = 0, -1, -2, -3, -4, -5
GA_DIST_EXP, GA_DIST_LOGNORMAL, GA_DIST_HETERO, GA_DIST_GAMMA_HOMO, GA_DIST_GAMMA_HETERO = range(5)
GA_SRC_QUADRATIC_NOISE, GA_SRC_BUFFERS = 0, 1
GA_PICK_BY_WORKER, GA_PICK_BY_ARRIVAL = 0, 1

FAMILIES = {"momentum": GA_FAMILY_MOMENTUM, "dana": GA_FAMILY_DANA, "adam": GA_FAMILY_ADAM}
MODES = {"asgd": GA_MODE_ASGD, "sa": GA_MODE_SA, "sa_step": GA_MODE_SA_STEP, "ga": GA_MODE_GA,
         "ga_hinge": GA_MODE_GA_HINGE}


class GaError(RuntimeError):
    def __init__(self, status, message):
        super().__init__("libga status %d: %s" % (status, message))
        self.status = status


class ga_grad_source(C.Structure):
    _fields_ = [("kind", C.c_int), ("dev_a", C.c_void_p), ("dev_theta_star", C.c_void_p), ("seed", C.c_uint64),
                ("sigma", C.c_float), ("persistent", C.c_int), ("dev_scratch_g", C.c_void_p),
                ("host_dev_bufs", C.POINTER(C.c_void_p)), ("n_bufs", C.c_uint32), ("dtype", C.c_int),
                ("pick", C.c_int)]


class ga_diag(C.Structure):
    _fields_ = [("mean_graw", C.c_double), ("frac_gt1", C.c_double), ("frac_gt0", C.c_double),
                ("n_nonfinite", C.c_uint64)]


class ga_config(C.Structure):
    _fields_ = [("N", C.c_uint64), ("n_workers", C.c_uint32), ("family", C.c_int), ("mode", C.c_int),
                ("eta", C.c_float), ("gamma", C.c_float), ("beta", C.c_float), ("eps", C.c_float),
                ("adam_beta1", C.c_float), ("adam_beta2", C.c_float), ("adam_eps", C.c_float),
                ("track_gap", C.c_int), ("gap_scope", C.c_int), ("n_layers", C.c_uint32),
                ("host_layer_sizes", C.c_void_p), ("nesterov", C.c_int)]


class ga_time_model(C.Structure):
    _fields_ = [("dist", C.c_int), ("sigma", C.c_double), ("mean", C.c_double), ("v_mach", C.c_double),
                ("v_task", C.c_double)]


class ga_arrival(C.Structure):
    _fields_ = [("worker", C.c_uint32), ("tau", C.c_float), ("lr", C.c_float), ("inv_bc_prev", C.c_float)]


ARRIVAL_DTYPE = np.dtype([("worker", np.uint32), ("tau", np.float32), ("lr", np.float32), ("inv_bc_prev", np.float32)])

_u64, _u32, _i, _f, _d, _p = C.c_uint64, C.c_uint32, C.c_int, C.c_float, C.c_double, C.c_void_p

# name -> (restype, argtypes); every symbol include/ga.h declares
SIGNATURES = {
    "ga_simulate_schedule": (_i, [_u32, _u64, _i, _d, _u64, _p]),
    "ga_simulate_schedule_ex": (_i, [_u32, _u64, C.POINTER(ga_time_model), _u64, _p, _p]),
    "ga_simulate_speedup": (_i, [_u32, _u64, C.POINTER(ga_time_model), _u64, C.POINTER(_d), C.POINTER(_d)]),
    "ga_delays_from_schedule": (_i, [_u32, _u64, _p, _u64, _p, _p]),
    "ga_plan_arrivals": (_i, [_u32, _u64, _p, _u64, _p, _i, _f, _f, _p]),
    "ga_config_init": (None, [C.POINTER(ga_config)]),
    "ga_workspace_bytes": (C.c_size_t, [_u64, _u32]),
    "ga_workspace_bytes_ex": (C.c_size_t, [C.POINTER(ga_config)]),
    "ga_create_ex": (_i, [C.POINTER(_p), C.POINTER(ga_config), _p, C.c_size_t, _p]),
    "ga_get_array": (_i, [_p, _i, _u32, _p]),
    "ga_get_layer_gaps": (_i, [_p, _p, _u32]),
    "ga_put_array": (_i, [_p, _i, _u32, _p]),
    "ga_create": (_i, [C.POINTER(_p), _u64, _u32, _f, _f, _i, _p, C.c_size_t, _p]),
    "ga_destroy": (None, [_p]),
    "ga_set_beta_eps": (_i, [_p, _f, _f]),
    "ga_set_eta_max": (_i, [_p, _f]),
    "ga_set_lr": (_i, [_p, _f]),
    "ga_set_track_gap": (_i, [_p, _i]),
    "ga_set_theta": (_i, [_p, _p]),
    "ga_set_resident_bytes": (_i, [_p, _u64]),
    "ga_get_resident_bytes": (_u64, [_p]),
    "ga_apply": (_i, [_p, _u32, _p, _i]),
    "ga_apply_queue": (_i, [_p, _u64, _p, _p, _i]),
    "ga_run_schedule": (_i, [_p, _p, _u64, C.POINTER(ga_grad_source)]),
    "ga_run_schedule_lr": (_i, [_p, _p, _u64, C.POINTER(ga_grad_source), _p]),
    "ga_warmup_lr": (_i, [_f, _u32, _u64, _u64, _u64, _p]),
    "ga_quadratic_gradient": (_i, [_p, _u32, C.POINTER(ga_grad_source), _p]),
    "ga_diagnostics": (_i, [_p, _u32, C.POINTER(ga_diag)]),
    "ga_diagnostics_async": (_i, [_p, _u32, _p]),
    "ga_gap_statistics_static": (_i, [_p, _p, _p, _u64, _u64, _f, _f, _f, _p, _p]),
    "ga_get_theta": (_i, [_p, _p]),
    "ga_get_v": (_i, [_p, _p]),
    "ga_get_m": (_i, [_p, _p]),
    "ga_get_snapshot": (_i, [_p, _u32, _p]),
    "ga_put_theta": (_i, [_p, _p]),
    "ga_put_v": (_i, [_p, _p]),
    "ga_put_m": (_i, [_p, _p]),
    "ga_put_snapshot": (_i, [_p, _u32, _p]),
    "ga_step": (_u64, [_p]),
    "ga_get_iter": (_i, [_p, _p]),
    "ga_get_delays": (_i, [_p, _p, _u64, C.POINTER(_u64)]),
    "ga_set_bookkeeping": (_i, [_p, _u64, _p]),
    "ga_get_config": (_i, [_p, C.POINTER(ga_config), C.POINTER(_f)]),
    "ga_state_bytes": (C.c_size_t, [_p]),
    "ga_export_state": (_i, [_p, _p, C.c_size_t, C.POINTER(_u64), _p]),
    "ga_import_state": (_i, [_p, _p, C.c_size_t, _u64, _p]),
    "ga_noise_fill": (_i, [_u64, _u64, _u64, _u64, _p, _p]),
    "ga_probe_streams": (_i, [_u32, _u32, _u64, _p, _p, _p]),
    "ga_probe_streams_ex": (_i, [_u32, _u32, _u32, _i, _u64, _p, _p, _p]),
    "ga_probe_valu": (_i, [_i, _u32, _u32, _p, _p]),
    "ga_box_muller_raw": (_i, [_p, _p, _u64, _p, _p, _p]),
    "ga_last_error": (C.c_char_p, [_p]),
    "ga_version": (C.c_char_p, []),
}

_lib = None


def lib():
    """Load libga.so (after torch, so that both use the same HIP runtime)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("libga.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
                              "or `python paper_1909_10802_amd/build.py` (there is no CPU fallback)")
        import torch  # noqa: F401  (loads the HIP runtime the library binds to)
        L = C.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(L, name)
            fn.restype = res
            fn.argtypes = args
        _lib = L
    return _lib


def _check(status, ctx=None):
    if status != GA_OK:
        raise GaError(status, lib().ga_last_error(ctx).decode())


def _dev(t, dtype=None, n=None):
    """Raw device pointer of a CUDA tensor (no copy)."""
    import torch
    assert isinstance(t, torch.Tensor) and t.is_cuda and t.is_contiguous(), "expected a contiguous CUDA tensor"
    if dtype is not None:
        assert t.dtype == dtype, (t.dtype, dtype)
    if n is not None:
        assert t.numel() >= n, (t.numel(), n)
    return t.data_ptr()


def _stream_ptr(stream):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream


def _np_ptr(a):
    return a.ctypes.data_as(_p)


# ------------------------------------------------------------------ host only
def ga_simulate_schedule(n_workers, T, dist=GA_DIST_EXP, sigma=1.0, seed=0):
    out = np.empty(T, dtype=np.uint32)
    _check(lib().ga_simulate_schedule(n_workers, T, dist, sigma, seed, _np_ptr(out)))
    return out


def time_model(dist, sigma=1.0, mean=128.0, v_mach=0.1, v_task=0.1):
    return ga_time_model(dist, sigma, mean, v_mach, v_task)


def ga_simulate_schedule_ex(n_workers, T, model, seed=0, with_times=False):
    out = np.empty(T, dtype=np.uint32)
    times = np.empty(T, dtype=np.float64) if with_times else None
    _check(lib().ga_simulate_schedule_ex(n_workers, T, C.byref(model), seed, _np_ptr(out),
                                         None if times is None else _np_ptr(times)))
    return (out, times) if with_times else out


def ga_simulate_speedup(n_workers, iters, model, seed=0):
    """(ASGD wall time, SSGD wall time) for n_workers * iters batches."""
    a, s = _d(), _d()
    _check(lib().ga_simulate_speedup(n_workers, iters, C.byref(model), seed, C.byref(a), C.byref(s)))
    return a.value, s.value


def ga_delays_from_schedule(n_workers, schedule, k0=0, host_iter=None):
    schedule = np.ascontiguousarray(schedule, dtype=np.uint32)
    it = np.zeros(n_workers, dtype=np.uint64) if host_iter is None else host_iter
    assert it.dtype == np.uint64 and it.size == n_workers
    tau = np.empty(schedule.size, dtype=np.uint64)
    _check(lib().ga_delays_from_schedule(n_workers, schedule.size, _np_ptr(schedule), k0, _np_ptr(it), _np_ptr(tau)))
    return tau, it


def ga_plan_arrivals(n_workers, schedule, k0, host_iter, mode, eta_k, beta):
    schedule = np.ascontiguousarray(schedule, dtype=np.uint32)
    assert host_iter.dtype == np.uint64 and host_iter.size == n_workers
    rows = np.empty(schedule.size, dtype=ARRIVAL_DTYPE)
    _check(lib().ga_plan_arrivals(n_workers, schedule.size, _np_ptr(schedule), k0, _np_ptr(host_iter), mode, eta_k,
                                  beta, _np_ptr(rows)))
    return rows


# ------------------------------------------------------------------ context
def ga_workspace_bytes(N, n_workers):
    return lib().ga_workspace_bytes(N, n_workers)


def ga_create(N, n_workers, eta, gamma, mode, dev_workspace, stream=None):
    """dev_workspace: a uint8 CUDA tensor of at least ga_workspace_bytes(N, n_workers) bytes."""
    import torch
    ctx = _p()
    ptr = _dev(dev_workspace, torch.uint8)
    _check(lib().ga_create(C.byref(ctx), N, n_workers, eta, gamma, mode, ptr, dev_workspace.numel(),
                           _stream_ptr(stream)))
    return ctx


def ga_config_init(**kw):
    """A ga_config with the library defaults, then the given fields."""
    cfg = ga_config()
    lib().ga_config_init(C.byref(cfg))
    sizes = kw.pop("layer_sizes", None)
    for k, v in kw.items():
        assert hasattr(cfg, k), k
        setattr(cfg, k, v)
    if sizes is not None:
        sizes = np.ascontiguousarray(sizes, dtype=np.uint64)
        cfg.gap_scope, cfg.n_layers, cfg.host_layer_sizes = GA_GAP_LAYER, sizes.size, sizes.ctypes.data
        cfg._keep = sizes
    return cfg


def ga_workspace_bytes_ex(cfg):
    return lib().ga_workspace_bytes_ex(C.byref(cfg))


def ga_create_ex(cfg, dev_workspace, stream=None):
    import torch
    ctx = _p()
    ptr = _dev(dev_workspace, torch.uint8)
    _check(lib().ga_create_ex(C.byref(ctx), C.byref(cfg), ptr, dev_workspace.numel(), _stream_ptr(stream)))
    return ctx


def ga_get_layer_gaps(ctx, n_layers):
    out = np.empty(n_layers, dtype=np.float32)
    _check(lib().ga_get_layer_gaps(ctx, _np_ptr(out), n_layers), ctx)
    return out


def ga_get_array(ctx, which, worker_id, dev_dst):
    import torch
    _check(lib().ga_get_array(ctx, which, worker_id, _dev(dev_dst, torch.float32)), ctx)
    return dev_dst


def ga_put_array(ctx, which, worker_id, dev_src):
    import torch
    _check(lib().ga_put_array(ctx, which, worker_id, _dev(dev_src, torch.float32)), ctx)


def ga_destroy(ctx):
    lib().ga_destroy(ctx)


def ga_set_beta_eps(ctx, beta, eps):
    _check(lib().ga_set_beta_eps(ctx, beta, eps), ctx)


def ga_set_eta_max(ctx, eta_max):
    _check(lib().ga_set_eta_max(ctx, eta_max), ctx)


def ga_set_lr(ctx, eta_k):
    _check(lib().ga_set_lr(ctx, eta_k), ctx)


def ga_set_track_gap(ctx, on):
    _check(lib().ga_set_track_gap(ctx, int(on)), ctx)


def ga_set_theta(ctx, dev_theta0):
    import torch
    _check(lib().ga_set_theta(ctx, _dev(dev_theta0, torch.float32)), ctx)


def ga_apply(ctx, worker_id, dev_grad, grad_dtype=None):
    import torch
    if grad_dtype is None:
        grad_dtype = GA_BF16 if dev_grad.dtype == torch.bfloat16 else GA_F32
    assert dev_grad.dtype == (torch.bfloat16 if grad_dtype == GA_BF16 else torch.float32)
    _check(lib().ga_apply(ctx, worker_id, _dev(dev_grad), grad_dtype), ctx)


def ga_apply_queue(ctx, host_workers, dev_grads, grad_dtype=None):
    """host_workers: worker ids; dev_grads: one CUDA tensor per arrival (all float32 or all bfloat16)."""
    import torch
    host_workers = np.ascontiguousarray(host_workers, dtype=np.uint32)
    assert host_workers.size == len(dev_grads)
    if grad_dtype is None:
        grad_dtype = GA_BF16 if len(dev_grads) and dev_grads[0].dtype == torch.bfloat16 else GA_F32
    want = {GA_BF16: torch.bfloat16, GA_F32: torch.float32}.get(grad_dtype)     # unknown codes: the library refuses
    ptrs = (C.c_void_p * max(len(dev_grads), 1))(*[_dev(g, want) for g in dev_grads])
    _check(lib().ga_apply_queue(ctx, host_workers.size, _np_ptr(host_workers), ptrs, grad_dtype), ctx)


def quadratic_source(dev_a, dev_theta_star, seed, sigma=0.01, persistent=True, dev_scratch_g=None):
    import torch
    s = ga_grad_source()
    s.kind = GA_SRC_QUADRATIC_NOISE
    s.dev_a = _dev(dev_a, torch.float32)
    s.dev_theta_star = _dev(dev_theta_star, torch.float32)
    s.seed = seed
    s.sigma = sigma
    s.persistent = int(persistent)
    s.dev_scratch_g = None if dev_scratch_g is None else _dev(dev_scratch_g, torch.float32)
    s._keep = (dev_a, dev_theta_star, dev_scratch_g)
    return s


def buffer_source(dev_bufs, pick=GA_PICK_BY_WORKER, persistent=False):
    """dev_bufs: list of CUDA tensors (all float32 or all bfloat16), N values each.
    persistent: apply the arrivals of a ga_run_schedule call as a queue, one launch per chunk of them."""
    import torch
    s = ga_grad_source()
    s.kind = GA_SRC_BUFFERS
    ptrs = (C.c_void_p * len(dev_bufs))(*[_dev(b) for b in dev_bufs])
    s.host_dev_bufs = C.cast(ptrs, C.POINTER(C.c_void_p))
    s.n_bufs = len(dev_bufs)
    s.dtype = GA_BF16 if dev_bufs[0].dtype == torch.bfloat16 else GA_F32
    assert all(b.dtype == dev_bufs[0].dtype for b in dev_bufs)
    s.pick = pick
    s.persistent = 1 if persistent else 0
    s._keep = (ptrs, list(dev_bufs))
    return s


def ga_run_schedule(ctx, host_schedule, src, T=None):
    host_schedule = np.ascontiguousarray(host_schedule, dtype=np.uint32)
    T = host_schedule.size if T is None else T
    assert T <= host_schedule.size
    _check(lib().ga_run_schedule(ctx, _np_ptr(host_schedule), T, C.byref(src)), ctx)


def ga_run_schedule_lr(ctx, host_schedule, src, host_eta):
    host_schedule = np.ascontiguousarray(host_schedule, dtype=np.uint32)
    host_eta = np.ascontiguousarray(host_eta, dtype=np.float32)
    assert host_eta.size == host_schedule.size
    _check(lib().ga_run_schedule_lr(ctx, _np_ptr(host_schedule), host_schedule.size, C.byref(src), _np_ptr(host_eta)), ctx)


def ga_warmup_lr(eta, n_workers, warmup_steps, k0, T):
    out = np.empty(T, dtype=np.float32)
    _check(lib().ga_warmup_lr(eta, n_workers, warmup_steps, k0, T, _np_ptr(out)))
    return out


def ga_quadratic_gradient(ctx, worker_id, src, dev_g_out):
    import torch
    _check(lib().ga_quadratic_gradient(ctx, worker_id, C.byref(src), _dev(dev_g_out, torch.float32)), ctx)


def ga_diagnostics(ctx, worker_id):
    d = ga_diag()
    _check(lib().ga_diagnostics(ctx, worker_id, C.byref(d)), ctx)
    return dict(mean_graw=d.mean_graw, frac_gt1=d.frac_gt1, frac_gt0=d.frac_gt0, n_nonfinite=d.n_nonfinite)


DIAG_BYTES = C.sizeof(ga_diag)


def diag_from_device(dev_out):
    """Read a device ga_diag (uint8 CUDA tensor of DIAG_BYTES) back as a dict; waits for the device."""
    raw = dev_out.cpu().numpy().tobytes()
    d = ga_diag.from_buffer_copy(raw)
    return dict(mean_graw=d.mean_graw, frac_gt1=d.frac_gt1, frac_gt0=d.frac_gt0, n_nonfinite=d.n_nonfinite)


def ga_diagnostics_async(ctx, worker_id, dev_out):
    """dev_out: uint8 CUDA tensor of at least DIAG_BYTES; nothing waits."""
    import torch
    _check(lib().ga_diagnostics_async(ctx, worker_id, _dev(dev_out, torch.uint8, DIAG_BYTES)), ctx)
    return dev_out


def ga_gap_statistics_static(dev_theta, dev_snapshot, dev_m, N, k, beta, eta_max, eps, dev_out, stream=None):
    import torch
    _check(lib().ga_gap_statistics_static(_dev(dev_theta, torch.float32, N), _dev(dev_snapshot, torch.float32, N),
                                          _dev(dev_m, torch.float32, N), N, k, beta, eta_max, eps,
                                          _dev(dev_out, torch.uint8, DIAG_BYTES), _stream_ptr(stream)))
    return dev_out


def _getter(name):
    def get(ctx, dev_dst):
        import torch
        _check(getattr(lib(), name)(ctx, _dev(dev_dst, torch.float32)), ctx)
        return dev_dst
    get.__name__ = name
    return get


ga_get_theta, ga_get_v, ga_get_m = _getter("ga_get_theta"), _getter("ga_get_v"), _getter("ga_get_m")
ga_put_theta, ga_put_v, ga_put_m = _getter("ga_put_theta"), _getter("ga_put_v"), _getter("ga_put_m")


def ga_get_snapshot(ctx, worker_id, dev_dst):
    import torch
    _check(lib().ga_get_snapshot(ctx, worker_id, _dev(dev_dst, torch.float32)), ctx)
    return dev_dst


def ga_put_snapshot(ctx, worker_id, dev_src):
    import torch
    _check(lib().ga_put_snapshot(ctx, worker_id, _dev(dev_src, torch.float32)), ctx)


def ga_step(ctx):
    return lib().ga_step(ctx)


def ga_get_iter(ctx, n_workers):
    out = np.empty(n_workers, dtype=np.uint64)
    _check(lib().ga_get_iter(ctx, _np_ptr(out)), ctx)
    return out


def ga_get_delays(ctx):
    n = _u64()
    _check(lib().ga_get_delays(ctx, None, 0, C.byref(n)), ctx)
    out = np.empty(n.value, dtype=np.uint64)
    _check(lib().ga_get_delays(ctx, _np_ptr(out), n.value, C.byref(n)), ctx)
    return out


def ga_get_config(ctx):
    """Returns (ga_config, eta_k)."""
    cfg, eta_k = ga_config(), _f()
    _check(lib().ga_get_config(ctx, C.byref(cfg), C.byref(eta_k)), ctx)
    return cfg, eta_k.value


def ga_set_resident_bytes(ctx, n_bytes):
    _check(lib().ga_set_resident_bytes(ctx, n_bytes), ctx)


def ga_get_resident_bytes(ctx):
    return lib().ga_get_resident_bytes(ctx)


def ga_set_bookkeeping(ctx, k, host_iter):
    host_iter = np.ascontiguousarray(host_iter, dtype=np.uint64)
    _check(lib().ga_set_bookkeeping(ctx, k, _np_ptr(host_iter)), ctx)


def ga_state_bytes(ctx):
    return lib().ga_state_bytes(ctx)


def ga_export_state(ctx, n_workers, dev_dst):
    """Copy the device state into dev_dst (uint8 CUDA tensor); returns (k, iter)."""
    import torch
    k = _u64()
    it = np.empty(n_workers, dtype=np.uint64)
    _check(lib().ga_export_state(ctx, _dev(dev_dst, torch.uint8), dev_dst.numel(), C.byref(k), _np_ptr(it)), ctx)
    return k.value, it


def ga_import_state(ctx, dev_src, k, host_iter):
    import torch
    host_iter = np.ascontiguousarray(host_iter, dtype=np.uint64)
    _check(lib().ga_import_state(ctx, _dev(dev_src, torch.uint8), dev_src.numel(), k, _np_ptr(host_iter)), ctx)


def ga_noise_fill(seed, k, j0, n, dev_out, stream=None):
    import torch
    _check(lib().ga_noise_fill(seed, k, j0, n, _dev(dev_out, torch.float32, n), _stream_ptr(stream)))
    return dev_out


def ga_box_muller_raw(dev_xa, dev_xb, dev_zc, dev_zs, stream=None):
    import torch
    n = dev_xa.numel()
    assert dev_xb.numel() == n and dev_zc.numel() == n and dev_zs.numel() == n
    _check(lib().ga_box_muller_raw(_dev(dev_xa, torch.int32), _dev(dev_xb, torch.int32), n, _dev(dev_zc, torch.float32),
                                   _dev(dev_zs, torch.float32), _stream_ptr(stream)))


PROBE_OPS = {"v_fma_f32": 0, "v_xor_b32": 1, "v_mul_hi_u32": 2, "v_mad_u64_u32": 3, "v_rcp_f32": 4, "v_sqrt_f32": 5,
             "v_div_scale_f32": 6, "v_div_fmas_f32": 7, "v_div_fixup_f32": 8}


def ga_probe_streams(reads, writes, n, stream=None, n_resident=0, tiled=False):
    """reads / writes: lists of float32 CUDA tensors of at least n elements; the first n_resident of each are
    accessed without the non-temporal hint (writes[i] may be reads[i]).  tiled: the first three of each are views
    of one buffer laid out as a master's theta, v, m (see ga_probe_streams_ex in include/ga.h)."""
    import torch
    r = (C.c_void_p * max(1, len(reads)))(*[_dev(t, torch.float32, n) for t in reads])
    w = (C.c_void_p * max(1, len(writes)))(*[_dev(t, torch.float32, n) for t in writes])
    if n_resident or tiled:
        _check(lib().ga_probe_streams_ex(len(reads), len(writes), n_resident, int(tiled), n, r, w, _stream_ptr(stream)))
    else:
        _check(lib().ga_probe_streams(len(reads), len(writes), n, r, w, _stream_ptr(stream)))


def ga_probe_valu(op, blocks, iterations, dev_out, stream=None):
    import torch
    _check(lib().ga_probe_valu(PROBE_OPS.get(op, op), blocks, iterations, _dev(dev_out, torch.int32, 1), _stream_ptr(stream)))


def ga_version():
    return lib().ga_version().decode()


# ------------------------------------------------------------------ convenience
class Master:
    """One master context plus the torch tensors it borrows (workspace)."""

    def __init__(self, N, n_workers, eta=0.1, gamma=0.9, mode=GA_MODE_GA, device="cuda:0", stream=None,
                 beta=None, eps=None, eta_max=None, track_gap=False, theta0=None, family=GA_FAMILY_MOMENTUM,
                 adam_beta1=0.9, adam_beta2=0.999, adam_eps=1e-8, gap_scope=GA_GAP_PARAMETER, layer_sizes=None,
                 nesterov=False):
        import torch
        self.N, self.W, self.mode = N, n_workers, MODES.get(mode, mode)
        self.family = FAMILIES.get(family, family)
        self.device = torch.device(device)
        cfg = ga_config_init(N=N, n_workers=n_workers, family=self.family, mode=self.mode, eta=eta, gamma=gamma,
                             adam_beta1=adam_beta1, adam_beta2=adam_beta2, adam_eps=adam_eps,
                             track_gap=int(track_gap), gap_scope=gap_scope, layer_sizes=layer_sizes,
                             nesterov=int(nesterov))
        self.n_layers = 0 if cfg.gap_scope == GA_GAP_PARAMETER else (1 if cfg.gap_scope == GA_GAP_GLOBAL else cfg.n_layers)
        if beta is not None:
            cfg.beta = beta
        if eps is not None:
            cfg.eps = eps
        self.ctx = None
        with torch.cuda.device(self.device):
            self.workspace = torch.empty(ga_workspace_bytes_ex(cfg), dtype=torch.uint8, device=self.device)
            self.ctx = ga_create_ex(cfg, self.workspace, stream)
        if eta_max is not None:
            ga_set_eta_max(self.ctx, eta_max)
        if theta0 is not None:
            ga_set_theta(self.ctx, theta0)

    def close(self):
        if getattr(self, "ctx", None) is not None:
            ga_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _new(self):
        import torch
        return torch.empty(self.N, dtype=torch.float32, device=self.device)

    def apply(self, worker_id, dev_grad):
        ga_apply(self.ctx, worker_id, dev_grad)

    def apply_queue(self, workers, dev_grads):
        ga_apply_queue(self.ctx, workers, dev_grads)

    def run_schedule(self, schedule, src):
        ga_run_schedule(self.ctx, schedule, src)

    def diagnostics(self, worker_id):
        return ga_diagnostics(self.ctx, worker_id)

    def diagnostics_async(self, worker_id, dev_out=None):
        import torch
        if dev_out is None:
            dev_out = torch.empty(DIAG_BYTES, dtype=torch.uint8, device=self.device)
        return ga_diagnostics_async(self.ctx, worker_id, dev_out)

    def theta(self):
        return ga_get_theta(self.ctx, self._new())

    def v(self):
        return ga_get_v(self.ctx, self._new())

    def m(self):
        return ga_get_m(self.ctx, self._new())

    def snapshot(self, w):
        return ga_get_snapshot(self.ctx, w, self._new())

    def layer_gaps(self):
        return ga_get_layer_gaps(self.ctx, self.n_layers)

    def array(self, which, worker_id=0):
        return ga_get_array(self.ctx, which, worker_id, self._new())

    @property
    def k(self):
        return ga_step(self.ctx)

    def iter(self):
        return ga_get_iter(self.ctx, self.W)

    def delays(self):
        return ga_get_delays(self.ctx)
