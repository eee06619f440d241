"""ctypes binding of libhop.so: same names as include/hop.h, argument marshalling only.

Every function of the C ABI is exposed under its C name and raises HopError on a
negative return code (hop_simulate returns its schedule also on a stall and
reports it through `.stalled`).  Nothing is computed here.
"""
import ctypes as C
import os

import numpy as np

HOP_MAX_A = 32
HOP_OK = 0
HOP_ERR_INVALID_ARG, HOP_ERR_BAD_GRAPH, HOP_ERR_BAD_WEIGHTS, HOP_ERR_BAD_BACKUP = -1, -2, -3, -4
HOP_ERR_ARENA_TOO_SMALL, HOP_ERR_DEADLOCK, HOP_ERR_SLOT_DEAD, HOP_ERR_HIP = -5, -6, -7, -8
HOP_ERR_NO_DEVICE, HOP_ERR_STATE, HOP_ERR_NOMEM = -9, -10, -11
HOP_DELAY_NONE, HOP_DELAY_EXP1, HOP_DELAY_BERNOULLI6, HOP_DELAY_TABLE = 0, 1, 2, 3
HOP_GRAD_ZERO, HOP_GRAD_SVM_DENSE, HOP_GRAD_SVM_CSR, HOP_GRAD_SYNTH, HOP_GRAD_EXTERNAL = 0, 1, 2, 3, 4
HOP_STEP, HOP_JUMP, HOP_APPLY, HOP_REDUCE = 0, 1, 2, 3
HOP_KERNEL_MIX, HOP_KERNEL_GRAD, HOP_KERNEL_SYNTH = 0, 1, 2
HOP_LOSS_HINGE, HOP_LOSS_LOG = 0, 1
HOP_TICKS_NEVER = 1 << 62

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libhop.so")

EXPORTS = [
    "hop_strerror", "hop_version", "hop_opts_default", "hop_layout", "hop_arena_bytes", "hop_init",
    "hop_destroy", "hop_set_params", "hop_set_rows", "hop_set_data_dense", "hop_set_data_csr",
    "hop_set_grad_source", "hop_simulate", "hop_schedule_view", "hop_schedule_free", "hop_step",
    "hop_params", "hop_slot", "hop_coef", "hop_profile", "hop_profile_read", "hop_mix",
    "hop_grad_scratch_floats", "hop_svm_grad_dense", "hop_svm_grad_csr", "hop_synth_grad", "hop_copy",
    "hop_download", "hop_use_graph", "hop_schedule_bytes", "hop_schedule_bind",
    "hop_svm_grad_dense_static",
]


class HopError(RuntimeError):
    def __init__(self, code, what):
        super().__init__("%s failed: %s (%d)" % (what, _strerror(code), code))
        self.code = code


class hop_graph(C.Structure):
    _fields_ = [("N", C.c_int32), ("row_ptr", C.POINTER(C.c_int32)), ("col", C.POINTER(C.c_int32))]


class hop_device(C.Structure):
    _fields_ = [("arena", C.c_void_p), ("arena_bytes", C.c_size_t), ("hip_stream", C.c_void_p)]


class hop_opts(C.Structure):
    _fields_ = [("max_ig", C.c_int32), ("skip_on", C.c_int32), ("max_skip", C.c_int32),
                ("trigger", C.c_int32), ("lr", C.c_float), ("lambda_", C.c_float),
                ("batch", C.c_int32), ("loss", C.c_int32), ("seed", C.c_uint64),
                ("momentum", C.c_float), ("max_latency", C.c_uint32), ("serial", C.c_int32),
                ("notify_ack", C.c_int32), ("grad_ahead", C.c_int32)]


class hop_delay_model(C.Structure):
    _fields_ = [("kind", C.c_int32), ("table_iters", C.c_int32), ("mult", C.POINTER(C.c_double)),
                ("table", C.POINTER(C.c_uint64))]


_I32P, _U64P, _F32P = C.POINTER(C.c_int32), C.POINTER(C.c_uint64), C.POINTER(C.c_float)


class hop_schedule_arrays(C.Structure):
    _fields_ = [("n_records", C.c_int32), ("n_sources", C.c_int32), ("n_waves", C.c_int32),
                ("n_workers", C.c_int32), ("depth", C.c_int32), ("batch", C.c_int32),
                ("stalled", C.c_int32), ("n_jumps", C.c_int32), ("late_sends", C.c_int32),
                ("reserved", C.c_int32),
                ("kind", _I32P), ("worker", _I32P), ("iter", _I32P), ("time", _U64P), ("wave", _I32P),
                ("out_slot", _I32P), ("src_begin", _I32P), ("src_worker", _I32P), ("src_tag", _I32P),
                ("src_slot", _I32P), ("src_weight", _F32P), ("batch_rows", _I32P),
                ("final_iter", _I32P), ("finish_time", _U64P), ("wave_begin", _I32P),
                ("wave_order", _I32P)]


class hop_mix_job(C.Structure):
    _fields_ = [("out", C.c_void_p), ("g", C.c_void_p), ("eta", C.c_float), ("A", C.c_int32),
                ("src", C.c_void_p * HOP_MAX_A), ("w", C.c_float * HOP_MAX_A),
                ("vel", C.c_void_p), ("mu", C.c_float)]


_lib = None


def load():
    """Loads libhop.so (after torch, so that both share one HIP runtime)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError("libhop.so is not built: run `python -m paper_1902_01064_amd.build` "
                          "(there is no fallback path)")
    try:
        import torch  # noqa: F401  (brings in the HIP runtime the library binds to)
    except ImportError:
        pass
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_float
    sig = {
        "hop_strerror": (C.c_char_p, [C.c_int]),
        "hop_version": (C.c_int, []),
        "hop_opts_default": (C.c_int, [C.POINTER(hop_opts)]),
        "hop_layout": (C.c_int, [i64, i32, C.POINTER(hop_opts), C.POINTER(i32), C.POINTER(i64)]),
        "hop_arena_bytes": (C.c_size_t, [i32, i64, i32, i32, C.POINTER(hop_opts)]),
        "hop_init": (C.c_int, [C.POINTER(vp), C.POINTER(hop_graph), _F32P, i32, i64, i32, i32,
                               C.POINTER(hop_opts), C.POINTER(hop_device)]),
        "hop_destroy": (C.c_int, [vp]),
        "hop_set_params": (C.c_int, [vp, vp, C.c_int, C.c_int]),
        "hop_set_rows": (C.c_int, [vp, i32, i64]),
        "hop_set_data_dense": (C.c_int, [vp, i32, vp, vp, i64]),
        "hop_set_data_csr": (C.c_int, [vp, i32, vp, vp, vp, vp, i64]),
        "hop_set_grad_source": (C.c_int, [vp, C.c_int, f32, vp]),
        "hop_simulate": (C.c_int, [vp, C.POINTER(hop_delay_model), i32, C.POINTER(vp)]),
        "hop_schedule_view": (C.c_int, [vp, C.POINTER(hop_schedule_arrays)]),
        "hop_schedule_free": (C.c_int, [vp]),
        "hop_schedule_bytes": (C.c_size_t, [vp]),
        "hop_schedule_bind": (C.c_int, [vp, vp, vp, C.c_size_t]),
        "hop_step": (C.c_int, [vp, vp, i32, i32]),
        "hop_params": (C.c_int, [vp, i32, C.POINTER(vp), C.POINTER(i32)]),
        "hop_slot": (C.c_int, [vp, i32, i32, C.POINTER(vp)]),
        "hop_coef": (C.c_int, [vp, vp, i32, C.POINTER(vp)]),
        "hop_profile": (C.c_int, [vp, C.c_int]),
        "hop_use_graph": (C.c_int, [vp, C.c_int]),
        "hop_profile_read": (C.c_int, [vp, C.c_int, C.POINTER(C.c_double), C.POINTER(i64),
                                       C.POINTER(C.c_double)]),
        "hop_mix": (C.c_int, [C.POINTER(hop_mix_job), i32, i64, vp]),
        "hop_grad_scratch_floats": (i64, [i64, i32]),
        "hop_svm_grad_dense": (C.c_int, [vp, vp, vp, vp, i32, i64, f32, i32, vp, vp, vp, vp]),
        "hop_svm_grad_dense_static": (C.c_int, [vp, vp, vp, vp, i32, i64, f32, i32, vp, vp, vp]),
        "hop_svm_grad_csr": (C.c_int, [vp, vp, vp, vp, vp, vp, i32, i64, f32, i32, vp, vp, vp]),
        "hop_synth_grad": (C.c_int, [C.c_uint64, i32, i32, f32, vp, i64, vp]),
        "hop_copy": (C.c_int, [vp, vp, C.c_size_t, vp]),
        "hop_download": (C.c_int, [vp, vp, C.c_size_t, vp]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    _lib = lib
    return lib


def _strerror(code):
    try:
        return load().hop_strerror(code).decode()
    except Exception:
        return "error"


def _check(code, what, allow=()):
    if code < 0 and code not in allow:
        raise HopError(code, what)
    return code


def _np_i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def make_opts(max_ig=0, skip_on=False, max_skip=10, trigger=1, lr=0.01, lam=1e-4, batch=0, seed=0,
              loss=HOP_LOSS_HINGE, momentum=0.0, max_latency=0, serial=False, notify_ack=False, grad_ahead=1):
    o = hop_opts()
    _check(load().hop_opts_default(C.byref(o)), "hop_opts_default")
    o.max_ig, o.skip_on, o.max_skip, o.trigger = int(max_ig), int(bool(skip_on)), int(max_skip), int(trigger)
    o.lr, o.lambda_, o.batch, o.seed = float(lr), float(lam), int(batch), int(seed)
    o.loss, o.momentum, o.max_latency = int(loss), float(momentum), int(max_latency)
    o.serial, o.notify_ack, o.grad_ahead = int(bool(serial)), int(bool(notify_ack)), int(grad_ahead)
    return o


def hop_version():
    return load().hop_version()


def hop_strerror(code):
    return _strerror(code)


def hop_layout(d, s, opts):
    depth, stride = C.c_int32(), C.c_int64()
    _check(load().hop_layout(d, s, C.byref(opts), C.byref(depth), C.byref(stride)), "hop_layout")
    return depth.value, stride.value


def hop_arena_bytes(N, d, s, b, opts):
    return load().hop_arena_bytes(N, d, s, b, C.byref(opts))


def hop_init(row_ptr, col, W, N, d, s, b, opts=None, arena_ptr=None, arena_bytes=0, stream=0):
    """Returns the context handle.  arena_ptr None = host-only context."""
    lib = load()
    row_ptr, col = _np_i32(row_ptr), _np_i32(col)
    W = np.ascontiguousarray(W, dtype=np.float32)
    g = hop_graph(int(N), row_ptr.ctypes.data_as(_I32P), col.ctypes.data_as(_I32P))
    dev = None
    if arena_ptr is not None:
        dev = C.byref(hop_device(C.c_void_p(arena_ptr), arena_bytes, C.c_void_p(stream)))
    ctx = C.c_void_p()
    _check(lib.hop_init(C.byref(ctx), C.byref(g), W.ctypes.data_as(_F32P), N, d, s, b,
                        C.byref(opts) if opts is not None else None, dev), "hop_init")
    return ctx


def hop_destroy(ctx):
    _check(load().hop_destroy(ctx), "hop_destroy")


def hop_set_params(ctx, p0_ptr, per_worker, on_device):
    _check(load().hop_set_params(ctx, C.c_void_p(p0_ptr), int(per_worker), int(on_device)), "hop_set_params")


def hop_set_rows(ctx, worker, rows):
    _check(load().hop_set_rows(ctx, worker, rows), "hop_set_rows")


def hop_set_data_dense(ctx, worker, X_ptr, y_ptr, rows):
    _check(load().hop_set_data_dense(ctx, worker, C.c_void_p(X_ptr), C.c_void_p(y_ptr), rows),
           "hop_set_data_dense")


def hop_set_data_csr(ctx, worker, rowptr_ptr, col_ptr, val_ptr, y_ptr, rows):
    _check(load().hop_set_data_csr(ctx, worker, C.c_void_p(rowptr_ptr), C.c_void_p(col_ptr),
                                   C.c_void_p(val_ptr), C.c_void_p(y_ptr), rows), "hop_set_data_csr")


def hop_set_grad_source(ctx, mode, variance=0.0, external_ptr=None):
    _check(load().hop_set_grad_source(ctx, mode, variance,
                                      C.c_void_p(external_ptr) if external_ptr else None),
           "hop_set_grad_source")


class Schedule:
    """Handle plus numpy views of hop_schedule_arrays (views die with the handle)."""

    def __init__(self, handle, rc):
        self.handle, self.rc = handle, rc
        v = hop_schedule_arrays()
        _check(load().hop_schedule_view(handle, C.byref(v)), "hop_schedule_view")
        self.view = v
        R, S, Wv, N = v.n_records, v.n_sources, v.n_waves, v.n_workers
        self.n_records, self.n_sources, self.n_waves, self.n_workers = R, S, Wv, N
        self.depth, self.batch, self.stalled, self.n_jumps = v.depth, v.batch, bool(v.stalled), v.n_jumps
        self.late_sends = v.late_sends

        def arr(p, n, dt):
            if n == 0 or not p:
                return np.zeros(0, dtype=dt)
            return np.ctypeslib.as_array(p, shape=(n,))
        for name in ("kind", "worker", "iter", "wave", "out_slot"):
            setattr(self, name, arr(getattr(v, name), R, np.int32))
        self.time = arr(v.time, R, np.uint64)
        self.src_begin = arr(v.src_begin, R + 1, np.int32)
        for name in ("src_worker", "src_tag", "src_slot"):
            setattr(self, name, arr(getattr(v, name), S, np.int32))
        self.src_weight = arr(v.src_weight, S, np.float32)
        self.batch_rows = arr(v.batch_rows, R * v.batch, np.int32).reshape(R, v.batch) if v.batch else None
        self.final_iter = arr(v.final_iter, N, np.int32)
        self.finish_time = arr(v.finish_time, N, np.uint64)
        self.wave_begin = arr(v.wave_begin, Wv + 1, np.int32)
        self.wave_order = arr(v.wave_order, R, np.int32)

    def free(self):
        if self.handle is not None:
            _check(load().hop_schedule_free(self.handle), "hop_schedule_free")
            self.handle = None


def hop_simulate(ctx, max_iter, kind=HOP_DELAY_NONE, mult=None, table=None):
    """Returns a Schedule; a stall (HOP_ERR_DEADLOCK) is reported in .stalled, not raised."""
    dm = hop_delay_model()
    dm.kind = int(kind)
    keep = []
    if mult is not None:
        m = np.ascontiguousarray(mult, dtype=np.float64)
        keep.append(m)
        dm.mult = m.ctypes.data_as(C.POINTER(C.c_double))
    if table is not None:
        t = np.ascontiguousarray(table, dtype=np.uint64)
        keep.append(t)
        dm.table = t.ctypes.data_as(_U64P)
        dm.table_iters = t.shape[1]
    h = C.c_void_p()
    rc = _check(load().hop_simulate(ctx, C.byref(dm), max_iter, C.byref(h)), "hop_simulate",
                allow=(HOP_ERR_DEADLOCK,))
    return Schedule(h, rc)


def hop_schedule_free(sched):
    sched.free()


def hop_schedule_bytes(sched):
    return load().hop_schedule_bytes(sched.handle)


def hop_schedule_bind(ctx, sched, workspace_ptr, nbytes):
    _check(load().hop_schedule_bind(ctx, sched.handle, C.c_void_p(workspace_ptr), nbytes), "hop_schedule_bind")


def hop_step(ctx, sched, wave_begin=0, wave_end=-1):
    _check(load().hop_step(ctx, sched.handle, wave_begin, wave_end), "hop_step")


def hop_params(ctx, worker):
    p, it = C.c_void_p(), C.c_int32()
    _check(load().hop_params(ctx, worker, C.byref(p), C.byref(it)), "hop_params")
    return p.value, it.value


def hop_slot(ctx, worker, slot):
    p = C.c_void_p()
    _check(load().hop_slot(ctx, worker, slot, C.byref(p)), "hop_slot")
    return p.value


def hop_coef(ctx, sched, record):
    p = C.c_void_p()
    _check(load().hop_coef(ctx, sched.handle, record, C.byref(p)), "hop_coef")
    return p.value


def hop_use_graph(ctx, enable):
    _check(load().hop_use_graph(ctx, int(enable)), "hop_use_graph")


def hop_profile(ctx, enable):
    _check(load().hop_profile(ctx, int(enable)), "hop_profile")


def hop_profile_read(ctx, kernel):
    ms, n, by = C.c_double(), C.c_int64(), C.c_double()
    _check(load().hop_profile_read(ctx, kernel, C.byref(ms), C.byref(n), C.byref(by)), "hop_profile_read")
    return ms.value, n.value, by.value


def hop_mix(jobs, d, stream=0):
    """jobs: list of dicts {out, g (or None), eta, src: [ptr...], w: [float...]} (device pointers)."""
    arr = (hop_mix_job * len(jobs))()
    for j, job in enumerate(jobs):
        arr[j].out = job["out"]
        arr[j].g = job.get("g") or None
        arr[j].eta = float(job.get("eta", 0.0))
        arr[j].A = len(job["src"])
        arr[j].vel = job.get("vel") or None
        arr[j].mu = float(job.get("mu", 0.0))
        for a, (p, w) in enumerate(zip(job["src"], job["w"])):
            if a < HOP_MAX_A:
                arr[j].src[a] = p
                arr[j].w[a] = float(w)
    _check(load().hop_mix(arr, len(jobs), d, C.c_void_p(stream)), "hop_mix")


def hop_grad_scratch_floats(d, B):
    return load().hop_grad_scratch_floats(d, B)


def hop_svm_grad_dense(X, y, w, rows, B, d, lam, g, coef, scratch, stream=0, loss=HOP_LOSS_HINGE):
    _check(load().hop_svm_grad_dense(X, y, w, rows, B, d, lam, loss, g, coef, scratch, C.c_void_p(stream)),
           "hop_svm_grad_dense")


def hop_svm_grad_dense_static(X, y, w, rows, B, d, lam, g, coef, stream=0, loss=HOP_LOSS_HINGE):
    _check(load().hop_svm_grad_dense_static(X, y, w, rows, B, d, lam, loss, g, coef, C.c_void_p(stream)),
           "hop_svm_grad_dense_static")


def hop_svm_grad_csr(rowptr, col, val, y, w, rows, B, d, lam, g, coef, stream=0, loss=HOP_LOSS_HINGE):
    _check(load().hop_svm_grad_csr(rowptr, col, val, y, w, rows, B, d, lam, loss, g, coef, C.c_void_p(stream)),
           "hop_svm_grad_csr")


def hop_synth_grad(seed, worker, it, variance, g, d, stream=0):
    _check(load().hop_synth_grad(seed, worker, it, variance, g, d, C.c_void_p(stream)), "hop_synth_grad")


def hop_copy(dst, src, nbytes, stream=0):
    _check(load().hop_copy(dst, src, nbytes, C.c_void_p(stream)), "hop_copy")


def hop_download(dev_ptr, n_floats, stream=0):
    """n_floats fp32 values at a device address, as a numpy array."""
    out = np.empty(n_floats, dtype=np.float32)
    _check(load().hop_download(out.ctypes.data_as(C.c_void_p), C.c_void_p(dev_ptr), n_floats * 4,
                               C.c_void_p(stream)), "hop_download")
    return out
