"""ctypes binding of the C-ABI library (include/sgemm_tuned.h): argument marshalling only.
Every function has the name of the C entry point it calls.  PyTorch appears only where a
caller passes tensors: their data_ptr() and the current HIP stream are handed to the library.

The library must have been built (paper_1703_06503_amd/build.py); loading fails loudly
otherwise, and there is no fallback path of any kind."""
import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "lib", "libsgemm_tuned.so")

OK = 0
E_BADARG, E_NOCONFIG, E_COMPILE, E_LAUNCH, E_VERIFY = -1, -2, -3, -4, -5
E_INVALID, E_IO, E_NODEVICE, E_RESOURCE, E_NOTREADY = -6, -7, -8, -9, -10
LAYOUT_A_TRANSPOSED, LAYOUT_B_TRANSPOSED = 1, 2
STRATEGY_FULL, STRATEGY_RANDOM, STRATEGY_ANNEALING, STRATEGY_PSO = 0, 1, 2, 3
SPACE_FULL, SPACE_SMALL, SPACE_MFMA, SPACE_EXT, SPACE_DIRECT, SPACE_CUSTOM, SPACE_KSPLIT = 0, 1, 2, 3, 4, 5, 6
BUILD_GUARDED, BUILD_READS_C_AHEAD = 1, 2          # flags of sgemm_kernel_compile / _resolve
NOALLOC_SCRATCH_BYTES = 32 << 20

CONFIG_FIELDS = ("mwg", "nwg", "kwg", "mdimc", "ndimc", "vwm", "vwn", "sa", "sb", "pad", "kwi",
                 "mfma", "grp", "sk", "ns", "ksw")


class sgemm_config(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int) for n in CONFIG_FIELDS]

    def as_tuple(self):
        return tuple(getattr(self, n) for n in CONFIG_FIELDS)

    def as_dict(self):
        return {n: getattr(self, n) for n in CONFIG_FIELDS}

    def __repr__(self):
        return "sgemm_config(" + ", ".join(f"{n}={getattr(self, n)}" for n in CONFIG_FIELDS) + ")"


def make_config(*args, **kw):
    """sgemm_config from positional values in field order (the last three, sk, ns and ksw, may
    be left out from the right and are then 1, 2 and 1), or from keywords."""
    c = sgemm_config()
    c.sk, c.ns, c.ksw = 1, 2, 1
    if args:
        tail = (1, 2, 1)
        missing = len(CONFIG_FIELDS) - len(args)
        if not 0 <= missing <= 3:
            raise ValueError("expected %d to %d values" % (len(CONFIG_FIELDS) - 3, len(CONFIG_FIELDS)))
        args = tuple(args) + tail[3 - missing:]
        kw = dict(zip(CONFIG_FIELDS, args))
    for k, v in kw.items():
        if k not in CONFIG_FIELDS:
            raise ValueError(f"unknown field {k}")
        setattr(c, k, int(v))
    return c


class sgemm_kernel_info(ctypes.Structure):
    _fields_ = [("vgprs", ctypes.c_int), ("agprs", ctypes.c_int), ("sgprs", ctypes.c_int),
                ("lds_bytes", ctypes.c_int), ("scratch_bytes", ctypes.c_int),
                ("code_bytes", ctypes.c_int), ("from_cache", ctypes.c_int),
                ("compile_ms", ctypes.c_float)]


class tune_opts(ctypes.Structure):
    _fields_ = [("space", ctypes.c_int), ("warmup", ctypes.c_int), ("reps", ctypes.c_int),
                ("verify_off", ctypes.c_int), ("cut_factor", ctypes.c_float),
                ("warmup_ms", ctypes.c_float),
                ("sa_T", ctypes.c_float), ("sa_raw_ms", ctypes.c_int), ("pso_S", ctypes.c_int),
                ("pso_alpha", ctypes.c_float), ("pso_beta", ctypes.c_float),
                ("pso_gamma", ctypes.c_float), ("random_fraction", ctypes.c_float),
                ("A", ctypes.c_void_p), ("B", ctypes.c_void_p), ("C", ctypes.c_void_p),
                ("C0", ctypes.c_void_p), ("lda", ctypes.c_int), ("ldb", ctypes.c_int),
                ("ldc", ctypes.c_int), ("log_path", ctypes.c_char_p),
                ("warm_start", ctypes.c_int), ("reserved", ctypes.c_int * 7)]


class tune_result(ctypes.Structure):
    _fields_ = [("best", sgemm_config), ("best_ms", ctypes.c_float),
                ("best_gflops", ctypes.c_float), ("best_index", ctypes.c_int),
                ("evaluations", ctypes.c_int), ("failed", ctypes.c_int),
                ("space_size", ctypes.c_int), ("evals_to_best", ctypes.c_int),
                ("total_ms", ctypes.c_float), ("compile_ms", ctypes.c_float),
                ("reserved", ctypes.c_int * 6)]


CONV_FIELDS = ("xwg", "ywg", "xwpt", "ywpt", "lmem", "vw", "pad", "unr")


class conv2d_config(ctypes.Structure):
    """include/conv2d_tuned.h: one configuration of the convolution kernel family."""
    _fields_ = [(n, ctypes.c_int) for n in CONV_FIELDS]

    def as_tuple(self):
        return tuple(getattr(self, n) for n in CONV_FIELDS)

    def __repr__(self):
        return "conv2d_config(" + ", ".join(f"{n}={getattr(self, n)}" for n in CONV_FIELDS) + ")"


def make_conv_config(*args):
    if len(args) != len(CONV_FIELDS):
        raise ValueError("expected %d values" % len(CONV_FIELDS))
    c = conv2d_config()
    for n, v in zip(CONV_FIELDS, args):
        setattr(c, n, int(v))
    return c


class conv2d_tune_result(ctypes.Structure):
    _fields_ = [("best", conv2d_config), ("best_ms", ctypes.c_float),
                ("best_gflops", ctypes.c_float), ("best_gbs", ctypes.c_float),
                ("best_index", ctypes.c_int), ("evaluations", ctypes.c_int),
                ("failed", ctypes.c_int), ("space_size", ctypes.c_int),
                ("evals_to_best", ctypes.c_int), ("total_ms", ctypes.c_float),
                ("compile_ms", ctypes.c_float), ("reserved", ctypes.c_int * 4)]


class ktuner_result(ctypes.Structure):
    _fields_ = [("best_index", ctypes.c_int), ("best_ms", ctypes.c_float),
                ("evaluations", ctypes.c_int), ("failed", ctypes.c_int),
                ("space_size", ctypes.c_int), ("evals_to_best", ctypes.c_int),
                ("failed_verify", ctypes.c_int), ("total_ms", ctypes.c_float),
                ("compile_ms", ctypes.c_float), ("reserved", ctypes.c_int * 7)]


KTUNER_CONSTRAINT = ctypes.CFUNCTYPE(ctypes.c_int, ctypes.POINTER(ctypes.c_int), ctypes.c_void_p)


EXPORTS = (
    "sgemm_tuned", "sgemm_tuned_on", "sgemm_tuned_noalloc", "sgemm_tuned_online", "sgemm_set_stream", "sgemm_run_config",
    "sgemm_run_config_padded", "sgemm_config_prefers_padding", "sgemm_reference",
    "tune", "tune_ex", "tune_replay", "sgemm_space_define_custom", "sgemm_space_size", "sgemm_space_raw_size",
    "sgemm_space_get", "sgemm_space_find", "sgemm_space_dims", "sgemm_space_values",
    "sgemm_config_check", "sgemm_config_lds_bytes", "sgemm_config_default",
    "sgemm_config_workspace_bytes",
    "sgemm_kernel_cache_dir", "sgemm_kernel_compile", "sgemm_kernel_resolve", "sgemm_kernel_macros",
    "sgemm_kernel_cache_path", "sgemm_config_get",
    "sgemm_config_set", "sgemm_config_select", "sgemm_cache_load", "sgemm_cache_save",
    "sgemm_cache_clear", "sgemm_cache_count", "sgemm_device_peak", "sgemm_status_string",
    "sgemm_last_error",
    # include/conv2d_tuned.h
    "conv2d_space_size", "conv2d_space_get", "conv2d_space_find", "conv2d_config_check",
    "conv2d_config_lds_bytes", "conv2d_config_threads", "conv2d_kernel_compile",
    "conv2d_run_config", "conv2d_reference", "conv2d_tuned", "conv2d_config_set",
    "conv2d_config_select", "conv2d_tune", "conv2d_tune_replay", "conv2d_cache_save",
    "conv2d_cache_load", "conv2d_cache_clear",
    # include/kernel_tuner.h
    "ktuner_create", "ktuner_destroy", "ktuner_add_parameter", "ktuner_mul_global_size",
    "ktuner_div_global_size", "ktuner_mul_local_size", "ktuner_div_local_size",
    "ktuner_add_constraint", "ktuner_add_argument_input", "ktuner_add_argument_output",
    "ktuner_add_argument_int", "ktuner_add_argument_float", "ktuner_set_reference",
    "ktuner_set_tolerance", "ktuner_space_size", "ktuner_space_get", "ktuner_compile",
    "ktuner_launch_shape", "ktuner_tune", "ktuner_time_of", "ktuner_read_output",
)

_lib = None


def lib():
    """The loaded shared library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_1703_06503_amd.build` "
                               "(there is no fallback implementation)")
        # One HIP runtime per process: the device pointers and streams handed to the library
        # come from PyTorch, so the library must resolve libamdhip64 / libhiprtc to the copies
        # PyTorch bundles (same SONAMEs as the system ones) rather than load a second runtime.
        import torch
        torch_lib = os.path.join(os.path.dirname(torch.__file__), "lib")
        for name in ("libamdhip64.so", "libhiprtc.so"):
            path = os.path.join(torch_lib, name)
            if os.path.exists(path):
                ctypes.CDLL(path, mode=ctypes.RTLD_GLOBAL)
        L = ctypes.CDLL(LIB_PATH)
        i, f, vp = ctypes.c_int, ctypes.c_float, ctypes.c_void_p
        cfgp = ctypes.POINTER(sgemm_config)
        gemm = [i, i, i, f, vp, i, vp, i, f, vp, i, i]
        L.sgemm_tuned.argtypes = gemm
        L.sgemm_tuned_on.argtypes = [vp] + gemm
        L.sgemm_tuned_noalloc.argtypes = [vp] + gemm
        L.sgemm_tuned_online.argtypes = [vp] + gemm + [i, i, i]
        L.sgemm_set_stream.argtypes = [vp]
        L.sgemm_run_config.argtypes = [vp, cfgp] + gemm
        L.sgemm_run_config_padded.argtypes = [vp, cfgp] + gemm
        L.sgemm_config_prefers_padding.argtypes = [cfgp, i, i, i, i, i, i, i, f]
        L.sgemm_reference.argtypes = [vp] + gemm
        L.tune.argtypes = [i, i, i, i, i]
        L.tune_ex.argtypes = [i, i, i, i, f, f, i, i, ctypes.c_ulonglong,
                              ctypes.POINTER(tune_opts), ctypes.POINTER(tune_result)]
        L.tune_replay.argtypes = [i, ctypes.POINTER(f), i, i, i, ctypes.c_ulonglong,
                                  ctypes.POINTER(tune_opts), ctypes.POINTER(i), i,
                                  ctypes.POINTER(tune_result)]
        L.sgemm_space_define_custom.argtypes = [ctypes.c_char_p]
        L.sgemm_space_size.argtypes = [i]
        L.sgemm_space_raw_size.argtypes = [i]
        L.sgemm_space_raw_size.restype = ctypes.c_longlong
        L.sgemm_space_get.argtypes = [i, i, cfgp]
        L.sgemm_space_find.argtypes = [i, cfgp]
        L.sgemm_space_dims.argtypes = [i]
        L.sgemm_space_values.argtypes = [i, i, ctypes.POINTER(i), i]
        L.sgemm_config_check.argtypes = [cfgp]
        L.sgemm_config_lds_bytes.argtypes = [cfgp]
        L.sgemm_config_default.argtypes = [i, i, i, i, cfgp]
        L.sgemm_kernel_cache_dir.argtypes = [ctypes.c_char_p]
        L.sgemm_kernel_compile.argtypes = [cfgp, i, i, ctypes.POINTER(sgemm_kernel_info)]
        L.sgemm_kernel_macros.argtypes = [cfgp, i, i, ctypes.c_char_p, i]
        L.sgemm_kernel_resolve.argtypes = [cfgp, i, i, i, i, i, i, i, ctypes.c_float, cfgp, ctypes.POINTER(i)]
        L.sgemm_config_get.argtypes = [i, i, i, i, cfgp]
        L.sgemm_config_set.argtypes = [i, i, i, i, cfgp, f]
        L.sgemm_config_select.argtypes = [i, i, i, i, cfgp]
        L.sgemm_cache_load.argtypes = [ctypes.c_char_p]
        L.sgemm_cache_save.argtypes = [ctypes.c_char_p]
        L.sgemm_cache_clear.argtypes = []
        L.sgemm_cache_count.argtypes = []
        L.sgemm_device_peak.argtypes = [ctypes.POINTER(f), ctypes.POINTER(i), ctypes.POINTER(i)]
        L.sgemm_status_string.argtypes = [i]
        L.sgemm_status_string.restype = ctypes.c_char_p
        L.sgemm_last_error.argtypes = []
        L.sgemm_last_error.restype = ctypes.c_char_p
        ccfgp = ctypes.POINTER(conv2d_config)
        conv = [i, i, i, i, f, vp, vp, i, vp, i]      # X Y Xf Yf w F A lda B ldb
        L.conv2d_space_size.argtypes = [i, i]
        L.conv2d_space_get.argtypes = [i, i, i, ccfgp]
        L.conv2d_space_find.argtypes = [i, i, ccfgp]
        L.conv2d_config_check.argtypes = [ccfgp, i, i]
        L.conv2d_config_lds_bytes.argtypes = [ccfgp, i, i]
        L.conv2d_config_threads.argtypes = [ccfgp, i, i]
        L.conv2d_kernel_compile.argtypes = [ccfgp, i, i, i, i, ctypes.POINTER(sgemm_kernel_info)]
        L.conv2d_run_config.argtypes = [vp, ccfgp] + conv
        L.conv2d_reference.argtypes = [vp] + conv
        L.conv2d_tuned.argtypes = conv
        L.conv2d_config_set.argtypes = [i, i, i, i, ccfgp, f]
        L.conv2d_config_select.argtypes = [i, i, i, i, ccfgp]
        L.conv2d_cache_save.argtypes = [ctypes.c_char_p]
        L.conv2d_cache_load.argtypes = [ctypes.c_char_p]
        L.conv2d_cache_clear.argtypes = []
        L.conv2d_tune.argtypes = [i, i, i, i, f, i, i, ctypes.c_ulonglong,
                                  ctypes.POINTER(tune_opts), ctypes.POINTER(conv2d_tune_result)]
        L.conv2d_tune_replay.argtypes = [i, i, ctypes.POINTER(f), i, i, i, ctypes.c_ulonglong,
                                         ctypes.POINTER(tune_opts), ctypes.POINTER(i), i,
                                         ctypes.POINTER(conv2d_tune_result)]
        i3 = ctypes.POINTER(ctypes.c_int)
        names3 = ctypes.POINTER(ctypes.c_char_p)
        L.ktuner_create.argtypes = [ctypes.c_char_p, ctypes.c_char_p, i3, i3]
        L.ktuner_create.restype = vp
        L.ktuner_destroy.argtypes = [vp]
        L.ktuner_destroy.restype = None
        L.ktuner_add_parameter.argtypes = [vp, ctypes.c_char_p, i3, i]
        for fn in (L.ktuner_mul_global_size, L.ktuner_div_global_size, L.ktuner_mul_local_size,
                   L.ktuner_div_local_size):
            fn.argtypes = [vp, names3]
        L.ktuner_add_constraint.argtypes = [vp, KTUNER_CONSTRAINT, names3, i, vp]
        L.ktuner_add_argument_input.argtypes = [vp, vp, ctypes.c_size_t]
        L.ktuner_add_argument_output.argtypes = [vp, vp, ctypes.c_size_t]
        L.ktuner_add_argument_int.argtypes = [vp, i]
        L.ktuner_add_argument_float.argtypes = [vp, f]
        L.ktuner_set_reference.argtypes = [vp, ctypes.c_char_p, ctypes.c_char_p, i3, i3]
        L.ktuner_set_tolerance.argtypes = [vp, f, f]
        L.ktuner_space_size.argtypes = [vp]
        L.ktuner_space_get.argtypes = [vp, i, i3]
        L.ktuner_compile.argtypes = [vp, i, ctypes.POINTER(sgemm_kernel_info)]
        L.ktuner_launch_shape.argtypes = [vp, i, i3, i3]
        L.ktuner_tune.argtypes = [vp, i, i, ctypes.c_ulonglong, ctypes.POINTER(tune_opts),
                                  ctypes.POINTER(ktuner_result)]
        L.ktuner_time_of.argtypes = [vp, i]
        L.ktuner_time_of.restype = f
        L.ktuner_read_output.argtypes = [vp, i, vp, ctypes.c_size_t]
        _lib = L
    return _lib


class SgemmError(RuntimeError):
    def __init__(self, status, what, message=None):
        self.status = status
        self.what = what
        if message is None:
            detail = sgemm_last_error()
            message = f"{what}: {sgemm_status_string(status)} ({status})" + (f": {detail}" if detail else "")
        super().__init__(message)

    def __reduce__(self):       # travels between processes (worker pools) with its text
        return (SgemmError, (self.status, self.what, str(self)))


def _check(status, what):
    if status < 0:
        raise SgemmError(status, what)
    return status


def sgemm_status_string(status):
    return lib().sgemm_status_string(int(status)).decode()


def sgemm_last_error():
    return lib().sgemm_last_error().decode(errors="replace")


def _ptr(t):
    """Device address of a torch tensor (or a raw int / None)."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def sgemm_tuned(M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, layout=0):
    return _check(lib().sgemm_tuned(M, N, K, alpha, _ptr(A), lda, _ptr(B), ldb, beta, _ptr(C),
                                    ldc, layout), "sgemm_tuned")


def sgemm_tuned_on(stream, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, layout=0):
    return _check(lib().sgemm_tuned_on(_stream(stream), M, N, K, alpha, _ptr(A), lda, _ptr(B),
                                       ldb, beta, _ptr(C), ldc, layout), "sgemm_tuned_on")


def sgemm_tuned_prepare(stream, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, layout=0, noalloc=False):
    """A callable that repeats this sgemm_tuned_on() (or sgemm_tuned_noalloc()) call with its
    arguments marshalled once: the stream handle and the device addresses are read now, so the
    tensors must stay alive and in place.  For loops in which the microseconds that looking
    them up costs per call would show (kernels of a few microseconds)."""
    fn = lib().sgemm_tuned_noalloc if noalloc else lib().sgemm_tuned_on
    what = "sgemm_tuned_noalloc" if noalloc else "sgemm_tuned_on"
    args = (ctypes.c_void_p(_stream(stream)), ctypes.c_int(M), ctypes.c_int(N), ctypes.c_int(K),
            ctypes.c_float(alpha), ctypes.c_void_p(_ptr(A)), ctypes.c_int(lda), ctypes.c_void_p(_ptr(B)),
            ctypes.c_int(ldb), ctypes.c_float(beta), ctypes.c_void_p(_ptr(C)), ctypes.c_int(ldc),
            ctypes.c_int(layout))

    def call():
        status = fn(*args)
        if status < 0:
            raise SgemmError(status, what)
        return status
    return call


def sgemm_tuned_noalloc(stream, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, layout=0):
    return _check(lib().sgemm_tuned_noalloc(_stream(stream), M, N, K, alpha, _ptr(A), lda, _ptr(B),
                                            ldb, beta, _ptr(C), ldc, layout), "sgemm_tuned_noalloc")


def sgemm_tuned_online(stream, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, layout=0,
                       space=SPACE_MFMA, strategy=STRATEGY_ANNEALING, budget=32):
    return _check(lib().sgemm_tuned_online(_stream(stream), M, N, K, alpha, _ptr(A), lda, _ptr(B),
                                           ldb, beta, _ptr(C), ldc, layout, space, strategy, budget),
                  "sgemm_tuned_online")


def sgemm_set_stream(stream):
    return _check(lib().sgemm_set_stream(_stream(stream)), "sgemm_set_stream")


def sgemm_run_config(stream, cfg, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, layout=0):
    return _check(lib().sgemm_run_config(_stream(stream), ctypes.byref(cfg), M, N, K, alpha,
                                         _ptr(A), lda, _ptr(B), ldb, beta, _ptr(C), ldc, layout),
                  "sgemm_run_config")


def sgemm_run_config_padded(stream, cfg, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, layout=0):
    return _check(lib().sgemm_run_config_padded(_stream(stream), ctypes.byref(cfg), M, N, K, alpha,
                                                _ptr(A), lda, _ptr(B), ldb, beta, _ptr(C), ldc,
                                                layout), "sgemm_run_config_padded")


def sgemm_config_prefers_padding(cfg, M, N, K, lda, ldb, ldc, layout=0, beta=0.0):
    return _check(lib().sgemm_config_prefers_padding(ctypes.byref(cfg), M, N, K, lda, ldb, ldc, layout,
                                                     beta), "sgemm_config_prefers_padding")


def sgemm_reference(stream, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, layout=0):
    return _check(lib().sgemm_reference(_stream(stream), M, N, K, alpha, _ptr(A), lda, _ptr(B),
                                        ldb, beta, _ptr(C), ldc, layout), "sgemm_reference")


def tune(M, N, K, strategy, budget):
    return _check(lib().tune(M, N, K, strategy, budget), "tune")


def tune_ex(M, N, K, layout, alpha, beta, strategy, budget, seed=0, opts=None):
    """Returns (evaluations, tune_result)."""
    res = tune_result()
    n = _check(lib().tune_ex(M, N, K, layout, alpha, beta, strategy, budget, seed,
                             ctypes.byref(opts) if opts is not None else None,
                             ctypes.byref(res)), "tune_ex")
    return n, res


def tune_replay(space, ms_table, strategy, budget, seed=0, opts=None):
    """Returns (evaluations, tune_result, visited indices)."""
    n = len(ms_table)
    table = (ctypes.c_float * n)(*ms_table)
    visited = (ctypes.c_int * n)()
    res = tune_result()
    ev = _check(lib().tune_replay(space, table, n, strategy, budget, seed,
                                  ctypes.byref(opts) if opts is not None else None, visited, n,
                                  ctypes.byref(res)), "tune_replay")
    return ev, res, list(visited[:ev])


def sgemm_space_define_custom(spec):
    """Number of valid configurations of the newly defined SPACE_CUSTOM."""
    return _check(lib().sgemm_space_define_custom(spec.encode()), "sgemm_space_define_custom")


def sgemm_space_size(space):
    return _check(lib().sgemm_space_size(space), "sgemm_space_size")


def sgemm_space_raw_size(space):
    return _check(lib().sgemm_space_raw_size(space), "sgemm_space_raw_size")


def sgemm_space_get(space, index):
    c = sgemm_config()
    _check(lib().sgemm_space_get(space, index, ctypes.byref(c)), "sgemm_space_get")
    return c


def sgemm_space_find(space, cfg):
    return lib().sgemm_space_find(space, ctypes.byref(cfg))


def sgemm_space_dims(space):
    return _check(lib().sgemm_space_dims(space), "sgemm_space_dims")


def sgemm_space_values(space, dim):
    buf = (ctypes.c_int * 16)()
    n = _check(lib().sgemm_space_values(space, dim, buf, 16), "sgemm_space_values")
    return list(buf[:n])


def sgemm_config_check(cfg):
    return lib().sgemm_config_check(ctypes.byref(cfg))


def sgemm_config_lds_bytes(cfg):
    return _check(lib().sgemm_config_lds_bytes(ctypes.byref(cfg)), "sgemm_config_lds_bytes")


def sgemm_config_workspace_bytes(cfg, M, N, K):
    """(bytes of device workspace, parts, k_chunk) of a call with cfg on an M x N x K problem."""
    parts, chunk = ctypes.c_int(), ctypes.c_int()
    f = lib().sgemm_config_workspace_bytes
    f.restype = ctypes.c_longlong
    n = f(ctypes.byref(cfg), M, N, K, ctypes.byref(parts), ctypes.byref(chunk))
    if n < 0:
        raise SgemmError(int(n), "sgemm_config_workspace_bytes")
    return int(n), parts.value, chunk.value


def sgemm_config_default(M, N, K, layout=0):
    c = sgemm_config()
    _check(lib().sgemm_config_default(M, N, K, layout, ctypes.byref(c)), "sgemm_config_default")
    return c


def sgemm_kernel_cache_dir(path):
    return _check(lib().sgemm_kernel_cache_dir(os.fsencode(path)), "sgemm_kernel_cache_dir")


def sgemm_kernel_compile(cfg, layout=0, edge=0):
    info = sgemm_kernel_info()
    _check(lib().sgemm_kernel_compile(ctypes.byref(cfg), layout, edge, ctypes.byref(info)),
           "sgemm_kernel_compile")
    return info


def sgemm_kernel_cache_path(cfg, layout=0, edge=0):
    buf = ctypes.create_string_buffer(4096)
    _check(lib().sgemm_kernel_cache_path(ctypes.byref(cfg), layout, edge, buf, 4096),
           "sgemm_kernel_cache_path")
    return os.fsdecode(buf.value)


def sgemm_kernel_resolve(cfg, M, N, K, lda, ldb, ldc, layout=0, beta=0.0):
    """Returns (configuration as built, build flags)."""
    out, build = sgemm_config(), ctypes.c_int(0)
    _check(lib().sgemm_kernel_resolve(ctypes.byref(cfg), M, N, K, lda, ldb, ldc, layout, float(beta),
                                      ctypes.byref(out), ctypes.byref(build)), "sgemm_kernel_resolve")
    return out, build.value


def sgemm_kernel_macros(cfg, layout=0, edge=0):
    buf = ctypes.create_string_buffer(512)
    _check(lib().sgemm_kernel_macros(ctypes.byref(cfg), layout, edge, buf, 512),
           "sgemm_kernel_macros")
    return buf.value.decode()


def sgemm_config_get(M, N, K, layout=0):
    c = sgemm_config()
    st = lib().sgemm_config_get(M, N, K, layout, ctypes.byref(c))
    if st == E_NOCONFIG:
        return None
    _check(st, "sgemm_config_get")
    return c


def sgemm_config_set(M, N, K, layout, cfg, ms=0.0):
    return _check(lib().sgemm_config_set(M, N, K, layout, ctypes.byref(cfg), ms),
                  "sgemm_config_set")


def sgemm_config_select(M, N, K, layout=0):
    c = sgemm_config()
    _check(lib().sgemm_config_select(M, N, K, layout, ctypes.byref(c)), "sgemm_config_select")
    return c


def sgemm_cache_load(path):
    return _check(lib().sgemm_cache_load(os.fsencode(path)), "sgemm_cache_load")


def sgemm_cache_save(path):
    return _check(lib().sgemm_cache_save(os.fsencode(path)), "sgemm_cache_save")


def sgemm_cache_clear():
    return _check(lib().sgemm_cache_clear(), "sgemm_cache_clear")


def sgemm_cache_count():
    return _check(lib().sgemm_cache_count(), "sgemm_cache_count")


def sgemm_device_peak():
    """(FP32 peak in GFLOP/s, compute units, clock in MHz) of the current device."""
    g, cu, mhz = ctypes.c_float(), ctypes.c_int(), ctypes.c_int()
    _check(lib().sgemm_device_peak(ctypes.byref(g), ctypes.byref(cu), ctypes.byref(mhz)),
           "sgemm_device_peak")
    return g.value, cu.value, mhz.value


# ---- include/conv2d_tuned.h -----------------------------------------------------------------
def conv2d_space_size(Xf, Yf):
    return _check(lib().conv2d_space_size(Xf, Yf), "conv2d_space_size")


def conv2d_space_get(Xf, Yf, index):
    c = conv2d_config()
    _check(lib().conv2d_space_get(Xf, Yf, index, ctypes.byref(c)), "conv2d_space_get")
    return c


def conv2d_space_find(Xf, Yf, cfg):
    return lib().conv2d_space_find(Xf, Yf, ctypes.byref(cfg))


def conv2d_config_check(cfg, Xf, Yf):
    return lib().conv2d_config_check(ctypes.byref(cfg), Xf, Yf)


def conv2d_config_lds_bytes(cfg, Xf, Yf):
    return _check(lib().conv2d_config_lds_bytes(ctypes.byref(cfg), Xf, Yf), "conv2d_config_lds_bytes")


def conv2d_config_threads(cfg, Xf, Yf):
    return _check(lib().conv2d_config_threads(ctypes.byref(cfg), Xf, Yf), "conv2d_config_threads")


def conv2d_kernel_compile(cfg, Xf, Yf, edge=0, vector=1):
    info = sgemm_kernel_info()
    _check(lib().conv2d_kernel_compile(ctypes.byref(cfg), Xf, Yf, edge, vector, ctypes.byref(info)),
           "conv2d_kernel_compile")
    return info


def conv2d_run_config(stream, cfg, X, Y, Xf, Yf, w, F, A, lda, B, ldb):
    return _check(lib().conv2d_run_config(_stream(stream), ctypes.byref(cfg), X, Y, Xf, Yf, w,
                                          _ptr(F), _ptr(A), lda, _ptr(B), ldb), "conv2d_run_config")


def conv2d_reference(stream, X, Y, Xf, Yf, w, F, A, lda, B, ldb):
    return _check(lib().conv2d_reference(_stream(stream), X, Y, Xf, Yf, w, _ptr(F), _ptr(A), lda,
                                         _ptr(B), ldb), "conv2d_reference")


def conv2d_tuned(X, Y, Xf, Yf, w, F, A, lda, B, ldb):
    return _check(lib().conv2d_tuned(X, Y, Xf, Yf, w, _ptr(F), _ptr(A), lda, _ptr(B), ldb),
                  "conv2d_tuned")


def conv2d_config_set(X, Y, Xf, Yf, cfg, ms=0.0):
    return _check(lib().conv2d_config_set(X, Y, Xf, Yf, ctypes.byref(cfg), ms), "conv2d_config_set")


def conv2d_config_select(X, Y, Xf, Yf):
    """Returns (exact, conv2d_config)."""
    c = conv2d_config()
    exact = _check(lib().conv2d_config_select(X, Y, Xf, Yf, ctypes.byref(c)), "conv2d_config_select")
    return exact, c


def conv2d_cache_save(path):
    return _check(lib().conv2d_cache_save(path.encode()), "conv2d_cache_save")


def conv2d_cache_load(path):
    return _check(lib().conv2d_cache_load(path.encode()), "conv2d_cache_load")


def conv2d_cache_clear():
    return _check(lib().conv2d_cache_clear(), "conv2d_cache_clear")


def conv2d_tune(X, Y, Xf, Yf, w, strategy, budget, seed=0, opts=None):
    """Returns (evaluations, conv2d_tune_result)."""
    res = conv2d_tune_result()
    n = _check(lib().conv2d_tune(X, Y, Xf, Yf, w, strategy, budget, seed,
                                 ctypes.byref(opts) if opts is not None else None,
                                 ctypes.byref(res)), "conv2d_tune")
    return n, res


def conv2d_tune_replay(Xf, Yf, ms_table, strategy, budget, seed=0, opts=None):
    """Returns (evaluations, conv2d_tune_result, visited indices)."""
    n = len(ms_table)
    table = (ctypes.c_float * n)(*ms_table)
    visited = (ctypes.c_int * n)()
    res = conv2d_tune_result()
    ev = _check(lib().conv2d_tune_replay(Xf, Yf, table, n, strategy, budget, seed,
                                         ctypes.byref(opts) if opts is not None else None,
                                         visited, n, ctypes.byref(res)), "conv2d_tune_replay")
    return ev, res, list(visited[:ev])


# ---- include/kernel_tuner.h -----------------------------------------------------------------
def _int3(v):
    return (ctypes.c_int * 3)(*v)


def _names3(names):
    return (ctypes.c_char_p * 3)(*[n.encode() if n else None for n in names])


def ktuner_create(source, entry, global_size, local_size):
    h = lib().ktuner_create(source.encode(), entry.encode(), _int3(global_size), _int3(local_size))
    if not h:
        raise SgemmError(E_BADARG, "ktuner_create")
    return h


def ktuner_destroy(t):
    lib().ktuner_destroy(t)
    _ktuner_callbacks.pop(t, None)


def ktuner_add_parameter(t, name, values):
    arr = (ctypes.c_int * len(values))(*values)
    return _check(lib().ktuner_add_parameter(t, name.encode(), arr, len(values)), "ktuner_add_parameter")


def ktuner_mul_global_size(t, names):
    return _check(lib().ktuner_mul_global_size(t, _names3(names)), "ktuner_mul_global_size")


def ktuner_div_global_size(t, names):
    return _check(lib().ktuner_div_global_size(t, _names3(names)), "ktuner_div_global_size")


def ktuner_mul_local_size(t, names):
    return _check(lib().ktuner_mul_local_size(t, _names3(names)), "ktuner_mul_local_size")


def ktuner_div_local_size(t, names):
    return _check(lib().ktuner_div_local_size(t, _names3(names)), "ktuner_div_local_size")


_ktuner_callbacks = {}   # handle -> ctypes callbacks that must outlive the tuner


def ktuner_add_constraint(t, fn, names):
    """fn(list of values) -> bool, for the named parameters in that order."""
    n = len(names)
    cb = KTUNER_CONSTRAINT(lambda values, _user: 1 if fn([values[k] for k in range(n)]) else 0)
    _ktuner_callbacks.setdefault(t, []).append(cb)
    arr = (ctypes.c_char_p * n)(*[x.encode() for x in names])
    return _check(lib().ktuner_add_constraint(t, cb, arr, n, None), "ktuner_add_constraint")


def ktuner_add_argument_input(t, array):
    """array: a contiguous numpy array (host)."""
    return _check(lib().ktuner_add_argument_input(t, array.ctypes.data, array.nbytes),
                  "ktuner_add_argument_input")


def ktuner_add_argument_output(t, array):
    return _check(lib().ktuner_add_argument_output(t, array.ctypes.data, array.nbytes),
                  "ktuner_add_argument_output")


def ktuner_add_argument_int(t, value):
    return _check(lib().ktuner_add_argument_int(t, value), "ktuner_add_argument_int")


def ktuner_add_argument_float(t, value):
    return _check(lib().ktuner_add_argument_float(t, value), "ktuner_add_argument_float")


def ktuner_set_reference(t, source, entry, global_size, local_size):
    return _check(lib().ktuner_set_reference(t, source.encode(), entry.encode(), _int3(global_size),
                                             _int3(local_size)), "ktuner_set_reference")


def ktuner_set_tolerance(t, abs_tol, rel_tol):
    return _check(lib().ktuner_set_tolerance(t, abs_tol, rel_tol), "ktuner_set_tolerance")


def ktuner_space_size(t):
    return _check(lib().ktuner_space_size(t), "ktuner_space_size")


def ktuner_space_get(t, index, n_params):
    v = (ctypes.c_int * n_params)()
    _check(lib().ktuner_space_get(t, index, v), "ktuner_space_get")
    return tuple(v)


def ktuner_compile(t, index):
    info = sgemm_kernel_info()
    _check(lib().ktuner_compile(t, index, ctypes.byref(info)), "ktuner_compile")
    return info


def ktuner_launch_shape(t, index):
    g, l = (ctypes.c_int * 3)(), (ctypes.c_int * 3)()
    _check(lib().ktuner_launch_shape(t, index, g, l), "ktuner_launch_shape")
    return tuple(g), tuple(l)


def ktuner_tune(t, strategy, budget=0, seed=0, opts=None):
    """Returns (evaluations, ktuner_result)."""
    res = ktuner_result()
    n = _check(lib().ktuner_tune(t, strategy, budget, seed,
                                 ctypes.byref(opts) if opts is not None else None,
                                 ctypes.byref(res)), "ktuner_tune")
    return n, res


def ktuner_time_of(t, index):
    return lib().ktuner_time_of(t, index)


def ktuner_read_output(t, which, array):
    return _check(lib().ktuner_read_output(t, which, array.ctypes.data, array.nbytes), "ktuner_read_output")
