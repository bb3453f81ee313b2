"""Thin ctypes binding of libautohete.so (the C ABI in include/autohete.h).

Argument marshalling only: every step of the update runs in the library's HIP kernels.
There is no CPU fallback -- if the library is missing, importing this module raises.
Function names are the C names.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libautohete.so")

AH_OK, AH_EINVAL, AH_EALIGN, AH_ENOMEM, AH_EHIP, AH_EINFEASIBLE, AH_ELIMIT = 0, -1, -2, -3, -4, -5, -6
AUTOHETE_STATIC_MAX_CHUNKS = 128
AH_BF16, AH_FP16 = 0, 1
AH_TUNE_STEP_BLOCKS_PER_CU, AH_TUNE_PREP_BLOCKS, AH_TUNE_STEP_VARIANT, AH_TUNE_CAST_BLOCKS_PER_CU = 0, 1, 2, 3
AH_TUNE_CARRY_ELEMS = 4


def step_variant(vec=4, block=64, mode=0):
    """Encode a value for AH_TUNE_STEP_VARIANT."""
    return vec | (mode << 4) | ((block // 64) << 8)

# PyTorch-ROCm ships its own copy of the HIP runtime (same SONAME as the system one).  The device
# pointers and streams this binding is handed belong to THAT runtime instance, so it must already
# be in the process when libautohete.so resolves its libamdhip64 dependency; loaded the other way
# round, the process ends up with two HIP runtimes that do not share allocations or streams.
try:
    import torch  # noqa: F401
except ImportError:  # a caller that manages device memory through the system HIP runtime
    pass

if not os.path.exists(LIB_PATH):
    raise ImportError("libautohete.so is not built (%s): run __graft_entry__.build() or "
                      "python paper_2503_01890_amd/build.py" % LIB_PATH)
_lib = ctypes.CDLL(LIB_PATH)


class autohete_chunk(ctypes.Structure):
    _fields_ = [("grad", ctypes.c_void_p), ("param_lp", ctypes.c_void_p), ("master", ctypes.c_void_p),
                ("exp_avg", ctypes.c_void_p), ("exp_avg_sq", ctypes.c_void_p), ("numel", ctypes.c_uint64)]


class autohete_hparams(ctypes.Structure):
    _fields_ = [(k, ctypes.c_float) for k in
                ("lr", "beta1", "beta2", "eps", "weight_decay", "max_grad_norm", "loss_scale")]


class autohete_grad_result(ctypes.Structure):
    _fields_ = [("sumsq", ctypes.c_double), ("norm_d", ctypes.c_double), ("norm", ctypes.c_float),
                ("found_inf", ctypes.c_uint32)]


class autohete_cost_model(ctypes.Structure):
    _fields_ = [("n_blocks", ctypes.c_uint32)] + [(k, ctypes.c_double) for k in (
        "act_elems", "act_in_elems", "param_elems", "gpu_const_bytes", "cpu_const_bytes", "gpu_capacity_bytes",
        "cpu_capacity_bytes", "t_fp", "t_bp", "t_h2d", "t_d2h", "t_optim_cpu", "t_optim_gpu")]


class autohete_strategy(ctypes.Structure):
    _fields_ = [("n_ckpt", ctypes.c_uint32), ("n_param_offload", ctypes.c_uint32), ("n_optim_offload", ctypes.c_uint32),
                ("feasible", ctypes.c_int), ("gpu_bytes", ctypes.c_double), ("cpu_bytes", ctypes.c_double),
                ("t_fwd", ctypes.c_double), ("t_sync", ctypes.c_double), ("t_bwd", ctypes.c_double)]


class AutoheteError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__("%s: %s (%d)" % (where, _lib.autohete_strerror(status).decode(), status))


_u64p = ctypes.POINTER(ctypes.c_uint64)
_lib.autohete_strerror.restype = ctypes.c_char_p
_lib.autohete_strerror.argtypes = [ctypes.c_int]
_lib.autohete_chunk_layout.restype = ctypes.c_int
_lib.autohete_chunk_layout.argtypes = [_u64p, ctypes.c_uint64, ctypes.c_uint64, _u64p, _u64p, _u64p, _u64p]
_lib.autohete_ws_create.restype = ctypes.c_int
_lib.autohete_ws_create.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_uint64]
_lib.autohete_ws_destroy.restype = ctypes.c_int
_lib.autohete_ws_destroy.argtypes = [ctypes.c_void_p]
_lib.autohete_ws_tune.restype = ctypes.c_int
_lib.autohete_ws_tune.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int64]
_lib.autohete_grad_prep.restype = ctypes.c_int
_lib.autohete_grad_prep.argtypes = [ctypes.c_void_p, ctypes.POINTER(autohete_chunk), ctypes.c_uint64, ctypes.c_int,
                                    ctypes.c_float, ctypes.c_double, ctypes.c_void_p,
                                    ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_uint32)]
_lib.autohete_grad_prep_accumulate.restype = ctypes.c_int
_lib.autohete_grad_prep_accumulate.argtypes = [ctypes.c_void_p, ctypes.POINTER(autohete_chunk), ctypes.c_uint64,
                                               ctypes.c_int, ctypes.c_float, ctypes.c_void_p]
_lib.autohete_grad_prep_static.restype = ctypes.c_int
_lib.autohete_grad_prep_static.argtypes = [ctypes.POINTER(autohete_chunk), ctypes.c_uint64, ctypes.c_int, ctypes.c_float,
                                           ctypes.c_double, ctypes.c_void_p, ctypes.c_void_p]
_lib.autohete_adamw_step.restype = ctypes.c_int
_lib.autohete_adamw_step.argtypes = [ctypes.c_void_p, ctypes.POINTER(autohete_chunk), ctypes.c_uint64, ctypes.c_int,
                                     ctypes.c_uint64, ctypes.POINTER(autohete_hparams), ctypes.c_void_p]
_lib.autohete_adamw_step_carry.restype = ctypes.c_int
_lib.autohete_adamw_step_carry.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.POINTER(autohete_chunk),
                                           ctypes.c_uint64, ctypes.c_int, ctypes.c_uint64,
                                           ctypes.POINTER(autohete_hparams), ctypes.c_void_p]
_lib.autohete_adamw_step_master.restype = ctypes.c_int
_lib.autohete_adamw_step_master.argtypes = _lib.autohete_adamw_step.argtypes
_lib.autohete_cast_params.restype = ctypes.c_int
_lib.autohete_cast_params.argtypes = [ctypes.c_void_p, ctypes.POINTER(autohete_chunk), ctypes.c_uint64, ctypes.c_int,
                                      ctypes.c_void_p]
_lib.autohete_grad_result_get.restype = ctypes.c_int
_lib.autohete_grad_result_get.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.POINTER(ctypes.c_double),
                                          ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_uint32)]
_lib.autohete_grad_result_set.restype = ctypes.c_int
_lib.autohete_grad_result_set.argtypes = [ctypes.c_void_p, ctypes.c_double, ctypes.c_uint32, ctypes.c_void_p]


_lib.autohete_strategy_eval.restype = ctypes.c_int
_lib.autohete_strategy_eval.argtypes = [ctypes.POINTER(autohete_cost_model), ctypes.c_uint32, ctypes.c_uint32,
                                        ctypes.c_uint32, ctypes.POINTER(autohete_strategy)]
_lib.autohete_strategy_search.restype = ctypes.c_int
_lib.autohete_strategy_search.argtypes = [ctypes.POINTER(autohete_cost_model), ctypes.POINTER(autohete_strategy)]


_lib.autohete_host_grad_sumsq.restype = ctypes.c_int
_lib.autohete_host_grad_sumsq.argtypes = [ctypes.POINTER(autohete_chunk), ctypes.c_uint64, ctypes.c_int, ctypes.c_float,
                                          ctypes.c_int, ctypes.POINTER(ctypes.c_double),
                                          ctypes.POINTER(ctypes.c_uint32)]
_lib.autohete_host_adamw_step.restype = ctypes.c_int
_lib.autohete_host_adamw_step.argtypes = [ctypes.POINTER(autohete_chunk), ctypes.c_uint64, ctypes.c_int, ctypes.c_uint64,
                                          ctypes.POINTER(autohete_hparams), ctypes.c_double, ctypes.c_uint32,
                                          ctypes.c_int]
_lib.autohete_host_force_scalar.restype = ctypes.c_int
_lib.autohete_host_force_scalar.argtypes = [ctypes.c_int]


def _check(rc, where):
    if rc != AH_OK:
        raise AutoheteError(rc, where)


def autohete_chunk_layout(tensor_numel, chunk_elems):
    """-> (tensor_offset list, n_chunks, total_elems, padded_elems).  Host only."""
    n = len(tensor_numel)
    numel = (ctypes.c_uint64 * max(n, 1))(*[int(x) for x in tensor_numel])
    off = (ctypes.c_uint64 * max(n, 1))()
    nc, tot, pad = ctypes.c_uint64(), ctypes.c_uint64(), ctypes.c_uint64()
    _check(_lib.autohete_chunk_layout(numel, n, int(chunk_elems), off, ctypes.byref(nc), ctypes.byref(tot),
                                      ctypes.byref(pad)), "autohete_chunk_layout")
    return list(off[:n]), nc.value, tot.value, pad.value


def autohete_grad_prep_static(chunks, n_chunks, lowp_dtype, loss_scale, extra_sumsq, stream, result_dev_ptr):
    """The workspace-free, allocation-free norm pass; result_dev_ptr: device address of 32 bytes
    (an autohete_grad_result) that the kernel fills on `stream`."""
    _check(_lib.autohete_grad_prep_static(chunks, n_chunks, lowp_dtype, loss_scale, extra_sumsq,
                                          ctypes.c_void_p(stream), ctypes.c_void_p(result_dev_ptr)),
           "autohete_grad_prep_static")


def autohete_strategy_eval(model, n_ckpt, n_param_offload, n_optim_offload):
    out = autohete_strategy()
    _check(_lib.autohete_strategy_eval(ctypes.byref(model), n_ckpt, n_param_offload, n_optim_offload,
                                       ctypes.byref(out)), "autohete_strategy_eval")
    return out


def autohete_strategy_search(model):
    out = autohete_strategy()
    _check(_lib.autohete_strategy_search(ctypes.byref(model), ctypes.byref(out)), "autohete_strategy_search")
    return out


def autohete_host_grad_sumsq(chunks, n_chunks, lowp_dtype, loss_scale, n_threads):
    """chunks: array from chunk_array() holding HOST addresses.  -> (sumsq, found_inf)"""
    s, f = ctypes.c_double(), ctypes.c_uint32()
    _check(_lib.autohete_host_grad_sumsq(chunks, n_chunks, lowp_dtype, loss_scale, n_threads, ctypes.byref(s),
                                         ctypes.byref(f)), "autohete_host_grad_sumsq")
    return s.value, f.value


def autohete_host_adamw_step(chunks, n_chunks, lowp_dtype, step, hp, sumsq, found_inf, n_threads):
    _check(_lib.autohete_host_adamw_step(chunks, n_chunks, lowp_dtype, int(step), ctypes.byref(hp), float(sumsq),
                                         int(found_inf), n_threads), "autohete_host_adamw_step")


def chunk_array(chunks):
    """Marshal a list of (grad, param_lp, master, exp_avg, exp_avg_sq, numel) device addresses."""
    arr = (autohete_chunk * max(len(chunks), 1))()
    for i, c in enumerate(chunks):
        arr[i] = autohete_chunk(*[int(x) if x is not None else None for x in c])
    return arr


class Workspace:
    """Owns one autohete_ws; use from one host thread, one stream at a time."""

    def __init__(self, max_chunks):
        self._h = ctypes.c_void_p()
        _check(_lib.autohete_ws_create(ctypes.byref(self._h), int(max_chunks)), "autohete_ws_create")

    def close(self):
        if self._h:
            _lib.autohete_ws_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def tune(self, knob, value):
        _check(_lib.autohete_ws_tune(self._h, knob, int(value)), "autohete_ws_tune")

    def autohete_grad_prep(self, chunks, n_chunks, lowp_dtype, loss_scale, extra_sumsq=0.0, stream=0,
                           want_result=False):
        """chunks: array from chunk_array().  With want_result -> (norm, found_inf) after a sync."""
        if want_result:
            norm, flag = ctypes.c_float(), ctypes.c_uint32()
            _check(_lib.autohete_grad_prep(self._h, chunks, n_chunks, lowp_dtype, loss_scale, extra_sumsq,
                                           ctypes.c_void_p(stream), ctypes.byref(norm), ctypes.byref(flag)),
                   "autohete_grad_prep")
            return norm.value, flag.value
        _check(_lib.autohete_grad_prep(self._h, chunks, n_chunks, lowp_dtype, loss_scale, extra_sumsq,
                                       ctypes.c_void_p(stream), None, None), "autohete_grad_prep")
        return None

    def autohete_grad_prep_accumulate(self, chunks, n_chunks, lowp_dtype, loss_scale, stream=0):
        _check(_lib.autohete_grad_prep_accumulate(self._h, chunks, n_chunks, lowp_dtype, loss_scale,
                                                  ctypes.c_void_p(stream)), "autohete_grad_prep_accumulate")

    def autohete_adamw_step(self, chunks, n_chunks, lowp_dtype, step, hp, stream=0):
        _check(_lib.autohete_adamw_step(self._h, chunks, n_chunks, lowp_dtype, int(step), ctypes.byref(hp),
                                        ctypes.c_void_p(stream)), "autohete_adamw_step")

    def autohete_adamw_step_carry(self, ws_next, chunks, n_chunks, lowp_dtype, step, hp, stream=0):
        _check(_lib.autohete_adamw_step_carry(self._h, ws_next._h if ws_next is not None else None, chunks,
                                              n_chunks, lowp_dtype, int(step), ctypes.byref(hp),
                                              ctypes.c_void_p(stream)), "autohete_adamw_step_carry")

    def autohete_adamw_step_master(self, chunks, n_chunks, lowp_dtype, step, hp, stream=0):
        _check(_lib.autohete_adamw_step_master(self._h, chunks, n_chunks, lowp_dtype, int(step), ctypes.byref(hp),
                                               ctypes.c_void_p(stream)), "autohete_adamw_step_master")

    def autohete_cast_params(self, chunks, n_chunks, lowp_dtype, stream=0):
        _check(_lib.autohete_cast_params(self._h, chunks, n_chunks, lowp_dtype, ctypes.c_void_p(stream)),
               "autohete_cast_params")

    def autohete_grad_result_get(self, stream=0):
        """-> (sumsq, norm, found_inf); waits for the stream."""
        s, n, f = ctypes.c_double(), ctypes.c_float(), ctypes.c_uint32()
        _check(_lib.autohete_grad_result_get(self._h, ctypes.c_void_p(stream), ctypes.byref(s), ctypes.byref(n),
                                             ctypes.byref(f)), "autohete_grad_result_get")
        return s.value, n.value, f.value

    def autohete_grad_result_set(self, sumsq, found_inf, stream=0):
        _check(_lib.autohete_grad_result_set(self._h, float(sumsq), int(found_inf), ctypes.c_void_p(stream)),
               "autohete_grad_result_set")


def hparams(lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01, max_grad_norm=1.0, loss_scale=1.0):
    return autohete_hparams(lr, beta1, beta2, eps, weight_decay, max_grad_norm, loss_scale)


def raw():
    """The ctypes CDLL itself (used by the symbol-export test)."""
    return _lib
