"""ctypes binding of libasgd_hip.so: same names as the C ABI, argument marshalling only.

PyTorch is used by callers for device memory and streams; nothing of the method is
computed here.  There is no fallback: if the library has not been built, importing a
symbol from it raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from . import build as _build

OK, EINVAL, ENOMEM, ESTATE, EHIP, ESYNC = 0, -1, -2, -3, -4, -5
OPT_EXCHANGE_EVERY, OPT_SEED, OPT_MODE, OPT_PARZEN, OPT_LR_MODE, OPT_DROP_RATE, OPT_KERNEL, OPT_TUNE, OPT_COOPERATIVE, OPT_BUFFERS, OPT_PARTS, OPT_WAIT_POLLS, OPT_DROP_UNANNOUNCED = range(1, 14)
MODE_DETERMINISTIC, MODE_FREE_RUNNING = 0, 1
LR_CONST, LR_INV_COUNT = 0, 1
KERNEL_AUTO, KERNEL_GENERIC, KERNEL_SMALL, KERNEL_MFMA = 0, 1, 2, 3

# every symbol include/asgd.h declares
SYMBOLS = (
    "asgd_create", "asgd_set_option", "asgd_load_shards", "asgd_set_state", "asgd_set_step",
    "asgd_run_epochs", "asgd_run_steps", "asgd_set_assign_dump", "asgd_get_state",
    "asgd_get_mean_state", "asgd_quant_error", "asgd_last_run_ms", "asgd_get_stats", "asgd_get_worker_counters",
    "asgd_schedule_peer", "asgd_schedule_peer_n", "asgd_last_hip_error", "asgd_destroy", "asgd_strerror",
    "asgd_quant_error_noalloc", "asgd_get_exchange", "asgd_set_exchange",
)


class asgd_stats(C.Structure):
    _fields_ = [("steps", C.c_int64), ("samples", C.c_int64), ("sent", C.c_int64),
                ("received", C.c_int64), ("accepted", C.c_int64), ("parzen_near_ties", C.c_int64),
                ("exact_rechecks", C.c_int64), ("last_run_ms", C.c_double),
                ("kernel", C.c_int32), ("launches", C.c_int32)]


class AsgdError(RuntimeError):
    def __init__(self, code, what, hip_error=0):
        self.code = code
        self.hip_error = hip_error
        extra = ", hipError_t %d" % hip_error if hip_error else ""
        super().__init__("%s failed: %s (code %d%s)" % (what, strerror(code), code, extra))


_lib = None


def lib():
    """The loaded library.  Builds it only if no built library is present; warns if the one present is stale."""
    global _lib
    if _lib is None:
        if not os.path.exists(_build.LIB_PATH):
            _build.build_library(verbose=False)
        elif _build.is_stale():
            # a source is newer than the built library: say so loudly, but run what is built (a build belongs before
            # the run, not inside it; ASGD_REBUILD_STALE=1 asks for it here all the same)
            if os.environ.get("ASGD_REBUILD_STALE") == "1":
                _build.build_library(verbose=False)
            else:
                import warnings
                warnings.warn("libasgd_hip.so is older than its sources: run `python -m paper_1505_04956_amd.build` "
                              "(or __graft_entry__.build()); loading the old library", RuntimeWarning, stacklevel=2)
        L = C.CDLL(_build.LIB_PATH)
        vp, i64, u64, dbl = C.c_void_p, C.c_int64, C.c_uint64, C.c_double
        sig = {
            "asgd_create": (C.c_int, [C.POINTER(vp), C.c_int, C.c_int, C.c_int, C.c_int, C.c_float]),
            "asgd_set_option": (C.c_int, [vp, C.c_int, dbl]),
            "asgd_load_shards": (C.c_int, [vp, vp, i64, vp]),
            "asgd_set_state": (C.c_int, [vp, C.c_int, vp]),
            "asgd_set_step": (C.c_int, [vp, i64]),
            "asgd_get_exchange": (C.c_int, [vp, vp, C.c_size_t, vp, C.c_size_t]),
            "asgd_set_exchange": (C.c_int, [vp, vp, vp]),
            "asgd_run_epochs": (C.c_int, [vp, C.c_int]),
            "asgd_run_steps": (C.c_int, [vp, i64]),
            "asgd_set_assign_dump": (C.c_int, [vp, vp, C.c_size_t]),
            "asgd_get_state": (C.c_int, [vp, C.c_int, vp, C.c_size_t]),
            "asgd_get_mean_state": (C.c_int, [vp, vp, C.c_size_t]),
            "asgd_quant_error": (C.c_int, [vp, C.c_int, C.POINTER(dbl)]),
            "asgd_last_run_ms": (C.c_int, [vp, C.POINTER(dbl)]),
            "asgd_get_stats": (C.c_int, [vp, C.POINTER(asgd_stats)]),
            "asgd_get_worker_counters": (C.c_int, [vp, vp, vp, vp]),
            "asgd_schedule_peer": (i64, [u64, i64, i64, i64]),
            "asgd_schedule_peer_n": (i64, [u64, i64, i64, i64, i64]),
            "asgd_last_hip_error": (C.c_int, [vp]),
            "asgd_destroy": (None, [vp]),
            "asgd_strerror": (C.c_char_p, [C.c_int]),
            "asgd_quant_error_noalloc": (C.c_int, [vp, i64, C.c_int, C.c_int, vp, vp, vp]),
        }
        for name, (res, args) in sig.items():
            fn = getattr(L, name)
            fn.restype, fn.argtypes = res, args
        _lib = L
    return _lib


def strerror(code: int) -> str:
    return lib().asgd_strerror(int(code)).decode()


def _check(code, what, h=None):
    if code != OK:
        hip_error = int(lib().asgd_last_hip_error(h)) if (h is not None and code == EHIP) else 0
        raise AsgdError(code, what, hip_error)


# ---- one function per C entry point ---------------------------------------------------
def asgd_create(k, d, W, b, lr):
    h = C.c_void_p()
    _check(lib().asgd_create(C.byref(h), k, d, W, b, lr), "asgd_create")
    return h


def asgd_set_option(h, key, value):
    _check(lib().asgd_set_option(h, key, float(value)), "asgd_set_option", h)


def asgd_load_shards(h, x_dev_ptr, N, stream=0):
    _check(lib().asgd_load_shards(h, x_dev_ptr, N, stream), "asgd_load_shards", h)


def asgd_set_state(h, worker, w_host: np.ndarray):
    w_host = np.ascontiguousarray(w_host, dtype=np.float32)
    _check(lib().asgd_set_state(h, worker, w_host.ctypes.data), "asgd_set_state", h)


def asgd_set_step(h, t):
    _check(lib().asgd_set_step(h, t), "asgd_set_step")


def asgd_get_exchange(h, values: np.ndarray, rounds: np.ndarray):
    assert values.dtype == np.float32 and rounds.dtype == np.int32
    assert values.flags["C_CONTIGUOUS"] and rounds.flags["C_CONTIGUOUS"]
    _check(lib().asgd_get_exchange(h, values.ctypes.data, values.nbytes, rounds.ctypes.data, rounds.nbytes),
           "asgd_get_exchange", h)


def asgd_set_exchange(h, values: np.ndarray, rounds: np.ndarray):
    values = np.ascontiguousarray(values, dtype=np.float32)
    rounds = np.ascontiguousarray(rounds, dtype=np.int32)
    _check(lib().asgd_set_exchange(h, values.ctypes.data, rounds.ctypes.data), "asgd_set_exchange", h)


def asgd_run_epochs(h, epochs):
    _check(lib().asgd_run_epochs(h, epochs), "asgd_run_epochs", h)


def asgd_run_steps(h, steps):
    _check(lib().asgd_run_steps(h, steps), "asgd_run_steps", h)


def asgd_set_assign_dump(h, dev_ptr, capacity):
    _check(lib().asgd_set_assign_dump(h, dev_ptr, capacity), "asgd_set_assign_dump")


def asgd_get_state(h, worker, out: np.ndarray):
    assert out.dtype == np.float32 and out.flags.c_contiguous
    _check(lib().asgd_get_state(h, worker, out.ctypes.data, out.nbytes), "asgd_get_state", h)


def asgd_get_mean_state(h, out: np.ndarray):
    assert out.dtype == np.float32 and out.flags.c_contiguous
    _check(lib().asgd_get_mean_state(h, out.ctypes.data, out.nbytes), "asgd_get_mean_state", h)


def asgd_quant_error(h, worker) -> float:
    v = C.c_double()
    _check(lib().asgd_quant_error(h, worker, C.byref(v)), "asgd_quant_error", h)
    return v.value


def asgd_quant_error_noalloc(x_dev_ptr, N, k, d, w_dev_ptr, out_dev_ptr, stream=0):
    _check(lib().asgd_quant_error_noalloc(x_dev_ptr, N, k, d, w_dev_ptr, out_dev_ptr, stream), "asgd_quant_error_noalloc")


def asgd_last_run_ms(h) -> float:
    v = C.c_double()
    _check(lib().asgd_last_run_ms(h, C.byref(v)), "asgd_last_run_ms")
    return v.value


def asgd_get_stats(h) -> asgd_stats:
    s = asgd_stats()
    _check(lib().asgd_get_stats(h, C.byref(s)), "asgd_get_stats")
    return s


def asgd_get_worker_counters(h, W):
    a = [np.zeros(W, dtype=np.int64) for _ in range(3)]
    _check(lib().asgd_get_worker_counters(h, *[v.ctypes.data for v in a]), "asgd_get_worker_counters")
    return a


def asgd_schedule_peer(seed, r, i, W) -> int:
    return int(lib().asgd_schedule_peer(seed, r, i, W))


def asgd_schedule_peer_n(seed, r, i, W, n) -> int:
    return int(lib().asgd_schedule_peer_n(seed, r, i, W, n))


def asgd_destroy(h):
    lib().asgd_destroy(h)


# ---- convenience wrapper: owns a handle, keeps the borrowed tensors alive -----------------
class ASGD:
    def __init__(self, k, d, W, b, lr, E=0, seed=1, mode=MODE_DETERMINISTIC, parzen=True,
                 lr_mode=LR_CONST, drop_rate=0.0, kernel=KERNEL_AUTO, tune=0, cooperative=True, buffers=1, parts=1):
        self.k, self.d, self.W, self.b, self.buffers = k, d, W, b, buffers
        self.h = asgd_create(k, d, W, b, lr)
        for key, val in ((OPT_EXCHANGE_EVERY, E), (OPT_SEED, seed), (OPT_MODE, mode),
                         (OPT_PARZEN, int(parzen)), (OPT_LR_MODE, lr_mode),
                         (OPT_DROP_RATE, drop_rate), (OPT_KERNEL, kernel), (OPT_TUNE, tune),
                         (OPT_COOPERATIVE, int(cooperative)), (OPT_BUFFERS, buffers), (OPT_PARTS, parts)):
            asgd_set_option(self.h, key, val)
        self._x = None
        self._dump = None

    def set_option(self, key, value):
        asgd_set_option(self.h, key, value)

    def load_shards(self, x):
        """x: torch float32 CUDA tensor, N x d, contiguous (borrowed, kept referenced here)."""
        import torch
        assert x.is_cuda and x.dtype == torch.float32 and x.is_contiguous() and x.shape[1] == self.d
        self._x = x
        stream = torch.cuda.current_stream(x.device).cuda_stream
        asgd_load_shards(self.h, x.data_ptr(), x.shape[0], stream)
        self.H = x.shape[0] // self.W
        self.S = self.H // self.b

    def enable_assign_dump(self, steps):
        import torch
        self._dump = torch.empty(steps * self.W * self.b, dtype=torch.int32, device=self._x.device)
        asgd_set_assign_dump(self.h, self._dump.data_ptr(), self._dump.numel())

    def disable_assign_dump(self):
        asgd_set_assign_dump(self.h, None, 0)
        self._dump = None

    def assign_dump(self, steps):
        return self._dump[:steps * self.W * self.b].cpu().numpy().reshape(steps, self.W, self.b)

    def set_state(self, worker, w):
        asgd_set_state(self.h, worker, w)

    def set_step(self, t):
        asgd_set_step(self.h, t)

    def get_exchange(self):
        """(values [buffers, W, k, d] float32, rounds [buffers, W] int32): the messages in flight."""
        values = np.empty((self.buffers, self.W, self.k, self.d), dtype=np.float32)
        rounds = np.empty((self.buffers, self.W), dtype=np.int32)
        asgd_get_exchange(self.h, values, rounds)
        return values, rounds

    def set_exchange(self, values, rounds):
        values, rounds = np.asarray(values), np.asarray(rounds)
        assert values.shape == (self.buffers, self.W, self.k, self.d) and rounds.shape == (self.buffers, self.W)
        asgd_set_exchange(self.h, values, rounds)

    def run_epochs(self, epochs):
        asgd_run_epochs(self.h, epochs)

    def run_steps(self, steps):
        asgd_run_steps(self.h, steps)

    def get_state(self, worker=-1):
        out = np.empty((self.W, self.k, self.d) if worker < 0 else (self.k, self.d), dtype=np.float32)
        asgd_get_state(self.h, worker, out)
        return out

    def get_mean_state(self):
        out = np.empty((self.k, self.d), dtype=np.float32)
        asgd_get_mean_state(self.h, out)
        return out

    def quant_error(self, worker=0):
        return asgd_quant_error(self.h, worker)

    def last_run_ms(self):
        return asgd_last_run_ms(self.h)

    def stats(self):
        return asgd_get_stats(self.h)

    def worker_counters(self):
        return np.stack(asgd_get_worker_counters(self.h, self.W), axis=1)   # W x (sent, received, accepted)

    def close(self):
        if self.h is not None:
            asgd_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
