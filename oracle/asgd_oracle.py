"""ctypes wrapper around the CPU oracle (asgd_oracle.c).  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this
module.  It marshals NumPy arrays into the C functions and holds the oracle's run
state (fp64 worker states, external buffers, counters); it does no arithmetic of
the method itself.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "asgd_oracle.c")
_LIB = os.path.join(_HERE, "libasgd_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP over workers)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
             "-ffp-contract=off", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        f64p = np.ctypeslib.ndpointer(np.float64, flags="C_CONTIGUOUS")
        i64p = np.ctypeslib.ndpointer(np.int64, flags="C_CONTIGUOUS")
        L.asgd_oracle_peer.restype = C.c_int64
        L.asgd_oracle_peer.argtypes = [C.c_uint64, C.c_int64, C.c_int64, C.c_int64]
        L.asgd_oracle_dropped.restype = C.c_int
        L.asgd_oracle_dropped.argtypes = [C.c_uint64, C.c_int64, C.c_int64, C.c_uint32]
        L.asgd_oracle_peer_n.restype = C.c_int64
        L.asgd_oracle_peer_n.argtypes = [C.c_uint64, C.c_int64, C.c_int64, C.c_int64, C.c_int64]
        L.asgd_oracle_dropped_n.restype = C.c_int
        L.asgd_oracle_dropped_n.argtypes = [C.c_uint64, C.c_int64, C.c_int64, C.c_int64, C.c_uint32]
        L.asgd_oracle_threads.restype = C.c_int
        L.asgd_oracle_set_threads.argtypes = [C.c_int]
        L.asgd_oracle_assign.restype = None
        L.asgd_oracle_assign.argtypes = [C.c_void_p, C.c_int64, C.c_int, C.c_int, f64p, C.c_void_p, C.c_void_p]
        L.asgd_oracle_quant_error.restype = C.c_double
        L.asgd_oracle_quant_error.argtypes = [C.c_void_p, C.c_int64, C.c_int, C.c_int, f64p]
        L.asgd_oracle_steps.restype = C.c_int
        L.asgd_oracle_steps.argtypes = [
            C.c_void_p, C.c_int64, C.c_int, C.c_int, C.c_int, C.c_int, C.c_double, C.c_int, C.c_int, C.c_int,
            C.c_uint64, C.c_int, C.c_int, C.c_uint32, C.c_int64,
            f64p, f64p, i64p, i64p, i64p, i64p, i64p, i64p, C.c_void_p, C.c_void_p]
        _lib = L
    return _lib


def _f32(X) -> np.ndarray:
    X = np.ascontiguousarray(X, dtype=np.float32)
    assert X.ndim == 2
    return X


def peer(seed: int, r: int, i: int, W: int, n: int = 0) -> int:
    return int(lib().asgd_oracle_peer_n(seed, r, i, W, n))


def dropped(seed: int, r: int, sender: int, threshold: int, n: int = 0) -> bool:
    return bool(lib().asgd_oracle_dropped_n(seed, r, sender, n, threshold))


def threads() -> int:
    return int(lib().asgd_oracle_threads())


def set_threads(n: int) -> None:
    lib().asgd_oracle_set_threads(int(n))


def assign(X, w, want_gap: bool = False):
    """s_i(w) for every row of X under one k x d state (fp64)."""
    X = _f32(X)
    w = np.ascontiguousarray(w, dtype=np.float64)
    k, d = w.shape
    assert X.shape[1] == d
    idx = np.empty(X.shape[0], dtype=np.int32)
    gap = np.empty(X.shape[0], dtype=np.float64) if want_gap else None
    lib().asgd_oracle_assign(X.ctypes.data, X.shape[0], d, k, w, idx.ctypes.data,
                             gap.ctypes.data if want_gap else None)
    return (idx, gap) if want_gap else idx


def quant_error(X, w) -> float:
    """Eq. 8 over all rows of X."""
    X = _f32(X)
    w = np.ascontiguousarray(w, dtype=np.float64)
    k, d = w.shape
    assert X.shape[1] == d
    return float(lib().asgd_oracle_quant_error(X.ctypes.data, X.shape[0], d, k, w))


def centre_error(w, centres) -> float:
    """Error against the centres the data was generated from, as the paper uses it for its synthetic sets (Sec. 5.3, last
    paragraph: the distance between the generating centres and the returned ones; a relative measure).  The paper prints
    no formula; reading: for every generating centre the Euclidean distance to the nearest returned centroid, averaged
    over the generating centres.  Plain loops, fp64."""
    w = np.asarray(w, dtype=np.float64)
    centres = np.asarray(centres, dtype=np.float64)
    total = 0.0
    for c in centres:
        nearest = np.inf
        for row in w.reshape(-1, centres.shape[1]):
            dist = float(np.sqrt(np.sum((c - row) * (c - row))))
            nearest = min(nearest, dist)
        total += nearest
    return total / len(centres)


def drop_threshold(rate: float) -> int:
    """24-bit fixed-point loss probability used by the message-loss test hook."""
    return int(round(float(rate) * (1 << 24)))


class OracleASGD:
    """Run state of the oracle: W fp64 states, `buffers` external buffers per worker (slot[n, i] is buffer n of
    worker i; with one buffer the leading axis is dropped), counters."""

    LR_CONST, LR_INV_COUNT = 0, 1

    def __init__(self, X, k, W, b, lr, E=0, seed=1, parzen=True, lr_mode=0, drop_rate=0.0, w0=None, buffers=1, parts=1):
        self.X = _f32(X)
        self.N, self.d = self.X.shape
        self.k, self.W, self.b, self.lr, self.E = int(k), int(W), int(b), float(lr), int(E)
        self.seed, self.parzen, self.lr_mode = int(seed), bool(parzen), int(lr_mode)
        self.drop_threshold = drop_threshold(drop_rate)
        self.H = self.N // self.W
        self.S = self.H // self.b
        if self.H < self.k or self.S < 1:
            raise ValueError("shard shorter than k or b")
        if w0 is None:   # every worker starts from the first k rows of its own shard
            self.w = np.stack([self.X[i * self.H:i * self.H + self.k].astype(np.float64)
                               for i in range(self.W)])
        else:            # one common w0 sent to all workers (Sec. 4, Initialization)
            w0 = np.asarray(w0, dtype=np.float64)
            self.w = np.ascontiguousarray(np.broadcast_to(w0, (self.W, self.k, self.d))).copy()
        self.w = np.ascontiguousarray(self.w)
        self.buffers = int(buffers)
        self.parts = int(parts)
        lead = () if self.buffers == 1 else (self.buffers,)
        self.slot = np.zeros(lead + (self.W, self.k, self.d), dtype=np.float64)
        self.slot_stamp = np.full(lead + (self.W,), -1, dtype=np.int64)
        self.ncum = np.zeros((self.W, self.k), dtype=np.int64)
        self.t = np.zeros(1, dtype=np.int64)
        self.counters = np.zeros((self.W, 3), dtype=np.int64)   # sent, received, accepted
        self.near = np.zeros(2, dtype=np.int64)                 # argmin / Parzen near-ties
        self.parzen_near = np.zeros(self.W, dtype=np.int64)     # Parzen near-ties per worker

    def run_steps(self, nsteps: int, dump: bool = False):
        nsteps = int(nsteps)
        a = np.empty((nsteps, self.W, self.b), dtype=np.int32) if dump else None
        g = np.empty((nsteps, self.W, self.b), dtype=np.float64) if dump else None
        rc = lib().asgd_oracle_steps(
            self.X.ctypes.data, self.N, self.k, self.d, self.W, self.b, self.lr, self.E, self.buffers, self.parts,
            self.seed, int(self.parzen), self.lr_mode, self.drop_threshold, nsteps,
            self.w.reshape(-1), self.slot.reshape(-1), self.slot_stamp.reshape(-1), self.ncum.reshape(-1),
            self.t, self.counters.reshape(-1), self.near, self.parzen_near,
            a.ctypes.data if dump else None, g.ctypes.data if dump else None)
        if rc != 0:
            raise ValueError("asgd_oracle_steps rejected its arguments")
        return (a, g) if dump else None

    def set_window(self, Xw, t_start: int):
        """Hand the oracle only the rows that the steps [t_start, t_start + n) touch: Xw holds, shard after shard, the
        n*b rows of those steps (n = rows per shard / b).  For inputs that do not fit the host as a whole.  Indexing
        only: the C routine finds the mini-batch of step t at row (t mod n)*b of a shard, which is the right one when
        the window starts at a multiple of n and does not cross the end of an epoch."""
        Xw = _f32(Xw)
        assert Xw.shape[1] == self.d and Xw.shape[0] % (self.W * self.b) == 0
        n = Xw.shape[0] // (self.W * self.b)
        assert int(self.t[0]) == t_start and t_start % n == 0
        self.X, self.N = Xw, Xw.shape[0]

    def run_epochs(self, epochs: int, dump: bool = False):
        return self.run_steps(int(epochs) * self.S, dump=dump)

    def quant_error(self, worker: int = 0) -> float:
        return quant_error(self.X, self.w[worker])
