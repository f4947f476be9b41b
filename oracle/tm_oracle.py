"""ctypes front end of the sequential C oracle (oracle/tm_oracle.c).

TEST INFRASTRUCTURE: only tests, the smoke check and the benchmark's
cpu_baseline leg may import this module.  It does argument marshalling only;
every step of the method is in the C file, which follows the paper section by
section.  Arrays are numpy: X uint8 [q][o], y int32 [q], state int32 [C][2o]
holding the TA state 1..2N.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tm_oracle.c")
_LIB = os.path.join(_HERE, "liboracle_tm.so")

INIT, GATE, TYPE1, NEGCLASS = 0, 1, 2, 3


def build(force=False):
    """Compile the oracle with gcc (plain -O2, no tuning flags)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-Wall", "-shared", "-fPIC", _SRC, "-o", tmp])
        os.replace(tmp, _LIB)
    return _LIB


class Config(ctypes.Structure):
    _fields_ = [("m", ctypes.c_int32), ("n", ctypes.c_int32), ("o", ctypes.c_int32),
                ("N", ctypes.c_int32), ("T", ctypes.c_int32), ("s", ctypes.c_double),
                ("seed", ctypes.c_uint64), ("boost", ctypes.c_int32), ("regression", ctypes.c_int32)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.otm_neg_class.restype = ctypes.c_int32
        _lib.otm_gate.restype = ctypes.c_int
        _lib.otm_gate_regression.restype = ctypes.c_int
        _lib.otm_threshold.restype = ctypes.c_int32
    return _lib


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _chk(a, dtype, shape=None):
    assert isinstance(a, np.ndarray) and a.dtype == dtype and a.flags["C_CONTIGUOUS"], (a.dtype, dtype)
    if shape is not None:
        assert tuple(a.shape) == tuple(shape), (a.shape, shape)
    return a


class Oracle:
    """Holds a configuration and the TA states; methods mirror the C functions."""

    def __init__(self, m, n, o, N, T, s, seed, init=True, boost=False, regression=False):
        assert not regression or m == 1
        self.cfg = Config(m, n, o, N, T, float(s), seed, 1 if boost else 0, 1 if regression else 0)
        self.m, self.n, self.o, self.N, self.T, self.s, self.seed = m, n, o, N, T, float(s), seed
        self.C, self.L = m * n, 2 * o
        self.state = np.zeros((self.C, self.L), dtype=np.int32)
        if init:
            lib().otm_init(ctypes.byref(self.cfg), _p(self.state))

    # ---- inference -------------------------------------------------------
    def clause_outputs(self, X):
        q = X.shape[0]
        _chk(X, np.uint8, (q, self.o))
        out = np.zeros((q, self.C), dtype=np.uint8)
        lib().otm_clause_outputs(ctypes.byref(self.cfg), _p(self.state), _p(X), ctypes.c_int64(q), _p(out))
        return out

    def class_sums(self, X, clamp=True):
        q = X.shape[0]
        _chk(X, np.uint8, (q, self.o))
        out = np.zeros((q, self.m), dtype=np.int32)
        lib().otm_class_sums(ctypes.byref(self.cfg), _p(self.state), _p(X), ctypes.c_int64(q),
                             ctypes.c_int(1 if clamp else 0), _p(out))
        return out

    def predict(self, X):
        q = X.shape[0]
        _chk(X, np.uint8, (q, self.o))
        out = np.zeros(q, dtype=np.int32)
        lib().otm_predict(ctypes.byref(self.cfg), _p(self.state), _p(X), ctypes.c_int64(q), _p(out))
        return out

    # ---- single pieces -----------------------------------------------------
    def neg_class(self, epoch, i, y):
        return int(lib().otm_neg_class(ctypes.byref(self.cfg), ctypes.c_uint32(epoch), ctypes.c_int64(i),
                                       ctypes.c_int32(y)))

    def gate(self, g, i, epoch, v, target):
        return int(lib().otm_gate(ctypes.byref(self.cfg), ctypes.c_int32(g), ctypes.c_int64(i),
                                  ctypes.c_uint32(epoch), ctypes.c_int32(v), ctypes.c_int(target)))

    def gate_regression(self, g, i, epoch, v, y):
        """0 no feedback, 1 Type I, 2 Type II."""
        return int(lib().otm_gate_regression(ctypes.byref(self.cfg), ctypes.c_int32(g), ctypes.c_int64(i),
                                             ctypes.c_uint32(epoch), ctypes.c_int32(v), ctypes.c_int32(y)))

    def threshold(self):
        return int(lib().otm_threshold(ctypes.byref(self.cfg)))

    def type1(self, st, lit, Cout, g, i, epoch):
        _chk(st, np.int32, (self.L,))
        _chk(lit, np.uint8, (self.L,))
        lib().otm_type1(ctypes.byref(self.cfg), _p(st), _p(lit), ctypes.c_int(Cout), ctypes.c_int32(g),
                        ctypes.c_int64(i), ctypes.c_uint32(epoch))

    def type2(self, st, lit, Cout):
        _chk(st, np.int32, (self.L,))
        _chk(lit, np.uint8, (self.L,))
        lib().otm_type2(ctypes.byref(self.cfg), _p(st), _p(lit), ctypes.c_int(Cout))

    # ---- training ------------------------------------------------------------
    def sync_tallies(self, X):
        q = X.shape[0]
        _chk(X, np.uint8, (q, self.o))
        tally = np.zeros((q, self.m), dtype=np.int32)
        ostar = np.zeros((self.C, q), dtype=np.uint8)
        lib().otm_sync_tallies(ctypes.byref(self.cfg), _p(self.state), _p(X), ctypes.c_int64(q), _p(tally),
                               _p(ostar))
        return tally, ostar

    def feedback_step(self, X, y, vhat, tally, ostar, epoch, i0, cnt):
        q = X.shape[0]
        _chk(X, np.uint8, (q, self.o)); _chk(y, np.int32, (q,))
        _chk(vhat, np.int32, (q, self.m)); _chk(tally, np.int32, (q, self.m))
        _chk(ostar, np.uint8, (self.C, q))
        fired = ctypes.c_int64(0)
        lib().otm_feedback_step(ctypes.byref(self.cfg), _p(self.state), _p(X), _p(y), ctypes.c_int64(q),
                                _p(vhat), _p(tally), _p(ostar), ctypes.c_uint32(epoch), ctypes.c_int64(i0),
                                ctypes.c_int64(cnt), ctypes.byref(fired))
        return fired.value

    def clause_outputs_subset(self, X, ids):
        q = X.shape[0]
        _chk(X, np.uint8, (q, self.o))
        ids = np.ascontiguousarray(ids, dtype=np.int32)
        out = np.zeros((len(ids), q), dtype=np.uint8)
        lib().otm_clause_outputs_subset(ctypes.byref(self.cfg), _p(self.state), _p(X), ctypes.c_int64(q), _p(ids),
                                        ctypes.c_int32(len(ids)), _p(out))
        return out

    def feedback_step_subset(self, X, y, vhat, ostar_sub, epoch, i0, cnt, ids):
        q = X.shape[0]
        ids = np.ascontiguousarray(ids, dtype=np.int32)
        _chk(X, np.uint8, (q, self.o)); _chk(y, np.int32, (q,))
        _chk(vhat, np.int32, (q, self.m)); _chk(ostar_sub, np.uint8, (len(ids), q))
        fired = ctypes.c_int64(0)
        lib().otm_feedback_step_subset(ctypes.byref(self.cfg), _p(self.state), _p(X), _p(y), ctypes.c_int64(q),
                                       _p(vhat), _p(ostar_sub), ctypes.c_uint32(epoch), ctypes.c_int64(i0),
                                       ctypes.c_int64(cnt), _p(ids), ctypes.c_int32(len(ids)), ctypes.byref(fired))
        return fired.value

    def async_epoch(self, X, y, tally, ostar, epoch, example_major=True):
        q = X.shape[0]
        _chk(X, np.uint8, (q, self.o)); _chk(y, np.int32, (q,))
        _chk(tally, np.int32, (q, self.m)); _chk(ostar, np.uint8, (self.C, q))
        lib().otm_async_epoch(ctypes.byref(self.cfg), _p(self.state), _p(X), _p(y), ctypes.c_int64(q),
                              _p(tally), _p(ostar), ctypes.c_uint32(epoch),
                              ctypes.c_int(1 if example_major else 0))

    def async_range(self, X, y, tally, ostar, epoch, i0, cnt, example_major=True):
        q = X.shape[0]
        _chk(X, np.uint8, (q, self.o)); _chk(y, np.int32, (q,))
        _chk(tally, np.int32, (q, self.m)); _chk(ostar, np.uint8, (self.C, q))
        lib().otm_async_range(ctypes.byref(self.cfg), _p(self.state), _p(X), _p(y), ctypes.c_int64(q),
                              _p(tally), _p(ostar), ctypes.c_uint32(epoch), ctypes.c_int64(i0),
                              ctypes.c_int64(cnt), ctypes.c_int(1 if example_major else 0))

    def sync_epoch(self, X, y, epoch):
        q = X.shape[0]
        _chk(X, np.uint8, (q, self.o)); _chk(y, np.int32, (q,))
        lib().otm_sync_epoch(ctypes.byref(self.cfg), _p(self.state), _p(X), _p(y), ctypes.c_int64(q),
                             ctypes.c_uint32(epoch))


def philox(ctr, key):
    c = (ctypes.c_uint32 * 4)(*ctr)
    k = (ctypes.c_uint32 * 2)(*key)
    out = (ctypes.c_uint32 * 4)()
    lib().otm_philox(c, k, out)
    return list(out)
