"""Thin Python binding of the C boundary in include/tm.h.

Argument marshalling only: tensors are allocated with torch (device memory
and streams), their data pointers are handed to the library, every step of
the method runs in the HIP kernels.  Function names are the C names.  If the
HIP library is missing the first call raises; there is no CPU fallback.
"""
import ctypes
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libtm_hip.so")

TM_OK, TM_EINVAL, TM_ESTATE, TM_EHIP, TM_ELIMIT = 0, -1, -2, -3, -4

EXPORTS = [
    "tm_state_bytes", "tm_train_ws_bytes", "tm_create", "tm_destroy", "tm_bind_train", "tm_fit_epoch", "tm_fit_batch",
    "tm_class_sums", "tm_predict", "tm_infer_ws_bytes", "tm_class_sums_ws", "tm_predict_ws", "tm_predict_static", "tm_get_ta_state", "tm_set_ta_state", "tm_clause_outputs",
    "tm_sync_tallies", "tm_get_tallies", "tm_get_prev_outputs", "tm_feedback_step", "tm_train_chunk", "tm_set_epoch",
    "tm_get_epoch", "tm_set_clause_groups", "tm_eval_shares", "tm_read_counters", "tm_kernel_timing", "tm_read_kernel_timing", "tm_strerror", "tm_last_hip_error",
]


class tm_config(ctypes.Structure):
    _fields_ = [("n_classes", ctypes.c_int32), ("clauses_per_class", ctypes.c_int32),
                ("n_features", ctypes.c_int32), ("states_per_action", ctypes.c_int32),
                ("T", ctypes.c_int32), ("s", ctypes.c_double), ("seed", ctypes.c_uint64),
                ("device", ctypes.c_int32), ("boost_true_positive", ctypes.c_int32),
                ("regression", ctypes.c_int32)]


class TMError(RuntimeError):
    def __init__(self, code, what):
        self.code = code
        super().__init__("%s failed: %s (code %d)" % (what, strerror(code), code))


_lib = None


def lib():
    """Opens the HIP library (built in-tree by build.build_library)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("HIP library %s is missing: run __graft_entry__.build() first "
                               "(there is no CPU fallback)" % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        L.tm_strerror.restype = ctypes.c_char_p
        for name in EXPORTS:
            getattr(L, name)
        _lib = L
    return _lib


def strerror(code):
    return lib().tm_strerror(ctypes.c_int(code)).decode()


def _check(code, what):
    if code != TM_OK:
        raise TMError(code, what)


def _ptr(t, dtype=None):
    if t is None:
        return ctypes.c_void_p(0)
    assert t.is_cuda and t.is_contiguous(), "device tensor, contiguous"
    if dtype is not None:
        assert t.dtype == dtype, (t.dtype, dtype)
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def make_config(m, n, o, N, T, s, seed, device=0, boost=False, regression=False):
    return tm_config(int(m), int(n), int(o), int(N), int(T), float(s), int(seed), int(device), 1 if boost else 0,
                     1 if regression else 0)


def tm_state_bytes(cfg):
    out = ctypes.c_size_t(0)
    _check(lib().tm_state_bytes(ctypes.byref(cfg), ctypes.byref(out)), "tm_state_bytes")
    return out.value


def tm_train_ws_bytes(cfg, q):
    out = ctypes.c_size_t(0)
    _check(lib().tm_train_ws_bytes(ctypes.byref(cfg), ctypes.c_int64(q), ctypes.byref(out)), "tm_train_ws_bytes")
    return out.value


def tm_create(cfg, state_buf):
    h = ctypes.c_void_p(0)
    _check(lib().tm_create(ctypes.byref(cfg), _ptr(state_buf), _stream(), ctypes.byref(h)), "tm_create")
    return h


def tm_destroy(h):
    _check(lib().tm_destroy(h), "tm_destroy")


def tm_bind_train(h, X, y, ws):
    q = X.shape[0]
    _check(lib().tm_bind_train(h, _ptr(X, torch.int32), _ptr(y, torch.int32), ctypes.c_int64(q), _ptr(ws),
                               _stream()), "tm_bind_train")


def tm_fit_epoch(h):
    _check(lib().tm_fit_epoch(h, _stream()), "tm_fit_epoch")


def tm_fit_batch(h, i0, cnt):
    _check(lib().tm_fit_batch(h, ctypes.c_int64(i0), ctypes.c_int64(cnt), _stream()), "tm_fit_batch")


def tm_class_sums(h, X, sums):
    _check(lib().tm_class_sums(h, _ptr(X, torch.int32), ctypes.c_int64(X.shape[0]), _ptr(sums, torch.int32),
                               _stream()), "tm_class_sums")


def tm_predict(h, X, pred, sums_scratch):
    _check(lib().tm_predict(h, _ptr(X, torch.int32), ctypes.c_int64(X.shape[0]), _ptr(pred, torch.int32),
                            _ptr(sums_scratch, torch.int32), _stream()), "tm_predict")


def tm_infer_ws_bytes(cfg, q):
    out = ctypes.c_size_t(0)
    _check(lib().tm_infer_ws_bytes(ctypes.byref(cfg), ctypes.c_int64(q), ctypes.byref(out)), "tm_infer_ws_bytes")
    return out.value


def tm_class_sums_ws(h, X, sums, ws):
    _check(lib().tm_class_sums_ws(h, _ptr(X, torch.int32), ctypes.c_int64(X.shape[0]), _ptr(sums, torch.int32),
                                  _ptr(ws), _stream()), "tm_class_sums_ws")


def tm_predict_ws(h, X, pred, sums_scratch, ws):
    _check(lib().tm_predict_ws(h, _ptr(X, torch.int32), ctypes.c_int64(X.shape[0]), _ptr(pred, torch.int32),
                               _ptr(sums_scratch, torch.int32), _ptr(ws), _stream()), "tm_predict_ws")


def tm_predict_static(h, X, pred):
    _check(lib().tm_predict_static(h, _ptr(X, torch.int32), ctypes.c_int64(X.shape[0]), _ptr(pred, torch.int32),
                                   _stream()), "tm_predict_static")


def tm_get_ta_state(h, out):
    _check(lib().tm_get_ta_state(h, _ptr(out, torch.uint8), _stream()), "tm_get_ta_state")


def tm_set_ta_state(h, inp):
    _check(lib().tm_set_ta_state(h, _ptr(inp, torch.uint8), _stream()), "tm_set_ta_state")


def tm_clause_outputs(h, X, bits):
    _check(lib().tm_clause_outputs(h, _ptr(X, torch.int32), ctypes.c_int64(X.shape[0]), _ptr(bits, torch.int32),
                                   _stream()), "tm_clause_outputs")


def tm_sync_tallies(h):
    _check(lib().tm_sync_tallies(h, _stream()), "tm_sync_tallies")


def tm_get_tallies(h, out):
    _check(lib().tm_get_tallies(h, _ptr(out, torch.int32), _stream()), "tm_get_tallies")


def tm_get_prev_outputs(h, bits):
    _check(lib().tm_get_prev_outputs(h, _ptr(bits, torch.int32), _stream()), "tm_get_prev_outputs")


def tm_feedback_step(h, snapshot, i0, cnt):
    _check(lib().tm_feedback_step(h, _ptr(snapshot, torch.int32), ctypes.c_int64(i0), ctypes.c_int64(cnt),
                                  _stream()), "tm_feedback_step")


def tm_train_chunk(h):
    c = ctypes.c_int64(0)
    _check(lib().tm_train_chunk(h, ctypes.byref(c)), "tm_train_chunk")
    return c.value


def tm_set_epoch(h, epoch):
    _check(lib().tm_set_epoch(h, ctypes.c_uint32(epoch)), "tm_set_epoch")


def tm_set_clause_groups(h, groups):
    _check(lib().tm_set_clause_groups(h, ctypes.c_int32(groups)), "tm_set_clause_groups")


def tm_eval_shares(cfg, q):
    """(shares, clauses per share) of the literal-list evaluation for q examples."""
    S, chunk = ctypes.c_int32(0), ctypes.c_int32(0)
    _check(lib().tm_eval_shares(ctypes.byref(cfg), ctypes.c_int64(q), ctypes.byref(S), ctypes.byref(chunk)),
           "tm_eval_shares")
    return S.value, chunk.value


def tm_get_epoch(h):
    e = ctypes.c_uint32(0)
    _check(lib().tm_get_epoch(h, ctypes.byref(e)), "tm_get_epoch")
    return e.value


TIMED_TRAIN, TIMED_PRECALC, TIMED_INFER, TIMED_ALL = 1, 2, 4, 7


def tm_kernel_timing(h, kinds):
    """kinds: bit mask of TIMED_TRAIN | TIMED_PRECALC | TIMED_INFER (True = all three, False / 0 = off)."""
    mask = TIMED_ALL if kinds is True else int(kinds or 0)
    _check(lib().tm_kernel_timing(h, ctypes.c_int(mask)), "tm_kernel_timing")


def tm_read_kernel_timing(h):
    """{"train" | "precalc" | "infer": (ms, launches)} since the last read."""
    ms = (ctypes.c_double * 3)()
    n = (ctypes.c_int64 * 3)()
    _check(lib().tm_read_kernel_timing(h, ms, n), "tm_read_kernel_timing")
    return {"train": (ms[0], n[0]), "precalc": (ms[1], n[1]), "infer": (ms[2], n[2])}


def tm_read_counters(h):
    out = (ctypes.c_uint64 * 10)()
    _check(lib().tm_read_counters(h, out, _stream()), "tm_read_counters")
    return {"pairs": out[0], "fired": out[1], "type1": out[2], "tally_changes": out[3],
            "candidates": out[4], "type2_active": out[5], "blocks_evaluated": out[6],
            "gate_draws": out[7], "blocks_listed": out[8], "automata_moved": out[9]}


class TsetlinMachine:
    """Convenience owner of the device buffers around one tm_handle.

    Bit-packed uint32 data travels in int32 tensors (torch has no full uint32
    support); the bit patterns are what matters."""

    def __init__(self, m, n, o, N, T, s, seed, device=0, boost=False, regression=False):
        self.m, self.n, self.o, self.N, self.T, self.s, self.seed = m, n, o, N, T, float(s), seed
        self.C, self.L, self.Wf = m * n, 2 * o, (o + 31) // 32
        self.dev = torch.device("cuda", device)
        self.cfg = make_config(m, n, o, N, T, s, seed, device, boost, regression)
        with torch.cuda.device(self.dev):
            self.state_buf = torch.empty(tm_state_bytes(self.cfg), dtype=torch.uint8, device=self.dev)
            self.h = tm_create(self.cfg, self.state_buf)
        self.ws = None
        self.infer_ws = None
        self.X = self.y = None

    def close(self):
        if self.h is not None:
            torch.cuda.synchronize(self.dev)
            tm_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- data ----------------------------------------------------------------
    def to_device_bits(self, packed_u32_numpy):
        """numpy uint32 [q][Wf] -> int32 device tensor with the same bits."""
        import numpy as np
        a = np.ascontiguousarray(packed_u32_numpy, dtype=np.uint32).view(np.int32)
        return torch.from_numpy(a).to(self.dev)

    def bind_train(self, X, y):
        """X int32 device [q][Wf] (bit-packed), y int32 device [q]."""
        q = X.shape[0]
        assert X.shape[1] == self.Wf
        with torch.cuda.device(self.dev):
            self.ws = torch.empty(tm_train_ws_bytes(self.cfg, q), dtype=torch.uint8, device=self.dev)
            self.X, self.y, self.q = X, y, q
            tm_bind_train(self.h, X, y, self.ws)

    # -- training --------------------------------------------------------------
    def fit_epoch(self):
        with torch.cuda.device(self.dev):
            tm_fit_epoch(self.h)

    def fit_batch(self, i0, cnt):
        with torch.cuda.device(self.dev):
            tm_fit_batch(self.h, i0, cnt)

    def feedback_step(self, snapshot, i0, cnt):
        with torch.cuda.device(self.dev):
            tm_feedback_step(self.h, snapshot, i0, cnt)

    def sync_tallies(self):
        with torch.cuda.device(self.dev):
            tm_sync_tallies(self.h)

    def tallies(self):
        out = torch.empty((self.q, self.m), dtype=torch.int32, device=self.dev)
        with torch.cuda.device(self.dev):
            tm_get_tallies(self.h, out)
        return out

    def prev_outputs(self):
        out = torch.empty((self.C, (self.q + 31) // 32), dtype=torch.int32, device=self.dev)
        with torch.cuda.device(self.dev):
            tm_get_prev_outputs(self.h, out)
        return out

    def counters(self):
        with torch.cuda.device(self.dev):
            return tm_read_counters(self.h)

    # -- inference -------------------------------------------------------------
    def _infer_ws(self, q):
        """Workspace of the literal-list inference calls, kept and grown as needed."""
        need = tm_infer_ws_bytes(self.cfg, q)
        if self.infer_ws is None or self.infer_ws.numel() < need:
            self.infer_ws = torch.empty(need, dtype=torch.uint8, device=self.dev)
        return self.infer_ws

    def class_sums(self, X, lists=True):
        """lists=True: tm_class_sums_ws (clauses evaluated from their literal lists);
        lists=False: tm_class_sums (from their include masks, no workspace)."""
        out = torch.empty((X.shape[0], self.m), dtype=torch.int32, device=self.dev)
        with torch.cuda.device(self.dev):
            if lists:
                tm_class_sums_ws(self.h, X, out, self._infer_ws(X.shape[0]))
            else:
                tm_class_sums(self.h, X, out)
        return out

    def predict(self, X, lists=True):
        pred = torch.empty((X.shape[0],), dtype=torch.int32, device=self.dev)
        scratch = torch.empty((X.shape[0], self.m), dtype=torch.int32, device=self.dev)
        with torch.cuda.device(self.dev):
            if lists:
                tm_predict_ws(self.h, X, pred, scratch, self._infer_ws(X.shape[0]))
            else:
                tm_predict(self.h, X, pred, scratch)
        return pred

    def clause_outputs(self, X):
        out = torch.empty((self.C, (X.shape[0] + 31) // 32), dtype=torch.int32, device=self.dev)
        with torch.cuda.device(self.dev):
            tm_clause_outputs(self.h, X, out)
        return out

    # -- state -----------------------------------------------------------------
    def get_ta_state(self):
        out = torch.empty((self.C, self.L), dtype=torch.uint8, device=self.dev)
        with torch.cuda.device(self.dev):
            tm_get_ta_state(self.h, out)
        return out

    def set_ta_state(self, t):
        assert tuple(t.shape) == (self.C, self.L)
        with torch.cuda.device(self.dev):
            tm_set_ta_state(self.h, t)
