"""numpy/ctypes front end of the CPU oracle in ssd_oracle.c.

TEST INFRASTRUCTURE ONLY: imported by tests, the smoke check and the
cpu_baseline leg of the benchmark.  It holds no arithmetic of its own; every
number comes from the scalar loops of ssd_oracle.c, which follow Algorithm 1,
Algorithm 2, Eq. (server), Eq. (glu-update) and Secs. 3.2.1 / 3.3 of the
SSD-SGD paper.  The model is one flat array of n elements: every rule of the
method is element-wise, so the split into layer tensors does not change any
value.
"""
import ctypes as C

import numpy as np

from . import build as _build

KIND_WARMUP, KIND_WARMUP_LAST, KIND_DELAY, KIND_DELAY_PULL = 0, 1, 2, 3

_libs = {}


def _lib(sfx):
    if sfx not in _libs:
        _libs[sfx] = C.CDLL(_build.build()[sfx])
    return _libs[sfx]


def _state_struct(real):
    class State(C.Structure):
        _fields_ = [("K", C.c_int), ("k", C.c_int), ("W", C.c_int),
                    ("lr", real), ("m", real), ("wd", real),
                    ("lr_loc", real), ("alpha", real), ("beta", real),
                    ("wd_loc", real), ("rescale", real), ("pre_scale", real),
                    ("n", C.c_long), ("num", C.c_long),
                    ("loc_update", C.POINTER(C.c_long)),
                    ("w", C.c_void_p), ("mom", C.c_void_p),
                    ("wl", C.c_void_p), ("pre", C.c_void_p),
                    ("wloc", C.c_void_p)]
    return State


class Oracle:
    """State of the server and of K workers, advanced by ssd_oracle_step.

    mode "f64": plain oracle, binary64 state and arithmetic.
    mode "f32": GPU-order oracle, binary32, one rounding per operation.
    Hyper-parameters are given as Python floats and are first rounded to
    binary32 (the precision in which the library's configuration carries
    them), then widened to the mode's type.
    """

    def __init__(self, w0, K, k, W, lr, m, wd, lr_loc=None, alpha=2.0,
                 beta=0.5, wd_loc=None, rescale=None, exact_w_minus=False, mode="f64"):
        assert mode in ("f32", "f64")
        self.mode = mode
        self.dtype = np.float32 if mode == "f32" else np.float64
        self.real = C.c_float if mode == "f32" else C.c_double
        self.lib = _lib(mode)
        f32 = lambda x: float(np.float32(x))
        if lr_loc is None:
            lr_loc = f32(np.float32(4.0) * np.float32(lr))
        if wd_loc is None:
            wd_loc = wd
        if rescale is None:
            rescale = f32(1.0 / K)
        w0 = np.ascontiguousarray(np.asarray(w0).reshape(-1))
        n = w0.size
        self.K, self.k, self.W, self.n = int(K), int(k), int(W), n
        self.exact_w_minus = bool(exact_w_minus)
        self.w = w0.astype(self.dtype).copy()
        self.mom = np.zeros(n, self.dtype)
        self.wl = np.zeros((K, n), self.dtype)
        self.pre = np.zeros((K, n), self.dtype)
        self.wloc = np.zeros((K, n), self.dtype)
        self.loc_update = (C.c_long * K)()
        S = _state_struct(self.real)
        self.s = S(K=K, k=k, W=W, lr=f32(lr), m=f32(m), wd=f32(wd),
                   lr_loc=f32(lr_loc), alpha=f32(alpha), beta=f32(beta),
                   wd_loc=f32(wd_loc), rescale=f32(rescale), pre_scale=1.0, n=n, num=0,
                   loc_update=self.loc_update,
                   w=self.w.ctypes.data, mom=self.mom.ctypes.data,
                   wl=self.wl.ctypes.data, pre=self.pre.ctypes.data,
                   wloc=self.wloc.ctypes.data)
        self._step = getattr(self.lib, "ssd_oracle_step_" + mode)
        self._step.restype = C.c_int
        self._set_pre_scale()
        getattr(self.lib, "ssd_oracle_begin_" + mode)(C.byref(self.s))

    def _set_pre_scale(self):
        if self.exact_w_minus:
            f = getattr(self.lib, "ssd_oracle_pre_scale_" + self.mode)
            f.restype = self.real
            self.s.pre_scale = f(self.real(self.s.lr), self.real(self.s.wd))
        else:
            self.s.pre_scale = 1.0

    def _gptrs(self, grads):
        keep = [np.ascontiguousarray(np.asarray(g).reshape(-1), self.dtype)
                for g in grads]
        assert len(keep) == self.K and all(a.size == self.n for a in keep)
        arr = (C.c_void_p * self.K)(*[a.ctypes.data for a in keep])
        return keep, arr

    def step(self, grads):
        """One iteration of Algorithm 1 for all workers; returns its kind."""
        keep, arr = self._gptrs(grads)
        return self._step(C.byref(self.s), arr)

    def set_lr(self, lr, lr_loc):
        self.s.lr = float(np.float32(lr))
        self.s.lr_loc = float(np.float32(lr_loc))
        self._set_pre_scale()

    @property
    def num(self):
        return self.s.num

    @property
    def d(self):
        return self.loc_update[0]

    # piecewise entry points -------------------------------------------
    def server(self, grads):
        """Eq. (server) + momentum rule only; no schedule change."""
        keep, arr = self._gptrs(grads)
        f = getattr(self.lib, "ssd_oracle_server_" + self.mode)
        f.restype = None
        r = self.real
        f(C.c_long(self.n), C.c_int(self.K), arr, r(self.s.rescale),
          r(self.s.lr), r(self.s.m), r(self.s.wd),
          C.c_void_p(self.w.ctypes.data), C.c_void_p(self.mom.ctypes.data))

    def c_sync(self):
        f = getattr(self.lib, "ssd_oracle_c_sync_" + self.mode)
        f.restype = self.real
        r = self.real
        return f(r(self.s.lr), r(self.s.m), C.c_int(self.k))

    def glu(self, i, grad):
        """One call of Algorithm 2 for worker i."""
        g = np.ascontiguousarray(np.asarray(grad).reshape(-1), self.dtype)
        assert g.size == self.n
        f = getattr(self.lib, "ssd_oracle_glu_" + self.mode)
        f.restype = None
        r = self.real
        lu = C.c_long(self.loc_update[i])
        f(C.c_long(self.n), C.c_int(self.k), C.c_void_p(g.ctypes.data),
          C.c_void_p(self.wl[i].ctypes.data),
          C.c_void_p(self.pre[i].ctypes.data), C.byref(lu),
          r(self.c_sync()), r(self.s.pre_scale), r(self.s.lr_loc), r(self.s.alpha),
          r(self.s.beta), r(self.s.wd_loc))
        self.loc_update[i] = lu.value

    def pull(self, i):
        """Alg. 1 Pull for worker i: w_loc <- w', then w' <- w."""
        self.wloc[i] = self.wl[i]
        self.wl[i] = self.w
