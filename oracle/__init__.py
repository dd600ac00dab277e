"""ctypes binding of the CPU oracle (test infrastructure, not the product).

Only tests, ``__graft_entry__.smoke()`` and the CPU-baseline leg of ``bench.py``
import this package.  It builds ``laa_oracle.c`` with gcc on first use:
``liblaa_oracle_f64.so`` (the oracle proper, fp64) and ``liblaa_oracle_f32.so``
(the same statements in fp32, used to calibrate tolerances).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "laa_oracle.c")

GEN_QUADRATIC, GEN_NOISE = 1, 2
OFF_NONE, OFF_ARRAY, OFF_PHILOX = 0, 1, 2
STREAM_OFFSET, STREAM_NOISE = 2, 3
OK, EINVAL, ESYNCDUE, EMODE = 0, -1, -3, -5


def lib_path(precision: str = "f64") -> str:
    return os.path.join(_HERE, f"liblaa_oracle_{precision}.so")


def build(precision: str = "f64", out: str | None = None, defines: tuple[str, ...] = (), force: bool = False) -> str:
    """Compile the oracle.  ``defines`` lets a test plant a mistake (ORA_PLANT_*)."""
    out = out or lib_path(precision)
    if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(_SRC):
        return out
    real = {"f64": "double", "f32": "float"}[precision]
    cmd = ["gcc", "-std=c11", "-O2", "-ffp-contract=off", "-fno-fast-math", "-shared", "-fPIC",
           f"-DORA_REAL={real}", *[f"-D{d}" for d in defines], _SRC, "-o", out + ".tmp", "-lm"]
    subprocess.run(cmd, check=True)
    os.replace(out + ".tmp", out)
    return out


class _Lib:
    def __init__(self, path: str):
        L = C.CDLL(path)
        self.L = L
        self.real_bytes = L.ora_real_bytes()
        self.np_real = np.float64 if self.real_bytes == 8 else np.float32
        rp = C.c_void_p
        L.ora_create.restype = C.c_void_p
        L.ora_create.argtypes = [C.c_int64, C.c_int32, C.c_int32, C.c_double, C.c_double, C.c_double]
        L.ora_destroy.argtypes = [C.c_void_p]
        L.ora_destroy.restype = None
        L.ora_set_columns.argtypes = [C.c_void_p, rp]
        L.ora_set_warmup.argtypes = [C.c_void_p, C.c_int64]
        L.ora_init_state.argtypes = [C.c_void_p, rp]
        L.ora_local_step_dense.argtypes = [C.c_void_p, rp]
        L.ora_step_dense.argtypes = [C.c_void_p, rp]
        L.ora_adagrad_step_dense.argtypes = [C.c_void_p, rp]
        L.ora_localsgd_step_dense.argtypes = [C.c_void_p, rp]
        L.ora_sync.argtypes = [C.c_void_p]
        L.ora_set_generator.argtypes = [C.c_void_p, C.c_int, C.c_uint64, rp, rp, rp, C.c_int, C.c_double, C.c_double]
        L.ora_gradient.argtypes = [C.c_void_p, C.c_int64, rp]
        L.ora_local_step_gen.argtypes = [C.c_void_p]
        L.ora_step_gen.argtypes = [C.c_void_p]
        L.ora_local_step_sparse.argtypes = [C.c_void_p, rp, rp, C.c_int32, C.c_int32]
        L.ora_step_sparse.argtypes = [C.c_void_p, rp, rp, C.c_int32, C.c_int32]
        L.ora_dirty_rows.argtypes = [C.c_void_p, rp, C.c_int64]
        L.ora_dirty_rows.restype = C.c_int64
        for f in ("ora_x", "ora_acc", "ora_snap"):
            getattr(L, f).argtypes = [C.c_void_p]
            getattr(L, f).restype = C.c_void_p
        L.ora_t.argtypes = [C.c_void_p]
        L.ora_t.restype = C.c_int64
        L.ora_steps_since_sync.argtypes = [C.c_void_p]
        L.ora_steps_since_sync.restype = C.c_int32
        L.ora_diagnostics.argtypes = [C.c_void_p, C.POINTER(C.c_double)]
        L.ora_philox4x32_10.argtypes = [rp, rp, rp]
        L.ora_philox4x32_10.restype = None
        L.ora_normals4.argtypes = [C.c_uint64, C.c_uint32, C.c_uint64, C.c_uint32, C.c_uint64, rp]
        L.ora_normals4.restype = None


_libs: dict[str, _Lib] = {}


def load(precision: str = "f64", path: str | None = None) -> _Lib:
    key = path or precision
    if key not in _libs:
        _libs[key] = _Lib(path or build(precision))
    return _libs[key]


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


class Oracle:
    """Local AdaAlter state machine on host arrays (Algorithm 3 of the paper)."""

    def __init__(self, d, W, H, eta, eps, b0=1.0, precision="f64", lib: _Lib | None = None):
        self.lib = lib or load(precision)
        self.L = self.lib.L
        self.dt = self.lib.np_real
        self.d, self.W, self.H = int(d), int(W), int(H)
        self.h = self.L.ora_create(self.d, self.W, self.H, float(eta), float(eps), float(b0))
        if not self.h:
            raise ValueError("ora_create rejected the arguments")

    def __del__(self):
        h = getattr(self, "h", None)
        if h:
            self.L.ora_destroy(h)
            self.h = None

    def _real(self, a, shape=None):
        if a is None:
            return None
        a = np.ascontiguousarray(a, dtype=self.dt)
        if shape is not None and a.shape != shape:
            raise ValueError(f"expected shape {shape}, got {a.shape}")
        return a

    @staticmethod
    def _chk(rc):
        if rc != OK:
            raise RuntimeError(f"oracle call failed with code {rc}")

    def set_columns(self, col):
        col = np.ascontiguousarray(col, dtype=np.int64)
        assert col.shape == (self.d,)
        self._chk(self.L.ora_set_columns(self.h, _ptr(col)))

    def set_warmup(self, warmup_steps):
        self._chk(self.L.ora_set_warmup(self.h, int(warmup_steps)))

    def init_state(self, x0=None):
        x0 = self._real(x0, (self.d,))
        self._chk(self.L.ora_init_state(self.h, _ptr(x0)))

    def set_generator(self, mode, seed, a, xstar=None, off=None, off_mode=OFF_NONE, noise_scale=0.1, off_scale=0.1):
        a = self._real(a, (self.d,))
        xstar = self._real(xstar, (self.d,))
        off = self._real(off, (self.W, self.d))
        self._chk(self.L.ora_set_generator(self.h, int(mode), int(seed), _ptr(a), _ptr(xstar), _ptr(off),
                                           int(off_mode), float(noise_scale), float(off_scale)))

    def gradient(self, t):
        G = np.empty((self.W, self.d), dtype=self.dt)
        self._chk(self.L.ora_gradient(self.h, int(t), _ptr(G)))
        return G

    def local_step_dense(self, G, rc_only=False):
        G = self._real(G, (self.W, self.d))
        rc = self.L.ora_local_step_dense(self.h, _ptr(G))
        if rc_only:
            return rc
        self._chk(rc)

    def step_dense(self, G):
        G = self._real(G, (self.W, self.d))
        self._chk(self.L.ora_step_dense(self.h, _ptr(G)))

    def adagrad_step_dense(self, G):
        G = self._real(G, (self.W, self.d))
        self._chk(self.L.ora_adagrad_step_dense(self.h, _ptr(G)))

    def localsgd_step_dense(self, G):
        G = self._real(G, (self.W, self.d))
        self._chk(self.L.ora_localsgd_step_dense(self.h, _ptr(G)))

    def local_step_gen(self):
        self._chk(self.L.ora_local_step_gen(self.h))

    def step_gen(self):
        self._chk(self.L.ora_step_gen(self.h))

    def _sparse_args(self, idx, vals, row_len):
        idx = np.ascontiguousarray(idx, dtype=np.int32)
        assert idx.ndim == 2 and idx.shape[0] == self.W
        k = idx.shape[1]
        vals = self._real(vals, (self.W, k, row_len))
        return idx, vals, k

    def local_step_sparse(self, idx, vals, row_len):
        idx, vals, k = self._sparse_args(idx, vals, row_len)
        self._chk(self.L.ora_local_step_sparse(self.h, _ptr(idx), _ptr(vals), k, int(row_len)))

    def step_sparse(self, idx, vals, row_len):
        idx, vals, k = self._sparse_args(idx, vals, row_len)
        self._chk(self.L.ora_step_sparse(self.h, _ptr(idx), _ptr(vals), k, int(row_len)))

    def dirty_rows(self):
        n = self.L.ora_dirty_rows(self.h, None, 0)
        out = np.empty(n, dtype=np.int32)
        self.L.ora_dirty_rows(self.h, _ptr(out), n)
        return out

    def sync(self):
        self._chk(self.L.ora_sync(self.h))

    def diagnostics(self):
        out = (C.c_double * 3)()
        self._chk(self.L.ora_diagnostics(self.h, out))
        return tuple(out)

    def _view(self, fn, shape):
        p = fn(self.h)
        n = int(np.prod(shape))
        buf = (C.c_byte * (n * self.lib.real_bytes)).from_address(p)
        return np.frombuffer(buf, dtype=self.dt).reshape(shape)

    @property
    def x(self):
        return self._view(self.L.ora_x, (self.W, self.d)).copy()

    @property
    def acc(self):
        return self._view(self.L.ora_acc, (self.W, self.d)).copy()

    @property
    def snap(self):
        return self._view(self.L.ora_snap, (self.d,)).copy()

    @property
    def t(self):
        return self.L.ora_t(self.h)

    @property
    def steps_since_sync(self):
        return self.L.ora_steps_since_sync(self.h)


def philox4x32_10(ctr, key, lib: _Lib | None = None):
    lib = lib or load()
    ctr = np.ascontiguousarray(ctr, dtype=np.uint32)
    key = np.ascontiguousarray(key, dtype=np.uint32)
    out = np.empty(4, dtype=np.uint32)
    lib.L.ora_philox4x32_10(_ptr(ctr), _ptr(key), _ptr(out))
    return out


def normals4(seed, stream, q, w, t, lib: _Lib | None = None):
    lib = lib or load()
    out = np.empty(4, dtype=lib.np_real)
    lib.L.ora_normals4(int(seed), int(stream), int(q), int(w), int(t), _ptr(out))
    return out
