"""Thin ctypes binding of the C-ABI library (``include/laa.h``): argument marshalling only.

PyTorch is used for device memory and the stream handle, nothing else; every
step of the method runs in the library's kernels.  There is no CPU fallback:
if ``liblaa.so`` is missing this module raises on first use.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# LAA_LIB names another build of the same library (for comparing builds); the default is the in-tree one.
LIB_PATH = os.environ.get("LAA_LIB") or os.path.join(_HERE, "liblaa.so")

OK, EINVAL, ENOTATTACHED, ESYNCDUE, EALIGN, EMODE, EHIP, ENODEVICE = 0, -1, -2, -3, -4, -5, -6, -7
GEN_QUADRATIC, GEN_NOISE = 1, 2
OFF_NONE, OFF_ARRAY, OFF_PHILOX = 0, 1, 2
ALGO_LOCAL_ADAALTER, ALGO_DIST_ADAGRAD, ALGO_LOCAL_SGD = 0, 1, 2

EXPORTS = [
    "laa_last_error", "laa_create", "laa_destroy", "laa_set_b0", "laa_set_warmup", "laa_set_algorithm",
    "laa_set_tile", "laa_set_lazy_replicas", "laa_set_sparse_coalesce", "laa_materialize", "laa_attach", "laa_attach_pitched", "laa_init_state", "laa_local_step_dense", "laa_set_generator",
    "laa_local_step_gen", "laa_run_periods_gen", "laa_get_replay_count", "laa_generate_gradient", "laa_local_step_sparse", "laa_sync", "laa_sync_static", "laa_step_dense",
    "laa_step_gen", "laa_step_sparse", "laa_get_counters", "laa_set_counters", "laa_set_shard", "laa_get_dirty_rows", "laa_diagnostics", "laa_bytes_moved",
    "laa_spread_alloc", "laa_spread_free", "laa_pool_create", "laa_pool_trim", "laa_pool_free", "laa_debug_philox", "laa_debug_copy",
]

_lib = None


class LaaError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"laa error {code}: {msg}")
        self.code = code


def lib():
    """Load liblaa.so (built by ``python -m paper_1911_09030_amd.build``); no fallback."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_1911_09030_amd.build` "
                          "(there is no CPU fallback)")
    L = C.CDLL(LIB_PATH)
    vp, i32, i64, u64, f32, f64 = C.c_void_p, C.c_int32, C.c_int64, C.c_uint64, C.c_float, C.c_double
    L.laa_last_error.restype = C.c_char_p
    L.laa_last_error.argtypes = []
    sig = {
        "laa_create": [i64, i32, i32, f64, f64, C.POINTER(vp)],
        "laa_destroy": [vp],
        "laa_set_b0": [vp, f64],
        "laa_set_warmup": [vp, i64],
        "laa_set_algorithm": [vp, i32],
        "laa_set_tile": [vp, i32],
        "laa_set_lazy_replicas": [vp, i32],
        "laa_materialize": [vp],
        "laa_attach": [vp, vp, vp, vp, vp],
        "laa_attach_pitched": [vp, vp, vp, vp, i64, vp],
        "laa_init_state": [vp, vp],
        "laa_local_step_dense": [vp, vp],
        "laa_set_generator": [vp, i32, u64, vp, vp, vp, i32, f32, f32],
        "laa_local_step_gen": [vp],
        "laa_generate_gradient": [vp, vp],
        "laa_local_step_sparse": [vp, vp, vp, i32, i32],
        "laa_sync": [vp],
        "laa_sync_static": [vp],
        "laa_step_dense": [vp, vp],
        "laa_step_gen": [vp],
        "laa_step_sparse": [vp, vp, vp, i32, i32],
        "laa_get_counters": [vp, C.POINTER(i64), C.POINTER(i32), C.POINTER(i64)],
        "laa_set_counters": [vp, i64, i32],
        "laa_run_periods_gen": [vp, i32],
        "laa_get_replay_count": [vp, C.POINTER(i64)],
        "laa_set_sparse_coalesce": [vp, i32],
        "laa_set_shard": [vp, i64, i32],
        "laa_get_dirty_rows": [vp, vp, i64, C.POINTER(i64)],
        "laa_diagnostics": [vp, C.POINTER(C.c_double)],
        "laa_bytes_moved": [vp, C.POINTER(u64), C.POINTER(u64)],
        "laa_spread_alloc": [i32, i64, i64, C.POINTER(vp), C.POINTER(i64)],
        "laa_spread_free": [vp],
        "laa_pool_create": [i64, i64, C.POINTER(vp), C.POINTER(i64), C.POINTER(i64)],
        "laa_pool_trim": [vp, i32, C.POINTER(i64), C.POINTER(i64)],
        "laa_pool_free": [vp],
        "laa_debug_philox": [vp, vp, vp],
        "laa_debug_copy": [vp, vp, i64, vp],
    }
    for name, argtypes in sig.items():
        fn = getattr(L, name)
        fn.argtypes = argtypes
        fn.restype = C.c_int
    _lib = L
    return L


def _check(rc):
    if rc != OK:
        raise LaaError(rc, lib().laa_last_error().decode())


def _dev_ptr(t, dtype=None):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous device tensor")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"expected dtype {dtype}, got {t.dtype}")
    return C.c_void_p(t.data_ptr())


class _DeviceArray:
    """A strided view of device memory that PyTorch can adopt through the CUDA array interface."""

    def __init__(self, ptr, shape, strides_bytes, owner):
        self.__cuda_array_interface__ = {"shape": tuple(shape), "typestr": "<f4", "data": (int(ptr), False),
                                         "version": 3, "strides": tuple(strides_bytes)}
        self._owner = owner


class SpreadAllocation:
    """Device memory from laa_spread_alloc; freed when the last reference goes away (or by close())."""

    def __init__(self, n_arrays, array_bytes, distance_bytes):
        base, dist = C.c_void_p(), C.c_int64()
        self._free = lib().laa_spread_free          # kept here: module globals may be gone when __del__ runs at exit
        _check(lib().laa_spread_alloc(int(n_arrays), int(array_bytes), int(distance_bytes), C.byref(base), C.byref(dist)))
        self.base, self.distance_bytes, self.n_arrays = base.value, dist.value, int(n_arrays)
        self._base_arg = C.c_void_p(base.value)

    def close(self):
        if getattr(self, "base", None):
            self._free(self._base_arg)
            self.base = None

    __del__ = close


class Pool:
    """Device memory from laa_pool_create: one address range backed by separately created chunks, so that the part a
    caller ends up using can be kept and the rest released (trim).  Tensors are views at element offsets."""

    def __init__(self, nbytes, chunk_bytes=1 << 30, device="cuda:0"):
        base, total, chunk = C.c_void_p(), C.c_int64(), C.c_int64()
        self._free = lib().laa_pool_free
        self.device = device
        _check(lib().laa_pool_create(int(nbytes), int(chunk_bytes), C.byref(base), C.byref(total), C.byref(chunk)))
        self.base, self.nbytes, self.chunk_bytes = base.value, total.value, chunk.value
        self._base_arg = C.c_void_p(base.value)

    def tensor(self, offset, shape, strides=None):
        """float32 view: `offset` and `strides` in elements."""
        import torch
        shape = tuple(int(v) for v in shape)
        if strides is None:
            strides, acc = [], 1
            for n in reversed(shape):
                strides.insert(0, acc)
                acc *= n
        last = int(offset) + sum((n - 1) * int(st) for n, st in zip(shape, strides))
        if offset < 0 or (last + 1) * 4 > self.nbytes:
            raise ValueError("view outside the pool")
        return torch.as_tensor(_DeviceArray(self.base + 4 * int(offset), shape, [4 * int(st) for st in strides], self),
                               device=self.device)

    def trim(self, ranges):
        """Keep only the chunks touched by the (offset, length) element ranges; the rest is released."""
        n = len(ranges)
        offs = (C.c_int64 * n)(*[4 * int(o) for o, _ in ranges])
        lens = (C.c_int64 * n)(*[4 * int(l) for _, l in ranges])
        _check(lib().laa_pool_trim(self._base_arg, n, offs, lens))

    def close(self):
        if getattr(self, "base", None):
            self._free(self._base_arg)
            self.base = None

    __del__ = close


def spread_arrays(d, W, n_matrices, n_vectors, row_distance, device="cuda:0", hold_gaps=False):
    """``n_matrices`` arrays [W][d] and ``n_vectors`` arrays [d] whose rows all start ``row_distance`` elements
    apart (less if W * n_matrices + n_vectors such rows would not fit into 90 % of the free device memory).
    Returns (backing, matrices, vectors, pitch); every matrix has row pitch ``pitch``; keep ``backing`` alive as
    long as the tensors are used.

    Why: on MI355X a thread's 2W read-modify-write streams mostly run faster when the arrays streamed together
    span most of the HBM address range (d = 4e8, W = 8: 8.7-8.9 ms per step with the arrays 10 GB apart against
    8.8-9.8 ms for ordinary packed tensors).  placement.tune over a Pool finds a good placement by measurement
    instead (8.7 ms), which is what bench.py uses.

    Default: laa_spread_alloc, which maps only the arrays themselves (the address range between them is
    reserved but unmapped, so it costs no device memory; never touch it).  hold_gaps=True: one ordinary
    PyTorch allocation, gaps included."""
    import torch
    d, W, rd = int(d), int(W), int(row_distance)
    n = W * int(n_matrices) + int(n_vectors)
    free = torch.cuda.mem_get_info(device)[0]
    rd = min(rd, int(0.9 * free / n) // 4)
    rd -= rd % 4
    if rd < d:
        raise ValueError(f"{n} arrays of {d} elements cannot be spread over {free / 1e9:.0f} GB of free memory")
    if hold_gaps:
        backing = torch.empty(n * rd, dtype=torch.float32, device=device)
        rows = backing.view(n, rd)
        mats = [rows[m * W:(m + 1) * W, :d] for m in range(n_matrices)]
        vecs = [rows[n_matrices * W + v, :d] for v in range(n_vectors)]
        return backing, mats, vecs, rd
    backing = SpreadAllocation(n, d * 4, rd * 4)
    db, base = backing.distance_bytes, backing.base

    def adopt(first, rows):
        shape, strides = ((rows, d), (db, 4)) if rows else ((d,), (4,))
        return torch.as_tensor(_DeviceArray(base + first * db, shape, strides, backing), device=device)

    mats = [adopt(m * W, W) for m in range(n_matrices)]
    vecs = [adopt(n_matrices * W + v, 0) for v in range(n_vectors)]
    return backing, mats, vecs, db // 4


def spread_buffers(d, W, row_distance, device="cuda:0", hold_gaps=False):
    """The 2W + 3 arrays of a dense quadratic workload through spread_arrays: x rows, then acc rows, then snap, a,
    xstar.  Returns (backing, x, acc, snap, a, xstar, pitch)."""
    if int(row_distance) < int(d) or int(row_distance) % 4:
        raise ValueError("row_distance must be >= d and a multiple of 4")
    backing, (x, acc), (snap, a, xstar), pitch = spread_arrays(d, W, 2, 3, row_distance, device, hold_gaps)
    return backing, x, acc, snap, a, xstar, pitch


class LocalAdaAlter:
    """One optimizer state (x, acc [W][d]; snap [d]) on the current device and stream.

    Method names mirror the C entry points without the ``laa_`` prefix.  With ``pitch`` > d the
    rows of x, acc and of every [W][.] array passed in are ``pitch`` elements apart
    (``self.x`` / ``self.acc`` are then [W][d] views of [W][pitch] buffers, and ``rows()`` makes
    such a buffer for gradients and offsets).
    """

    def __init__(self, d, W, H, eta, eps, b0=None, device="cuda:0", x=None, acc=None, snap=None, stream=None,
                 pitch=None):
        import torch
        self.torch = torch
        self.L = lib()
        self.d, self.W, self.H = int(d), int(W), int(H)
        h = C.c_void_p()
        _check(self.L.laa_create(self.d, self.W, self.H, float(eta), float(eps), C.byref(h)))
        self.h = h
        if b0 is not None:
            _check(self.L.laa_set_b0(self.h, float(b0)))
        self.device = torch.device(device)
        f = dict(dtype=torch.float32, device=self.device)
        self.pitch = int(pitch) if pitch else (x.stride(0) if x is not None and x.dim() == 2 else self.d)
        self.x = x if x is not None else self.rows()
        self.acc = acc if acc is not None else self.rows()
        self.snap = snap if snap is not None else torch.empty((self.d,), **f)
        self.stream = stream if stream is not None else torch.cuda.current_stream(self.device)
        self._keep = []
        _check(self.L.laa_attach_pitched(self.h, self._rows_ptr(self.x), self._rows_ptr(self.acc),
                                         _dev_ptr(self.snap, torch.float32), self.pitch,
                                         C.c_void_p(self.stream.cuda_stream)))

    def attach(self, x, acc, snap):
        """Hand other state arrays (same shapes, same row pitch) to the handle."""
        for t, shape in ((x, (self.W, self.d)), (acc, (self.W, self.d)), (snap, (self.d,))):
            if tuple(t.shape) != shape:
                raise ValueError(f"expected an array of shape {shape}, got {tuple(t.shape)}")
        if x.stride(0) != self.pitch or acc.stride(0) != self.pitch:
            raise ValueError(f"rows must be {self.pitch} elements apart")
        self.x, self.acc, self.snap = x, acc, snap
        _check(self.L.laa_attach_pitched(self.h, self._rows_ptr(self.x), self._rows_ptr(self.acc),
                                         _dev_ptr(self.snap, self.torch.float32), self.pitch,
                                         C.c_void_p(self.stream.cuda_stream)))

    def rows(self, src=None):
        """A [W][d] device array whose rows are ``pitch`` apart (a view of a [W][pitch] buffer), optionally
        filled from ``src`` (a [W][d] tensor)."""
        torch = self.torch
        buf = torch.empty((self.W, self.pitch), dtype=torch.float32, device=self.device)
        view = buf[:, :self.d]
        if src is not None:
            view.copy_(src)
        return view

    def _rows_ptr(self, t):
        if t is None:
            return None
        if (not t.is_cuda or t.dtype != self.torch.float32 or t.shape != (self.W, self.d) or t.stride(1) != 1
                or (self.W > 1 and t.stride(0) != self.pitch)):
            raise ValueError(f"expected a float32 device array [W={self.W}][d={self.d}] with row pitch {self.pitch}")
        return C.c_void_p(t.data_ptr())

    def close(self):
        if getattr(self, "h", None):
            self.L.laa_destroy(self.h)
            self.h = None

    __del__ = close

    # configuration -------------------------------------------------------------------------
    def set_warmup(self, warmup_steps):
        _check(self.L.laa_set_warmup(self.h, int(warmup_steps)))

    def set_algorithm(self, algo):
        _check(self.L.laa_set_algorithm(self.h, int(algo)))

    def set_tile(self, workers_per_batch):
        _check(self.L.laa_set_tile(self.h, int(workers_per_batch)))

    def set_lazy_replicas(self, on=True):
        _check(self.L.laa_set_lazy_replicas(self.h, 1 if on else 0))

    def materialize(self):
        _check(self.L.laa_materialize(self.h))

    def init_state(self, x0=None):
        _check(self.L.laa_init_state(self.h, _dev_ptr(x0, self.torch.float32)))

    def set_generator(self, mode, seed, a, xstar=None, off=None, off_mode=OFF_NONE, noise_scale=0.1, off_scale=0.1):
        f32 = self.torch.float32
        self._keep = [a, xstar, off]       # the library reads these arrays on every generator step
        _check(self.L.laa_set_generator(self.h, int(mode), int(seed), _dev_ptr(a, f32), _dev_ptr(xstar, f32),
                                        self._rows_ptr(off), int(off_mode), float(noise_scale), float(off_scale)))

    # steps ---------------------------------------------------------------------------------
    def local_step_dense(self, grads):
        _check(self.L.laa_local_step_dense(self.h, self._rows_ptr(grads)))

    def step_dense(self, grads):
        _check(self.L.laa_step_dense(self.h, self._rows_ptr(grads)))

    def local_step_gen(self):
        _check(self.L.laa_local_step_gen(self.h))

    def step_gen(self):
        _check(self.L.laa_step_gen(self.h))

    def generate_gradient(self, out=None):
        if out is None:
            out = self.rows()
        _check(self.L.laa_generate_gradient(self.h, self._rows_ptr(out)))
        return out

    def local_step_sparse(self, idx, vals, row_len):
        k = idx.shape[1] if idx is not None else 0
        _check(self.L.laa_local_step_sparse(self.h, _dev_ptr(idx, self.torch.int32), _dev_ptr(vals, self.torch.float32),
                                            int(k), int(row_len)))

    def step_sparse(self, idx, vals, row_len):
        k = idx.shape[1] if idx is not None else 0
        _check(self.L.laa_step_sparse(self.h, _dev_ptr(idx, self.torch.int32), _dev_ptr(vals, self.torch.float32),
                                      int(k), int(row_len)))

    def sync(self):
        _check(self.L.laa_sync(self.h))

    def sync_static(self):
        _check(self.L.laa_sync_static(self.h))

    # queries -------------------------------------------------------------------------------
    def counters(self, with_bad=False):
        t, s, bad = C.c_int64(), C.c_int32(), C.c_int64()
        _check(self.L.laa_get_counters(self.h, C.byref(t), C.byref(s), C.byref(bad) if with_bad else None))
        return (t.value, s.value, bad.value) if with_bad else (t.value, s.value)

    def set_sparse_coalesce(self, on=True):
        _check(self.L.laa_set_sparse_coalesce(self.h, 1 if on else 0))

    def run_periods_gen(self, n_periods=1):
        _check(self.L.laa_run_periods_gen(self.h, int(n_periods)))

    def replay_count(self):
        n = C.c_int64(0)
        _check(self.L.laa_get_replay_count(self.h, C.byref(n)))
        return n.value

    def set_shard(self, first_column=0, first_worker=0):
        _check(self.L.laa_set_shard(self.h, int(first_column), int(first_worker)))

    def set_counters(self, t, steps_since_sync):
        _check(self.L.laa_set_counters(self.h, int(t), int(steps_since_sync)))

    def dirty_rows(self):
        n = C.c_int64()
        _check(self.L.laa_get_dirty_rows(self.h, None, 0, C.byref(n)))
        out = np.empty(n.value, dtype=np.int32)
        if n.value:
            _check(self.L.laa_get_dirty_rows(self.h, out.ctypes.data_as(C.c_void_p), n.value, C.byref(n)))
        return out

    def diagnostics(self):
        """(||xbar - xstar||^2, ||grad F(xbar)||^2, mean_w ||x_w - xbar||^2) of the quadratic workload."""
        out = (C.c_double * 3)()
        _check(self.L.laa_diagnostics(self.h, out))
        return tuple(out)

    def bytes_moved(self, literal=False):
        """Bytes the launches so far read and wrote; literal=True: (moved, literal) with the traffic of the same
        iterations as separate step and Synchronize passes over full replicas."""
        b, lit = C.c_uint64(), C.c_uint64()
        _check(self.L.laa_bytes_moved(self.h, C.byref(b), C.byref(lit)))
        return (b.value, lit.value) if literal else b.value


def debug_philox(ctr, key):
    ctr = np.ascontiguousarray(ctr, dtype=np.uint32)
    key = np.ascontiguousarray(key, dtype=np.uint32)
    out = np.empty(4, dtype=np.uint32)
    _check(lib().laa_debug_philox(ctr.ctypes.data_as(C.c_void_p), key.ctypes.data_as(C.c_void_p),
                                  out.ctypes.data_as(C.c_void_p)))
    return out


def debug_copy(dst, src):
    import torch
    _check(lib().laa_debug_copy(_dev_ptr(dst, torch.float32), _dev_ptr(src, torch.float32), dst.numel(),
                                C.c_void_p(torch.cuda.current_stream().cuda_stream)))
