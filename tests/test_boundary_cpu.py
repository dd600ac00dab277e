"""CPU tests of the C-ABI boundary: the library loads, exports what include/laa.h declares,
and rejects bad arguments on the host (no kernel is launched here)."""
import ctypes as C
import os
import re

import pytest

from paper_1911_09030_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(binding.LIB_PATH):
        from paper_1911_09030_amd import build
        build.build()
    return binding.lib()


def test_exports_match_header(L):
    hdr = open(os.path.join(ROOT, "include", "laa.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = sorted(set(re.findall(r"\b(laa_[a-z0-9_]+)\s*\(", hdr)))
    assert declared, "no declarations found"
    for name in declared:
        assert hasattr(L, name), f"{name} declared in laa.h but not exported"
    assert sorted(binding.EXPORTS) == declared


def test_create_validation(L):
    h = C.c_void_p()
    bad = [(0, 1, 1, .5, 1.), (-4, 1, 1, .5, 1.), (4, 0, 1, .5, 1.), (4, 1, 0, .5, 1.), (4, 1, 1, float("inf"), 1.),
           (4, 1, 1, float("nan"), 1.), (4, 1, 1, .5, -1.), (4, 1, 1, .5, float("nan"))]
    for args in bad:
        assert L.laa_create(*args, C.byref(h)) == binding.EINVAL, args
        assert L.laa_last_error()
    assert L.laa_create(4, 1, 1, .5, 1., None) == binding.EINVAL
    assert L.laa_create(8, 2, 3, .5, 1., C.byref(h)) == binding.OK and h.value
    assert L.laa_destroy(h) == binding.OK
    assert L.laa_destroy(None) == binding.OK


def test_host_error_paths(L):
    h = C.c_void_p()
    assert L.laa_create(12, 4, 2, .5, 1., C.byref(h)) == binding.OK
    # nothing attached yet
    assert L.laa_local_step_gen(h) == binding.ENOTATTACHED
    assert L.laa_sync(h) == binding.ENOTATTACHED
    assert L.laa_init_state(h, None) == binding.ENOTATTACHED
    assert b"attach" in L.laa_last_error()
    # setters
    assert L.laa_set_b0(h, -1.0) == binding.EINVAL
    assert L.laa_set_b0(h, 2.0) == binding.OK
    assert L.laa_set_warmup(h, -3) == binding.EINVAL
    assert L.laa_set_warmup(h, 600) == binding.OK
    assert L.laa_set_algorithm(h, 7) == binding.EINVAL
    assert L.laa_set_algorithm(h, binding.ALGO_LOCAL_SGD) == binding.OK
    assert L.laa_set_tile(h, 3) == binding.EINVAL
    assert L.laa_set_tile(h, 8) == binding.EINVAL          # does not divide W=4
    assert L.laa_set_tile(h, 2) == binding.OK
    assert L.laa_set_generator(h, 9, 0, C.c_void_p(16), None, None, 0, .1, .1) == binding.EMODE
    assert L.laa_set_generator(h, binding.GEN_QUADRATIC, 0, C.c_void_p(16), None, None, 0, .1, .1) == binding.EINVAL
    assert L.laa_set_generator(h, binding.GEN_QUADRATIC, 0, C.c_void_p(16), C.c_void_p(32), None,
                               binding.OFF_ARRAY, .1, .1) == binding.EINVAL
    assert L.laa_set_generator(h, binding.GEN_NOISE, 0, C.c_void_p(18), None, None, 0, .1, .1) == binding.EALIGN
    assert L.laa_set_generator(h, binding.GEN_NOISE, 0, C.c_void_p(16), None, None, 0, -.1, .1) == binding.EINVAL   # a standard deviation
    assert L.laa_set_generator(h, binding.GEN_QUADRATIC, 0, C.c_void_p(16), C.c_void_p(32), None, 0, .1, float("nan")) == binding.EINVAL
    assert L.laa_set_tile(h, 0) == binding.OK              # one worker per block in non-averaging steps
    assert L.laa_set_lazy_replicas(h, 1) == binding.OK
    assert L.laa_set_lazy_replicas(None, 1) == binding.EINVAL
    assert L.laa_materialize(h) == binding.ENOTATTACHED
    out = (C.c_double * 3)()
    assert L.laa_diagnostics(h, out) == binding.ENOTATTACHED
    assert L.laa_attach_pitched(h, C.c_void_p(16), C.c_void_p(32), C.c_void_p(48), 8, None) == binding.EINVAL  # pitch < d
    assert L.laa_attach(h, None, None, None, None) == binding.EINVAL
    assert L.laa_attach(h, C.c_void_p(2), C.c_void_p(16), C.c_void_p(16), None) == binding.EALIGN
    t, s = C.c_int64(-1), C.c_int32(-1)
    assert L.laa_get_counters(h, C.byref(t), C.byref(s), None) == binding.OK and (t.value, s.value) == (0, 0)
    assert L.laa_run_periods_gen(h, 1) == binding.ENOTATTACHED
    assert L.laa_set_shard(h, 6, 0) == binding.EINVAL            # not a multiple of 4
    assert L.laa_set_shard(h, -4, 0) == binding.EINVAL
    assert L.laa_set_shard(h, 8, -1) == binding.EINVAL
    assert L.laa_set_shard(h, 2**62, 2**31 - 1) == binding.EINVAL   # first_worker + W overflows
    assert L.laa_set_shard(h, 2**40, 3) == binding.OK
    assert L.laa_set_shard(h, 0, 0) == binding.OK
    assert L.laa_set_counters(h, 5, 3) == binding.EINVAL        # more local steps than H = 2
    assert L.laa_set_counters(h, 1, 2) == binding.EINVAL        # more local steps than iterations
    assert L.laa_set_counters(h, 7, 1) == binding.OK
    assert L.laa_get_counters(h, C.byref(t), C.byref(s), None) == binding.OK and (t.value, s.value) == (7, 1)
    assert L.laa_set_counters(h, 0, 0) == binding.OK
    b = C.c_uint64(5)
    lit = C.c_uint64(5)
    assert L.laa_bytes_moved(h, C.byref(b), C.byref(lit)) == binding.OK and b.value == 0 and lit.value == 0
    assert L.laa_bytes_moved(h, None, C.byref(lit)) == binding.OK
    assert L.laa_bytes_moved(h, None, None) == binding.EINVAL
    assert L.laa_sync_static(h) == binding.ENOTATTACHED
    assert L.laa_destroy(h) == binding.OK
    # the chunked pool: argument checks happen before any device is touched
    base = C.c_void_p()
    assert L.laa_pool_create(0, 1 << 21, C.byref(base), None, None) == binding.EINVAL
    assert L.laa_pool_create(1 << 21, 0, C.byref(base), None, None) == binding.EINVAL
    assert L.laa_pool_create(1 << 21, 1 << 21, None, None, None) == binding.EINVAL
    assert L.laa_pool_trim(None, 0, None, None) == binding.EINVAL
    assert L.laa_pool_trim(C.c_void_p(1 << 21), 0, None, None) == binding.EINVAL       # not a pool
    assert L.laa_pool_free(None) == binding.OK
    assert L.laa_pool_free(C.c_void_p(1 << 21)) == binding.EINVAL


def test_attach_without_gpu_fails_loudly(L):
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    h = C.c_void_p()
    assert L.laa_create(8, 2, 2, .5, 1., C.byref(h)) == binding.OK
    assert L.laa_attach(h, C.c_void_p(16), C.c_void_p(32), C.c_void_p(48), None) == binding.ENODEVICE
    L.laa_destroy(h)
