"""ctypes loader for the CPU oracle (oracle/ftar_oracle.cpp).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
CPU-baseline leg of bench.py.  Nothing in the product package imports it and it
imports nothing from the product package.

Every wrapper below only marshals numpy arrays into the C calls; the arithmetic
is in the C++ file.  Arrays of bf16 data are numpy uint16 arrays holding the
raw bf16 bit patterns; fp32 data are numpy float32 arrays.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ftar_oracle.cpp")
_LIB = os.path.join(_HERE, "libftar_oracle.so")

F32 = 0
BF16 = 1

_lib = None


def build(force=False):
    """Compile the oracle with the host compiler (no GPU toolchain involved)."""
    if not force and os.path.exists(_LIB) and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC):
        return _LIB
    cmd = ["g++", "-std=c++17", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fPIC",
           "-shared", "-Wall", "-Wextra", "-o", _LIB, _SRC]
    subprocess.run(cmd, check=True)
    return _LIB


def lib():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        vp, u64, sz, ci = ctypes.c_void_p, ctypes.c_uint64, ctypes.c_size_t, ctypes.c_int
        L.oracle_bf16_to_f32_bits.restype = ctypes.c_uint32
        L.oracle_bf16_to_f32_bits.argtypes = [ctypes.c_uint16]
        L.oracle_f32_bits_to_bf16.restype = ctypes.c_uint16
        L.oracle_f32_bits_to_bf16.argtypes = [ctypes.c_uint32]
        L.oracle_f32_to_bf16_array.restype = None
        L.oracle_f32_to_bf16_array.argtypes = [vp, vp, sz]
        L.oracle_bf16_to_f32_array.restype = None
        L.oracle_bf16_to_f32_array.argtypes = [vp, vp, sz]
        L.oracle_live_ring.restype = ci
        L.oracle_live_ring.argtypes = [ci, u64, vp]
        L.oracle_scale_bits.restype = ctypes.c_uint32
        L.oracle_scale_bits.argtypes = [ci]
        L.oracle_geometry.restype = ci
        L.oracle_geometry.argtypes = [ci, u64, sz, sz, vp]
        L.oracle_reduce_masked.restype = ci
        L.oracle_reduce_masked.argtypes = [vp, ci, u64, sz, ci, ci, vp]
        L.oracle_reduce_masked_zero.restype = ci
        L.oracle_reduce_masked_zero.argtypes = [vp, ci, u64, u64, ci, sz, ci, vp]
        L.oracle_reduce_masked_ex.restype = ci
        L.oracle_reduce_masked_ex.argtypes = [vp, ci, u64, u64, ci, sz, ci, ci, ci, vp]
        L.oracle_lr_factors.restype = ci
        L.oracle_lr_factors.argtypes = [ci, u64, u64, vp, vp]
        L.oracle_ring_closed_form_zero.restype = ci
        L.oracle_ring_closed_form_zero.argtypes = [vp, ci, u64, u64, ci, sz, sz, ci, sz, sz, vp]
        L.oracle_reduce_f64.restype = ci
        L.oracle_reduce_f64.argtypes = [vp, ci, u64, sz, ci, ci, vp, vp]
        L.oracle_ring_per_rank.restype = ci
        L.oracle_ring_per_rank.argtypes = [vp, ci, u64, sz, sz, ci, ci, ci, ci, vp]
        L.oracle_ring_schedule.restype = ci
        L.oracle_ring_schedule.argtypes = [ci, u64, vp, vp]
        L.oracle_ring_closed_form.restype = ci
        L.oracle_ring_closed_form.argtypes = [vp, ci, u64, sz, sz, ci, ci, sz, sz, vp]
        L.oracle_ring_partial.restype = ci
        L.oracle_ring_partial.argtypes = [vp, ci, u64, sz, sz, ci, ci, sz, sz, vp]
        _lib = L
    return _lib


class OracleError(ValueError):
    pass


def _check(rc):
    if rc < 0:
        raise OracleError({-1: "invalid argument", -2: "no live replica",
                           -3: "mask bit beyond n_replicas", -4: "bad step"}.get(rc, str(rc)))
    return rc


def _np_dtype(dtype):
    return np.float32 if dtype == F32 else np.uint16


def _ptr_table(bufs, dtype, mask):
    """Host pointer table; dead replicas may be None (NULL in the table)."""
    n = len(bufs)
    tab = (ctypes.c_void_p * n)()
    for r, b in enumerate(bufs):
        if b is None:
            if (mask >> r) & 1:
                raise OracleError("live replica %d has no buffer" % r)
            tab[r] = None
            continue
        assert b.dtype == _np_dtype(dtype) and b.flags["C_CONTIGUOUS"], (b.dtype, dtype)
        tab[r] = b.ctypes.data
    return tab


def f32_to_bf16(x):
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(x.shape, dtype=np.uint16)
    lib().oracle_f32_to_bf16_array(x.ctypes.data, out.ctypes.data, x.size)
    return out


def bf16_to_f32(h):
    h = np.ascontiguousarray(h, dtype=np.uint16)
    out = np.empty(h.shape, dtype=np.float32)
    lib().oracle_bf16_to_f32_array(h.ctypes.data, out.ctypes.data, h.size)
    return out


def live_ring(n, mask):
    ring = np.zeros(64, dtype=np.int32)
    N = _check(lib().oracle_live_ring(n, mask, ring.ctypes.data))
    return [int(v) for v in ring[:N]]


def scale(N):
    return np.array([lib().oracle_scale_bits(N)], dtype=np.uint32).view(np.float32)[0]


def geometry(n, mask, count, chunk_elems):
    sb = np.zeros(65, dtype=np.uint64)
    N = _check(lib().oracle_geometry(n, mask, count, chunk_elems, sb.ctypes.data))
    return [int(v) for v in sb[:N + 1]]


def reduce_masked(bufs, mask, dtype, sum_only=False, count=None):
    n = len(bufs)
    live = [b for b in bufs if b is not None]
    count = live[0].size if count is None else count
    out = np.empty(count, dtype=_np_dtype(dtype))
    tab = _ptr_table(bufs, dtype, mask)
    _check(lib().oracle_reduce_masked(tab, n, mask, count, dtype, int(sum_only), out.ctypes.data))
    return out


def reduce_masked_zero(bufs, live_mask, zero_mask, dtype, contributors_only=False):
    """Zero participants' buffers are never read and may be None."""
    n = len(bufs)
    count = [b for r, b in enumerate(bufs) if b is not None and not (zero_mask >> r) & 1][0].size \
        if any(b is not None and not (zero_mask >> r) & 1 for r, b in enumerate(bufs)) \
        else [b for b in bufs if b is not None][0].size
    out = np.empty(count, dtype=_np_dtype(dtype))
    tab = _ptr_table(bufs, dtype, live_mask & ~zero_mask)
    _check(lib().oracle_reduce_masked_zero(tab, n, live_mask, zero_mask, int(contributors_only), count,
                                           dtype, out.ctypes.data))
    return out


def reduce_masked_ex(bufs, live_mask, dtype, out_dtype=None, zero_mask=0, contributors_only=False,
                     sum_only=False, count=None):
    """One-shot reduction with a result type and operation of choice; zero participants may be None."""
    n = len(bufs)
    out_dtype = dtype if out_dtype is None else out_dtype
    if count is None:
        count = [b for b in bufs if b is not None][0].size
    out = np.empty(count, dtype=_np_dtype(out_dtype))
    tab = _ptr_table(bufs, dtype, live_mask & ~zero_mask)
    _check(lib().oracle_reduce_masked_ex(tab, n, live_mask, zero_mask, int(contributors_only), count,
                                         dtype, out_dtype, int(sum_only), out.ctypes.data))
    return out


def lr_factors(n, live_mask, zero_mask=0):
    """(linear, sqrt) learning-rate factors as two numpy float32 scalars."""
    lin, root = np.zeros(1, np.float32), np.zeros(1, np.float32)
    _check(lib().oracle_lr_factors(n, live_mask, zero_mask, lin.ctypes.data, root.ctypes.data))
    return lin[0], root[0]


def ring_closed_form_zero(bufs, live_mask, zero_mask, count, chunk_elems, dtype, contributors_only=False,
                          begin=0, length=None):
    n = len(bufs)
    length = [b for b in bufs if b is not None][0].size if length is None else length
    out = np.empty(length, dtype=_np_dtype(dtype))
    tab = _ptr_table(bufs, dtype, live_mask & ~zero_mask)
    _check(lib().oracle_ring_closed_form_zero(tab, n, live_mask, zero_mask, int(contributors_only), count,
                                              chunk_elems, dtype, begin, length, out.ctypes.data))
    return out


def reduce_f64(bufs, mask, dtype, sum_only=False):
    n = len(bufs)
    count = [b for b in bufs if b is not None][0].size
    out = np.empty(count, dtype=np.float64)
    mag = np.empty(count, dtype=np.float64)
    tab = _ptr_table(bufs, dtype, mask)
    _check(lib().oracle_reduce_f64(tab, n, mask, count, dtype, int(sum_only),
                                   out.ctypes.data, mag.ctypes.data))
    return out, mag


def ring_per_rank(bufs, mask, chunk_elems, dtype, rs_steps=None, ag_steps=None, sum_only=False):
    """In place on `bufs` (list of numpy arrays). Returns the fp32 in-flight image."""
    n = len(bufs)
    N = len(live_ring(n, mask))
    rs_steps = N - 1 if rs_steps is None else rs_steps
    ag_steps = (N - 1 if rs_steps == N - 1 else 0) if ag_steps is None else ag_steps
    count = [b for b in bufs if b is not None][0].size
    acc = np.zeros(count, dtype=np.float32)
    tab = _ptr_table(bufs, dtype, mask)
    _check(lib().oracle_ring_per_rank(tab, n, mask, count, chunk_elems, dtype, int(sum_only),
                                      rs_steps, ag_steps, acc.ctypes.data))
    return acc


def ring_schedule(n, mask):
    N = len(live_ring(n, mask))
    rs = np.zeros(max(1, N * (N - 1)), dtype=np.int32)
    ag = np.zeros(max(1, N * (N - 1)), dtype=np.int32)
    _check(lib().oracle_ring_schedule(n, mask, rs.ctypes.data, ag.ctypes.data))
    return rs[:N * (N - 1)].reshape(N - 1, N), ag[:N * (N - 1)].reshape(N - 1, N)


def ring_closed_form(bufs, mask, count, chunk_elems, dtype, begin=0, length=None, sum_only=False):
    """bufs[r] holds elements [begin, begin+length) of replica r's original data."""
    n = len(bufs)
    length = [b for b in bufs if b is not None][0].size if length is None else length
    out = np.empty(length, dtype=_np_dtype(dtype))
    tab = _ptr_table(bufs, dtype, mask)
    _check(lib().oracle_ring_closed_form(tab, n, mask, count, chunk_elems, dtype, int(sum_only),
                                         begin, length, out.ctypes.data))
    return out


def ring_partial(bufs, mask, count, chunk_elems, dtype, rs_steps, begin=0, length=None):
    n = len(bufs)
    length = [b for b in bufs if b is not None][0].size if length is None else length
    acc = np.empty(length, dtype=np.float32)
    tab = _ptr_table(bufs, dtype, mask)
    _check(lib().oracle_ring_partial(tab, n, mask, count, chunk_elems, dtype, rs_steps,
                                     begin, length, acc.ctypes.data))
    return acc
