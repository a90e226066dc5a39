"""Thin Python binding over the C ABI in include/ftar.h (same names, argument
marshalling only; every step of the path runs in the HIP kernels of libftar.so).

Buffers are torch tensors living on the GPU (torch is used for device memory and
streams only); each wrapper passes their data pointers and the current torch
stream's handle to the C call and raises FtarError on a non-zero status.
There is no fallback: if libftar.so is missing or fails to load, the first call
raises.
"""
import ctypes
import os
from typing import List, Optional, Sequence

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libftar.so")

FTAR_F32 = 0
FTAR_BF16 = 1

FTAR_OK = 0
FTAR_ERR_INVALID_ARG = 1
FTAR_ERR_NO_LIVE = 2
FTAR_ERR_BAD_MASK = 3
FTAR_ERR_BAD_STEP = 4
FTAR_ERR_TOO_LARGE = 5
FTAR_ERR_STALE_PLAN = 16
FTAR_ERR_SKIPPED = 17
FTAR_ERR_DEVICE = 32

FTAR_MEAN = 0
FTAR_SUM = 1

FTAR_PERSIST_PUBLISH = 1
FTAR_PERSIST_ALIGN = 2
FTAR_PERSIST_CHUNKS = 4

# every symbol include/ftar.h declares
EXPORTS = [
    "ftar_plan", "ftar_plan_destroy", "ftar_plan_set_dtype", "ftar_plan_n_live",
    "ftar_plan_n_steps", "ftar_plan_acc_bytes", "ftar_plan_scale", "ftar_plan_segment",
    "ftar_reduce_step", "ftar_allgather_step", "ftar_reduce_masked",
    "ftar_reduce_masked_bucketed", "ftar_last_error", "ftar_status_is_retryable",
    "ftar_status_str",
    "ftar_ctrl_create", "ftar_ctrl_destroy", "ftar_ring_persistent", "ftar_ctrl_release",
    "ftar_ctrl_cancel", "ftar_ctrl_progress", "ftar_ctrl_result",
    "ftar_plan_set_partition", "ftar_plan_n_partitions", "ftar_plan_n_slots",
    "ftar_plan_partition_segment", "ftar_allreduce_onepass", "ftar_plan_set_zero_mask",
    "ftar_reduce_masked_zero", "ftar_plan_set_op", "ftar_reduce_masked_ex", "ftar_plan_lr_factors",
    "ftar_allgather_all", "ftar_reduce_scatter_all",
    "ftar_ring_persistent_static", "ftar_plan_n_gate_units", "ftar_ctrl_last_ticket",
    "ftar_ctrl_release_call", "ftar_ctrl_progress_call", "ftar_ctrl_result_call",
]

# every symbol include/ftar_measure.h declares: measurement hooks in libftar.so, probe kernels in
# the bench-only libftar_measure.so
MEASURE_HOOKS = ["ftar_set_tuning", "ftar_time_next_launch"]
MEASURE_EXPORTS = ["ftar_probe_stream", "ftar_probe_stream_windows", "ftar_probe_stream_workgroups"]
MEASURE_LIB_PATH = os.path.join(_PKG, "libftar_measure.so")

_lib = None
_measure_lib = None


class FtarError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib().ftar_status_str(status).decode()
        super().__init__("%s: %s (status %d)" % (where, msg, status))


def lib():
    """Loads libftar.so once.  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError("libftar.so is not built: run `python -m paper_2602_00277_amd.build` "
                          "(there is no fallback path)")
    L = ctypes.CDLL(LIB_PATH)
    vp, u64, sz, ci = ctypes.c_void_p, ctypes.c_uint64, ctypes.c_size_t, ctypes.c_int
    L.ftar_plan.restype = vp
    L.ftar_plan.argtypes = [ci, u64, sz, sz]
    L.ftar_plan_destroy.restype = None
    L.ftar_plan_destroy.argtypes = [vp]
    L.ftar_plan_set_dtype.restype = ci
    L.ftar_plan_set_dtype.argtypes = [vp, ci]
    L.ftar_plan_n_live.restype = ci
    L.ftar_plan_n_live.argtypes = [vp]
    L.ftar_plan_n_steps.restype = ci
    L.ftar_plan_n_steps.argtypes = [vp]
    L.ftar_plan_acc_bytes.restype = sz
    L.ftar_plan_acc_bytes.argtypes = [vp]
    L.ftar_plan_scale.restype = ctypes.c_float
    L.ftar_plan_scale.argtypes = [vp]
    L.ftar_plan_segment.restype = ci
    L.ftar_plan_segment.argtypes = [vp, ci, ctypes.POINTER(sz), ctypes.POINTER(sz),
                                    ctypes.POINTER(ci)]
    L.ftar_reduce_step.restype = ci
    L.ftar_reduce_step.argtypes = [vp, ci, vp, vp, vp]
    L.ftar_allgather_step.restype = ci
    L.ftar_allgather_step.argtypes = [vp, ci, vp, vp]
    L.ftar_reduce_masked.restype = ci
    L.ftar_reduce_masked.argtypes = [vp, ci, u64, sz, ci, vp, vp]
    L.ftar_reduce_masked_bucketed.restype = ci
    L.ftar_reduce_masked_bucketed.argtypes = [vp, ci, vp, sz, sz, sz, ci, vp, vp]
    L.ftar_last_error.restype = ci
    L.ftar_last_error.argtypes = []
    L.ftar_status_is_retryable.restype = ci
    L.ftar_status_is_retryable.argtypes = [ci]
    L.ftar_status_str.restype = ctypes.c_char_p
    L.ftar_status_str.argtypes = [ci]
    L.ftar_set_tuning.restype = None
    L.ftar_set_tuning.argtypes = [ci, ci]
    L.ftar_time_next_launch.restype = None
    L.ftar_time_next_launch.argtypes = [vp, vp]
    L.ftar_plan_set_partition.restype = ci
    L.ftar_plan_set_partition.argtypes = [vp, sz]
    L.ftar_plan_n_partitions.restype = ci
    L.ftar_plan_n_partitions.argtypes = [vp]
    L.ftar_plan_n_slots.restype = ci
    L.ftar_plan_n_slots.argtypes = [vp]
    L.ftar_plan_partition_segment.restype = ci
    L.ftar_plan_partition_segment.argtypes = [vp, ci, ci, ctypes.POINTER(sz), ctypes.POINTER(sz),
                                              ctypes.POINTER(ci)]
    L.ftar_plan_set_zero_mask.restype = ci
    L.ftar_plan_set_zero_mask.argtypes = [vp, u64, ci]
    L.ftar_reduce_masked_zero.restype = ci
    L.ftar_reduce_masked_zero.argtypes = [vp, ci, u64, u64, ci, sz, ci, vp, vp]
    L.ftar_plan_set_op.restype = ci
    L.ftar_plan_set_op.argtypes = [vp, ci]
    L.ftar_reduce_masked_ex.restype = ci
    L.ftar_reduce_masked_ex.argtypes = [vp, ci, u64, u64, ci, sz, ci, ci, ci, vp, vp]
    L.ftar_plan_lr_factors.restype = ci
    L.ftar_plan_lr_factors.argtypes = [vp, vp, vp]
    L.ftar_reduce_scatter_all.restype = ci
    L.ftar_reduce_scatter_all.argtypes = [vp, vp, vp]
    L.ftar_allgather_all.restype = ci
    L.ftar_allgather_all.argtypes = [vp, vp, vp]
    L.ftar_allreduce_onepass.restype = ci
    L.ftar_allreduce_onepass.argtypes = [vp, vp, vp]
    L.ftar_ctrl_create.restype = vp
    L.ftar_ctrl_create.argtypes = []
    L.ftar_ctrl_destroy.restype = None
    L.ftar_ctrl_destroy.argtypes = [vp]
    L.ftar_ring_persistent.restype = ci
    L.ftar_ring_persistent.argtypes = [vp, vp, vp, vp, ci, ctypes.c_uint, ctypes.c_uint, vp]
    L.ftar_ring_persistent_static.restype = ci
    L.ftar_ring_persistent_static.argtypes = [vp, vp, vp, ci, ctypes.c_uint, ctypes.c_uint, vp]
    L.ftar_plan_n_gate_units.restype = ci
    L.ftar_plan_n_gate_units.argtypes = [vp, ctypes.c_uint]
    L.ftar_ctrl_last_ticket.restype = ci
    L.ftar_ctrl_last_ticket.argtypes = [vp]
    L.ftar_ctrl_release_call.restype = None
    L.ftar_ctrl_release_call.argtypes = [vp, ci, ci]
    L.ftar_ctrl_progress_call.restype = ci
    L.ftar_ctrl_progress_call.argtypes = [vp, ci]
    L.ftar_ctrl_result_call.restype = ci
    L.ftar_ctrl_result_call.argtypes = [vp, ci, ctypes.POINTER(ci)]
    L.ftar_ctrl_release.restype = None
    L.ftar_ctrl_release.argtypes = [vp, ci]
    L.ftar_ctrl_cancel.restype = None
    L.ftar_ctrl_cancel.argtypes = [vp]
    L.ftar_ctrl_progress.restype = ci
    L.ftar_ctrl_progress.argtypes = [vp]
    L.ftar_ctrl_result.restype = ci
    L.ftar_ctrl_result.argtypes = [vp, ctypes.POINTER(ci)]
    _lib = L
    return L


def measure_lib():
    """Loads the bench-only libftar_measure.so once (after libftar.so, which it links against)."""
    global _measure_lib
    if _measure_lib is not None:
        return _measure_lib
    lib()
    if not os.path.exists(MEASURE_LIB_PATH):
        raise ImportError("libftar_measure.so is not built: run `python -m paper_2602_00277_amd.build`")
    M = ctypes.CDLL(MEASURE_LIB_PATH)
    M.ftar_probe_stream.restype = ctypes.c_int
    M.ftar_probe_stream.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_size_t,
                                    ctypes.c_uint32, ctypes.c_void_p]
    M.ftar_probe_stream_windows.restype = ctypes.c_int
    M.ftar_probe_stream_windows.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t, ctypes.c_uint,
                                            ctypes.c_uint, ctypes.c_void_p]
    M.ftar_probe_stream_workgroups.restype = ctypes.c_int
    M.ftar_probe_stream_workgroups.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t, ctypes.c_uint,
                                               ctypes.c_uint, ctypes.c_uint, ctypes.c_void_p]
    _measure_lib = M
    return M


def dtype_code(dtype: torch.dtype) -> int:
    if dtype == torch.float32:
        return FTAR_F32
    if dtype == torch.bfloat16:
        return FTAR_BF16
    raise TypeError("FTAR buffers are float32 or bfloat16, not %s" % dtype)


def _ptr_array(bufs: Sequence[Optional[torch.Tensor]]):
    """Host array of device pointers; None (a dead replica without a buffer) becomes NULL."""
    arr = (ctypes.c_void_p * len(bufs))()
    for r, b in enumerate(bufs):
        arr[r] = None if b is None else b.data_ptr()
    return arr


def _stream_handle(stream) -> int:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _check_bufs(bufs, live_mask, count=None, dtype=None):
    for r, b in enumerate(bufs):
        if b is None:
            continue
        if not b.is_cuda or not b.is_contiguous():
            raise ValueError("replica buffer %d must be a contiguous GPU tensor" % r)
        if dtype is not None and b.dtype != dtype:
            raise TypeError("replica buffer %d has dtype %s, expected %s" % (r, b.dtype, dtype))
        if count is not None and (live_mask >> r) & 1 and b.numel() < count:
            raise ValueError("replica buffer %d is shorter than count" % r)


class Plan:
    """Owner of an ftar_plan_t* (destroyed with the object)."""

    def __init__(self, handle: int, n_replicas: int, live_mask: int, count: int, chunk_elems: int):
        self.handle = handle
        self.n_replicas = n_replicas
        self.live_mask = live_mask
        self.count = count
        self.chunk_elems = chunk_elems
        self.dtype = torch.bfloat16

    @property
    def n_live(self) -> int:
        return lib().ftar_plan_n_live(self.handle)

    @property
    def n_steps(self) -> int:
        return lib().ftar_plan_n_steps(self.handle)

    @property
    def acc_bytes(self) -> int:
        return lib().ftar_plan_acc_bytes(self.handle)

    @property
    def scale(self) -> float:
        return lib().ftar_plan_scale(self.handle)

    def segment(self, k: int):
        b, e, o = ctypes.c_size_t(), ctypes.c_size_t(), ctypes.c_int()
        st = lib().ftar_plan_segment(self.handle, k, ctypes.byref(b), ctypes.byref(e), ctypes.byref(o))
        if st != FTAR_OK:
            raise FtarError(st, "ftar_plan_segment")
        return b.value, e.value, o.value

    @property
    def n_partitions(self) -> int:
        return lib().ftar_plan_n_partitions(self.handle)

    @property
    def n_slots(self) -> int:
        return lib().ftar_plan_n_slots(self.handle)

    def n_gate_units(self, flags: int = 0) -> int:
        return lib().ftar_plan_n_gate_units(self.handle, flags)

    def set_partition(self, partition_elems: int) -> None:
        st = lib().ftar_plan_set_partition(self.handle, partition_elems)
        if st != FTAR_OK:
            raise FtarError(st, "ftar_plan_set_partition")
        self.partition_elems = partition_elems

    def partition_segment(self, partition: int, k: int):
        b, e, o = ctypes.c_size_t(), ctypes.c_size_t(), ctypes.c_int()
        st = lib().ftar_plan_partition_segment(self.handle, partition, k, ctypes.byref(b),
                                               ctypes.byref(e), ctypes.byref(o))
        if st != FTAR_OK:
            raise FtarError(st, "ftar_plan_partition_segment")
        return b.value, e.value, o.value

    def destroy(self):
        if self.handle:
            lib().ftar_plan_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def ftar_plan(n_replicas: int, live_mask: int, count: int, chunk_elems: int,
              dtype: Optional[torch.dtype] = None) -> Plan:
    h = lib().ftar_plan(n_replicas, live_mask, count, chunk_elems)
    if not h:
        raise FtarError(lib().ftar_last_error(), "ftar_plan")
    p = Plan(h, n_replicas, live_mask, count, chunk_elems)
    if dtype is not None:
        ftar_plan_set_dtype(p, dtype)
    return p


def ftar_plan_destroy(plan: Plan) -> None:
    plan.destroy()


def ftar_plan_set_partition(plan: Plan, partition_elems: int) -> None:
    plan.set_partition(partition_elems)


def ftar_plan_set_dtype(plan: Plan, dtype: torch.dtype) -> None:
    st = lib().ftar_plan_set_dtype(plan.handle, dtype_code(dtype))
    if st != FTAR_OK:
        raise FtarError(st, "ftar_plan_set_dtype")
    plan.dtype = dtype


def ftar_reduce_step(plan: Plan, step: int, bufs: Sequence[Optional[torch.Tensor]],
                     acc: Optional[torch.Tensor], stream=None) -> None:
    _check_bufs(bufs, plan.live_mask, plan.count, plan.dtype)
    if len(bufs) != plan.n_replicas:
        raise ValueError("bufs must have one entry per replica slot")
    if acc is not None and (acc.dtype != torch.float32 or acc.numel() < plan.count or not acc.is_cuda):
        raise ValueError("acc must be a GPU float32 tensor of at least count elements")
    st = lib().ftar_reduce_step(plan.handle, step, _ptr_array(bufs),
                                None if acc is None else acc.data_ptr(), _stream_handle(stream))
    if st != FTAR_OK:
        raise FtarError(st, "ftar_reduce_step")


def ftar_allgather_step(plan: Plan, step: int, bufs: Sequence[Optional[torch.Tensor]],
                        stream=None) -> None:
    _check_bufs(bufs, plan.live_mask, plan.count, plan.dtype)
    if len(bufs) != plan.n_replicas:
        raise ValueError("bufs must have one entry per replica slot")
    st = lib().ftar_allgather_step(plan.handle, step, _ptr_array(bufs), _stream_handle(stream))
    if st != FTAR_OK:
        raise FtarError(st, "ftar_allgather_step")


def ftar_reduce_masked(bufs: Sequence[Optional[torch.Tensor]], live_mask: int, out: torch.Tensor,
                       count: Optional[int] = None, stream=None) -> torch.Tensor:
    count = out.numel() if count is None else count
    _check_bufs(list(bufs) + [out], live_mask | (1 << len(bufs)), count, out.dtype)
    st = lib().ftar_reduce_masked(_ptr_array(bufs), len(bufs), live_mask, count,
                                  dtype_code(out.dtype), out.data_ptr(), _stream_handle(stream))
    if st != FTAR_OK:
        raise FtarError(st, "ftar_reduce_masked")
    return out


def ftar_reduce_masked_zero(bufs: Sequence[Optional[torch.Tensor]], live_mask: int, zero_mask: int,
                            out: torch.Tensor, contributors_only: bool = False,
                            count: Optional[int] = None, stream=None) -> torch.Tensor:
    count = out.numel() if count is None else count
    _check_bufs(list(bufs) + [out], (live_mask & ~zero_mask) | (1 << len(bufs)), count, out.dtype)
    st = lib().ftar_reduce_masked_zero(_ptr_array(bufs), len(bufs), live_mask, zero_mask,
                                       int(contributors_only), count, dtype_code(out.dtype),
                                       out.data_ptr(), _stream_handle(stream))
    if st != FTAR_OK:
        raise FtarError(st, "ftar_reduce_masked_zero")
    return out


def ftar_reduce_masked_ex(bufs: Sequence[Optional[torch.Tensor]], live_mask: int, out: torch.Tensor,
                          zero_mask: int = 0, contributors_only: bool = False, op: int = FTAR_MEAN,
                          count: Optional[int] = None, stream=None) -> torch.Tensor:
    """in_dtype is the buffers' dtype, out_dtype is out's."""
    count = out.numel() if count is None else count
    read = live_mask & ~zero_mask
    srcs = [b for r, b in enumerate(bufs) if b is not None and (read >> r) & 1] or \
           [b for b in bufs if b is not None]
    in_dtype = srcs[0].dtype if srcs else out.dtype
    _check_bufs(bufs, read, count, in_dtype)
    _check_bufs([out], 1, count, out.dtype)
    st = lib().ftar_reduce_masked_ex(_ptr_array(bufs), len(bufs), live_mask, zero_mask,
                                     int(contributors_only), count, dtype_code(in_dtype),
                                     dtype_code(out.dtype), op, out.data_ptr(), _stream_handle(stream))
    if st != FTAR_OK:
        raise FtarError(st, "ftar_reduce_masked_ex")
    return out


def ftar_plan_set_op(plan: "Plan", op: int) -> None:
    st = lib().ftar_plan_set_op(plan.handle, op)
    if st != FTAR_OK:
        raise FtarError(st, "ftar_plan_set_op")


def ftar_plan_lr_factors(plan: "Plan"):
    """(linear, sqrt) learning-rate factors as Python floats holding fp32 values."""
    lin, root = ctypes.c_float(), ctypes.c_float()
    st = lib().ftar_plan_lr_factors(plan.handle, ctypes.byref(lin), ctypes.byref(root))
    if st != FTAR_OK:
        raise FtarError(st, "ftar_plan_lr_factors")
    return lin.value, root.value


def ftar_plan_set_zero_mask(plan: "Plan", zero_mask: int, contributors_only: bool = False) -> None:
    st = lib().ftar_plan_set_zero_mask(plan.handle, zero_mask, int(contributors_only))
    if st != FTAR_OK:
        raise FtarError(st, "ftar_plan_set_zero_mask")


def ftar_reduce_masked_bucketed(bufs: Sequence[Optional[torch.Tensor]], masks: Sequence[int],
                                bucket_elems: int, out: torch.Tensor,
                                count: Optional[int] = None, stream=None) -> torch.Tensor:
    count = out.numel() if count is None else count
    any_live = 0
    for m in masks:
        any_live |= m
    _check_bufs(list(bufs) + [out], any_live | (1 << len(bufs)), count, out.dtype)
    marr = (ctypes.c_uint64 * len(masks))(*masks)
    st = lib().ftar_reduce_masked_bucketed(_ptr_array(bufs), len(bufs), marr, len(masks),
                                           bucket_elems, count, dtype_code(out.dtype),
                                           out.data_ptr(), _stream_handle(stream))
    if st != FTAR_OK:
        raise FtarError(st, "ftar_reduce_masked_bucketed")
    return out


def ftar_probe_stream(read: Sequence[torch.Tensor], written: Sequence[torch.Tensor], fill: int = 0,
                      stream=None) -> None:
    """Measurement only: bare streaming kernel over equally sized buffers."""
    bufs = list(read) + list(written)
    nbytes = bufs[0].numel() * bufs[0].element_size()
    for b in bufs:
        if not b.is_cuda or not b.is_contiguous() or b.numel() * b.element_size() != nbytes:
            raise ValueError("probe buffers must be contiguous GPU tensors of one size")
    st = measure_lib().ftar_probe_stream(_ptr_array(bufs), len(read), len(written), nbytes, fill,
                                         _stream_handle(stream))
    if st != FTAR_OK:
        raise FtarError(st, "ftar_probe_stream")


def ftar_probe_stream_windows(read: Sequence[torch.Tensor], written: torch.Tensor, period_ticks: int = 4096,
                              window_ticks: int = 512, stream=None) -> None:
    """Measurement only: the bare streaming kernel with its writes placed in windows of the wall clock."""
    bufs = list(read) + [written]
    nbytes = bufs[0].numel() * bufs[0].element_size()
    for b in bufs:
        if not b.is_cuda or not b.is_contiguous() or b.numel() * b.element_size() != nbytes:
            raise ValueError("probe buffers must be contiguous GPU tensors of one size")
    st = measure_lib().ftar_probe_stream_windows(_ptr_array(bufs), len(read), nbytes, period_ticks, window_ticks,
                                                 _stream_handle(stream))
    if st != FTAR_OK:
        raise FtarError(st, "ftar_probe_stream_windows")


def ftar_probe_stream_workgroups(read: Sequence[torch.Tensor], written: torch.Tensor, n_workgroups: int,
                                 threads: int = 256, vectors_per_lane: int = 8, stream=None) -> None:
    """Measurement only: the bare streaming kernel on exactly n_workgroups workgroups."""
    bufs = list(read) + [written]
    nbytes = bufs[0].numel() * bufs[0].element_size()
    for b in bufs:
        if not b.is_cuda or not b.is_contiguous() or b.numel() * b.element_size() != nbytes:
            raise ValueError("probe buffers must be contiguous GPU tensors of one size")
    st = measure_lib().ftar_probe_stream_workgroups(_ptr_array(bufs), len(read), nbytes, n_workgroups, threads,
                                                    vectors_per_lane, _stream_handle(stream))
    if st != FTAR_OK:
        raise FtarError(st, "ftar_probe_stream_workgroups")


def ftar_set_tuning(blocks_per_cu: int = 0, flags: int = 0) -> None:
    lib().ftar_set_tuning(blocks_per_cu, flags)


def ftar_time_next_launch(start_event, stop_event) -> None:
    """start_event / stop_event: raw hipEvent_t handles (ints or ctypes void pointers) or None."""
    lib().ftar_time_next_launch(start_event, stop_event)


def ftar_status_is_retryable(status: int) -> bool:
    return bool(lib().ftar_status_is_retryable(status))


def ftar_status_str(status: int) -> str:
    return lib().ftar_status_str(status).decode()


def ftar_last_error() -> int:
    return lib().ftar_last_error()


def ftar_reduce_scatter_all(plan: Plan, bufs: Sequence[Optional[torch.Tensor]], stream=None) -> None:
    _check_bufs(bufs, plan.live_mask, plan.count, plan.dtype)
    if len(bufs) != plan.n_replicas:
        raise ValueError("bufs must have one entry per replica slot")
    st = lib().ftar_reduce_scatter_all(plan.handle, _ptr_array(bufs), _stream_handle(stream))
    if st != FTAR_OK:
        raise FtarError(st, "ftar_reduce_scatter_all")


def ftar_allgather_all(plan: Plan, bufs: Sequence[Optional[torch.Tensor]], stream=None) -> None:
    _check_bufs(bufs, plan.live_mask, plan.count, plan.dtype)
    if len(bufs) != plan.n_replicas:
        raise ValueError("bufs must have one entry per replica slot")
    st = lib().ftar_allgather_all(plan.handle, _ptr_array(bufs), _stream_handle(stream))
    if st != FTAR_OK:
        raise FtarError(st, "ftar_allgather_all")


def ftar_allreduce_onepass(plan: Plan, bufs: Sequence[Optional[torch.Tensor]], stream=None) -> None:
    _check_bufs(bufs, plan.live_mask, plan.count, plan.dtype)
    if len(bufs) != plan.n_replicas:
        raise ValueError("bufs must have one entry per replica slot")
    st = lib().ftar_allreduce_onepass(plan.handle, _ptr_array(bufs), _stream_handle(stream))
    if st != FTAR_OK:
        raise FtarError(st, "ftar_allreduce_onepass")


class Ctrl:
    """Owner of a control block for ftar_ring_persistent (coherent host-pinned memory)."""

    def __init__(self):
        self.handle = lib().ftar_ctrl_create()
        if not self.handle:
            raise FtarError(lib().ftar_last_error(), "ftar_ctrl_create")

    def last_ticket(self) -> int:
        """Ticket of the call enqueued last on this control block (-1: none)."""
        return lib().ftar_ctrl_last_ticket(self.handle)

    def release(self, n_units: int, ticket: Optional[int] = None) -> None:
        if ticket is None:
            lib().ftar_ctrl_release(self.handle, n_units)
        else:
            lib().ftar_ctrl_release_call(self.handle, ticket, n_units)

    def cancel(self) -> None:
        lib().ftar_ctrl_cancel(self.handle)

    def progress(self, ticket: Optional[int] = None) -> int:
        if ticket is None:
            return lib().ftar_ctrl_progress(self.handle)
        return lib().ftar_ctrl_progress_call(self.handle, ticket)

    def result(self, ticket: Optional[int] = None):
        """(status, units_done); call after the stream has been synchronised."""
        done = ctypes.c_int()
        if ticket is None:
            st = lib().ftar_ctrl_result(self.handle, ctypes.byref(done))
        else:
            st = lib().ftar_ctrl_result_call(self.handle, ticket, ctypes.byref(done))
        return st, done.value

    def destroy(self) -> None:
        if self.handle:
            lib().ftar_ctrl_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def ftar_ctrl_create() -> Ctrl:
    return Ctrl()


def ftar_ctrl_destroy(ctrl: Ctrl) -> None:
    ctrl.destroy()


def ftar_ctrl_release(ctrl: Ctrl, n_units: int) -> None:
    ctrl.release(n_units)


def ftar_ctrl_last_ticket(ctrl: Ctrl) -> int:
    return ctrl.last_ticket()


def ftar_ctrl_release_call(ctrl: Ctrl, ticket: int, n_units: int) -> None:
    ctrl.release(n_units, ticket)


def ftar_ctrl_progress_call(ctrl: Ctrl, ticket: int) -> int:
    return ctrl.progress(ticket)


def ftar_ctrl_result_call(ctrl: Ctrl, ticket: int):
    return ctrl.result(ticket)


def ftar_plan_n_gate_units(plan: Plan, flags: int = 0) -> int:
    return plan.n_gate_units(flags)


def ftar_ctrl_cancel(ctrl: Ctrl) -> None:
    ctrl.cancel()


def ftar_ctrl_progress(ctrl: Ctrl) -> int:
    return ctrl.progress()


def ftar_ctrl_result(ctrl: Ctrl):
    return ctrl.result()


def ftar_ring_persistent(plan: Plan, bufs: Sequence[Optional[torch.Tensor]],
                         acc: Optional[torch.Tensor], ctrl: Ctrl, n_blocks: int = 0,
                         timeout_us: int = 2_000_000, flags: int = 0, stream=None) -> None:
    _check_bufs(bufs, plan.live_mask, plan.count, plan.dtype)
    if len(bufs) != plan.n_replicas:
        raise ValueError("bufs must have one entry per replica slot")
    if acc is not None and (acc.dtype != torch.float32 or acc.numel() * 4 < plan.acc_bytes or not acc.is_cuda):
        raise ValueError("acc must be a GPU float32 tensor of at least one partition")
    st = lib().ftar_ring_persistent(plan.handle, _ptr_array(bufs),
                                    None if acc is None else acc.data_ptr(), ctrl.handle, n_blocks,
                                    timeout_us, flags, _stream_handle(stream))
    if st != FTAR_OK:
        raise FtarError(st, "ftar_ring_persistent")


def ftar_ring_persistent_static(plan: Plan, bufs: Sequence[Optional[torch.Tensor]], ctrl: Ctrl,
                                n_blocks: int = 0, timeout_us: int = 2_000_000, flags: int = 0,
                                stream=None) -> None:
    """ftar_ring_persistent on the library's static scratch: no acc argument, nothing allocated."""
    _check_bufs(bufs, plan.live_mask, plan.count, plan.dtype)
    if len(bufs) != plan.n_replicas:
        raise ValueError("bufs must have one entry per replica slot")
    st = lib().ftar_ring_persistent_static(plan.handle, _ptr_array(bufs), ctrl.handle, n_blocks,
                                           timeout_us, flags, _stream_handle(stream))
    if st != FTAR_OK:
        raise FtarError(st, "ftar_ring_persistent_static")


def ring_allreduce(plan: Plan, bufs: Sequence[Optional[torch.Tensor]], acc: Optional[torch.Tensor],
                   stream=None) -> None:
    """The full schedule as the caller would drive it: N-1 ReduceScatter then N-1 AllGather calls."""
    for s in range(plan.n_steps):
        ftar_reduce_step(plan, s, bufs, acc, stream)
    for t in range(plan.n_steps):
        ftar_allgather_step(plan, t, bufs, stream)
