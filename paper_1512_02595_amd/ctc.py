"""ctypes binding of libctc_mi355x.so: argument marshalling only.

The functions mirror include/ctc_mi355x.h.  Device buffers are passed as integer
addresses (for instance torch.Tensor.data_ptr()), host arrays as numpy int32
arrays.  There is no fallback: if the library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libctc_mi355x.so")

STATUS_SUCCESS = 0
STATUS_INVALID_VALUE = 1
STATUS_WORKSPACE_TOO_SMALL = 2
STATUS_HIP_ERROR = 3
STATUS_UNSUPPORTED = 4
STATUS_NOT_READY = 5

DTYPE_F32 = 0
DTYPE_BF16 = 1

MAX_LABEL_LENGTH = 1023
NUM_KERNELS = 3

KERNEL_BACKTRACE = 3          # name index of the third launch of best_path

EXPORTS = ("ctc_workspace_size", "ctc_loss_and_grad", "ctc_profile_kernels",
           "ctc_best_path", "ctc_profile_best_path",
           "ctc_workspace_size_device", "ctc_loss_and_grad_device", "ctc_loss_and_grad_device_static",
           "ctc_profile_kernels_device", "ctc_debug_set_sequential_chains",
           "ctc_kernel_name", "ctc_status_string", "ctc_last_hip_error", "ctc_debug_set_poll_budget",
           "ctc_debug_staging_allocations", "ctc_debug_set_overlap", "ctc_debug_replay_emission_fetches")

_lib = None


class CTCError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


def load() -> ctypes.CDLL:
    """Loads the HIP library (once).  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_1512_02595_amd.build` "
                          "(there is no CPU fallback)")
    lib = ctypes.CDLL(LIB_PATH)
    i32p = ctypes.POINTER(ctypes.c_int32)
    vp, st, ci = ctypes.c_void_p, ctypes.c_int, ctypes.c_int
    lib.ctc_workspace_size.restype = st
    lib.ctc_workspace_size.argtypes = [ci, ci, ci, i32p, i32p, ci, ctypes.POINTER(ctypes.c_size_t)]
    common = [vp, i32p, i32p, i32p, ci, ci, ci, ci, ci, vp, vp, vp, ctypes.c_size_t, vp]
    lib.ctc_loss_and_grad.restype = st
    lib.ctc_loss_and_grad.argtypes = common
    lib.ctc_profile_kernels.restype = st
    lib.ctc_profile_kernels.argtypes = common + [ctypes.POINTER(ctypes.c_float)]
    lib.ctc_best_path.restype = st
    lib.ctc_best_path.argtypes = common
    lib.ctc_profile_best_path.restype = st
    lib.ctc_profile_best_path.argtypes = common + [ctypes.POINTER(ctypes.c_float)]
    lib.ctc_workspace_size_device.restype = st
    lib.ctc_workspace_size_device.argtypes = [ci, ci, ci, ci, ci, ctypes.POINTER(ctypes.c_size_t)]
    lib.ctc_loss_and_grad_device.restype = st
    lib.ctc_loss_and_grad_device.argtypes = [vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, vp, vp, vp, vp,
                                             ctypes.c_size_t, vp]
    lib.ctc_profile_kernels_device.restype = st
    lib.ctc_profile_kernels_device.argtypes = [vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, vp, vp, vp, vp,
                                               ctypes.c_size_t, vp, ctypes.POINTER(ctypes.c_float)]
    lib.ctc_loss_and_grad_device_static.restype = st
    lib.ctc_loss_and_grad_device_static.argtypes = [vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, vp, vp, vp, vp]
    lib.ctc_kernel_name.restype = ctypes.c_char_p
    lib.ctc_kernel_name.argtypes = [ci]
    lib.ctc_status_string.restype = ctypes.c_char_p
    lib.ctc_status_string.argtypes = [st]
    lib.ctc_last_hip_error.restype = ci
    lib.ctc_last_hip_error.argtypes = []
    lib.ctc_debug_set_poll_budget.restype = None
    lib.ctc_debug_set_poll_budget.argtypes = [ci]
    lib.ctc_debug_replay_emission_fetches.restype = ctypes.c_long
    lib.ctc_debug_replay_emission_fetches.argtypes = [ci, ci, ci, i32p, i32p, ci, ctypes.POINTER(ctypes.c_long)]
    lib.ctc_debug_set_overlap.restype = None
    lib.ctc_debug_set_overlap.argtypes = [ci]
    lib.ctc_debug_set_sequential_chains.restype = None
    lib.ctc_debug_set_sequential_chains.argtypes = [ci]
    lib.ctc_debug_staging_allocations.restype = ctypes.c_long
    lib.ctc_debug_staging_allocations.argtypes = []
    _lib = lib
    return lib


def _i32(a, allow_none=False):
    if a is None and allow_none:
        return None, None
    arr = np.ascontiguousarray(a, dtype=np.int32).reshape(-1)
    return arr, arr.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def status_string(status: int) -> str:
    return load().ctc_status_string(int(status)).decode()


def kernel_name(index: int):
    s = load().ctc_kernel_name(int(index))
    return s.decode() if s is not None else None


def last_hip_error() -> int:
    return int(load().ctc_last_hip_error())


def workspace_size_status(T, B, A, label_lengths, input_lengths, dtype=DTYPE_F32):
    """(status, bytes) of ctc_workspace_size, without raising."""
    _ll, llp = _i32(label_lengths, allow_none=True)
    _il, ilp = _i32(input_lengths, allow_none=True)
    out = ctypes.c_size_t(0)
    st = load().ctc_workspace_size(int(T), int(B), int(A), llp, ilp, int(dtype), ctypes.byref(out))
    return int(st), int(out.value)


def workspace_size(T, B, A, label_lengths, input_lengths, dtype=DTYPE_F32) -> int:
    st, n = workspace_size_status(T, B, A, label_lengths, input_lengths, dtype)
    if st != STATUS_SUCCESS:
        raise CTCError(st, "ctc_workspace_size")
    return n


def loss_and_grad_status(activations_ptr, flat_labels, label_lengths, input_lengths, T, B, A, blank,
                         dtype, costs_ptr, grads_ptr, workspace_ptr, workspace_bytes, stream=0,
                         kernel_ms=None) -> int:
    """Raw call; returns the status.  With `kernel_ms` (float32 numpy array of NUM_KERNELS)
    the profiling entry point is used and the array is filled.  grads_ptr None (or 0): costs only."""
    _fl, flp = _i32(flat_labels, allow_none=True)
    _ll, llp = _i32(label_lengths, allow_none=True)
    _il, ilp = _i32(input_lengths, allow_none=True)
    args = [ctypes.c_void_p(activations_ptr), flp, llp, ilp, int(T), int(B), int(A), int(blank),
            int(dtype), ctypes.c_void_p(costs_ptr), ctypes.c_void_p(grads_ptr),
            ctypes.c_void_p(workspace_ptr), ctypes.c_size_t(workspace_bytes), ctypes.c_void_p(stream)]
    lib = load()
    if kernel_ms is None:
        return int(lib.ctc_loss_and_grad(*args))
    assert kernel_ms.dtype == np.float32 and kernel_ms.size >= NUM_KERNELS
    return int(lib.ctc_profile_kernels(*args, kernel_ms.ctypes.data_as(ctypes.POINTER(ctypes.c_float))))


def loss_and_grad(activations_ptr, flat_labels, label_lengths, input_lengths, T, B, A, blank,
                  dtype, costs_ptr, grads_ptr, workspace_ptr, workspace_bytes, stream=0,
                  kernel_ms=None) -> None:
    st = loss_and_grad_status(activations_ptr, flat_labels, label_lengths, input_lengths, T, B, A,
                              blank, dtype, costs_ptr, grads_ptr, workspace_ptr, workspace_bytes,
                              stream, kernel_ms)
    if st != STATUS_SUCCESS:
        extra = f" (hipError {last_hip_error()})" if st == STATUS_HIP_ERROR else ""
        raise CTCError(st, "ctc_loss_and_grad" + extra)


def best_path_status(activations_ptr, flat_labels, label_lengths, input_lengths, T, B, A, blank,
                     dtype, scores_ptr, alignment_ptr, workspace_ptr, workspace_bytes, stream=0,
                     kernel_ms=None) -> int:
    """Raw ctc_best_path (ctc_profile_best_path with `kernel_ms`); returns the status."""
    _fl, flp = _i32(flat_labels, allow_none=True)
    _ll, llp = _i32(label_lengths, allow_none=True)
    _il, ilp = _i32(input_lengths, allow_none=True)
    args = [ctypes.c_void_p(activations_ptr), flp, llp, ilp, int(T), int(B), int(A), int(blank),
            int(dtype), ctypes.c_void_p(scores_ptr), ctypes.c_void_p(alignment_ptr),
            ctypes.c_void_p(workspace_ptr), ctypes.c_size_t(workspace_bytes), ctypes.c_void_p(stream)]
    lib = load()
    if kernel_ms is None:
        return int(lib.ctc_best_path(*args))
    assert kernel_ms.dtype == np.float32 and kernel_ms.size >= NUM_KERNELS
    return int(lib.ctc_profile_best_path(*args, kernel_ms.ctypes.data_as(ctypes.POINTER(ctypes.c_float))))


def best_path(activations_ptr, flat_labels, label_lengths, input_lengths, T, B, A, blank,
              dtype, scores_ptr, alignment_ptr, workspace_ptr, workspace_bytes, stream=0,
              kernel_ms=None) -> None:
    st = best_path_status(activations_ptr, flat_labels, label_lengths, input_lengths, T, B, A,
                          blank, dtype, scores_ptr, alignment_ptr, workspace_ptr, workspace_bytes,
                          stream, kernel_ms)
    if st != STATUS_SUCCESS:
        extra = f" (hipError {last_hip_error()})" if st == STATUS_HIP_ERROR else ""
        raise CTCError(st, "ctc_best_path" + extra)


def workspace_size_device_status(T, B, A, max_label_length, dtype=DTYPE_F32):
    out = ctypes.c_size_t(0)
    st = load().ctc_workspace_size_device(int(T), int(B), int(A), int(max_label_length), int(dtype),
                                          ctypes.byref(out))
    return int(st), int(out.value)


def workspace_size_device(T, B, A, max_label_length, dtype=DTYPE_F32) -> int:
    st, n = workspace_size_device_status(T, B, A, max_label_length, dtype)
    if st != STATUS_SUCCESS:
        raise CTCError(st, "ctc_workspace_size_device")
    return n


def loss_and_grad_device_status(activations_ptr, labels_ptr, label_lengths_ptr, input_lengths_ptr,
                                max_label_length, T, B, A, blank, dtype, costs_ptr, grads_ptr,
                                status_ptr, workspace_ptr, workspace_bytes, stream=0, kernel_ms=None) -> int:
    """Raw ctc_loss_and_grad_device: every array argument is a device address.  With `kernel_ms` (float32
    numpy array of NUM_KERNELS) the profiling entry point is used and the array is filled."""
    if kernel_ms is not None:
        assert kernel_ms.dtype == np.float32 and kernel_ms.size >= NUM_KERNELS
        return int(load().ctc_profile_kernels_device(
            ctypes.c_void_p(activations_ptr), ctypes.c_void_p(labels_ptr), ctypes.c_void_p(label_lengths_ptr),
            ctypes.c_void_p(input_lengths_ptr), int(max_label_length), int(T), int(B), int(A), int(blank),
            int(dtype), ctypes.c_void_p(costs_ptr), ctypes.c_void_p(grads_ptr), ctypes.c_void_p(status_ptr),
            ctypes.c_void_p(workspace_ptr), ctypes.c_size_t(workspace_bytes), ctypes.c_void_p(stream),
            kernel_ms.ctypes.data_as(ctypes.POINTER(ctypes.c_float))))
    return int(load().ctc_loss_and_grad_device(
        ctypes.c_void_p(activations_ptr), ctypes.c_void_p(labels_ptr), ctypes.c_void_p(label_lengths_ptr),
        ctypes.c_void_p(input_lengths_ptr), int(max_label_length), int(T), int(B), int(A), int(blank),
        int(dtype), ctypes.c_void_p(costs_ptr), ctypes.c_void_p(grads_ptr), ctypes.c_void_p(status_ptr),
        ctypes.c_void_p(workspace_ptr), ctypes.c_size_t(workspace_bytes), ctypes.c_void_p(stream)))


STATIC_WORKSPACE_BYTES = 64 << 20


def loss_and_grad_device_static_status(activations_ptr, labels_ptr, label_lengths_ptr, input_lengths_ptr,
                                       max_label_length, T, B, A, blank, dtype, costs_ptr, grads_ptr,
                                       status_ptr, stream=0) -> int:
    """Raw ctc_loss_and_grad_device_static: the device-metadata call on the library's own workspace."""
    return int(load().ctc_loss_and_grad_device_static(
        ctypes.c_void_p(activations_ptr), ctypes.c_void_p(labels_ptr), ctypes.c_void_p(label_lengths_ptr),
        ctypes.c_void_p(input_lengths_ptr), int(max_label_length), int(T), int(B), int(A), int(blank),
        int(dtype), ctypes.c_void_p(costs_ptr), ctypes.c_void_p(grads_ptr), ctypes.c_void_p(status_ptr),
        ctypes.c_void_p(stream)))


def loss_and_grad_device(*args, **kw) -> None:
    st = loss_and_grad_device_status(*args, **kw)
    if st != STATUS_SUCCESS:
        extra = f" (hipError {last_hip_error()})" if st == STATUS_HIP_ERROR else ""
        raise CTCError(st, "ctc_loss_and_grad_device" + extra)


def debug_set_poll_budget(polls: int) -> None:
    """LDS polls a lattice wavefront may spend waiting on its neighbour (negative: default)."""
    load().ctc_debug_set_poll_budget(int(polls))


def debug_staging_allocations() -> int:
    """Pinned host allocations the library has made so far in this process."""
    return int(load().ctc_debug_staging_allocations())


def debug_set_sequential_chains(on: bool) -> None:
    """Measurements: forward and backward recursions in two launches, one after the other."""
    load().ctc_debug_set_sequential_chains(1 if on else 0)


def debug_set_overlap(percent: int) -> None:
    """Gradient rows inside the lattice launch where it leaves compute units idle: 0 off, 1..100 the
    share of the launch within which an utterance's chains must end, negative the default."""
    load().ctc_debug_set_overlap(int(percent))


def debug_replay_emission_fetches(T, B, A, label_lengths, input_lengths, max_label_length=-1):
    """(reads outside their region, smallest margin in floats) of the chains' emission fetch schedule,
    replayed on the host against the workspace layout (host-metadata layout, or bounds layout)."""
    _ll, llp = _i32(label_lengths)
    _il, ilp = _i32(input_lengths)
    margin = ctypes.c_long(0)
    n = load().ctc_debug_replay_emission_fetches(int(T), int(B), int(A), llp, ilp, int(max_label_length),
                                                 ctypes.byref(margin))
    return int(n), int(margin.value)
