"""ctypes front end of the double-precision CPU oracle (oracle/ctc_oracle.c).

TEST INFRASTRUCTURE: not imported by the product package.  The shared object is
built with gcc on first use (and rebuilt when the C source is newer).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ctc_oracle.c")
_LIB = os.path.join(_HERE, "libctc_oracle.so")
_lock = threading.Lock()
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc -O2 -fopenmp; returns the library path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.run(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                        "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"], check=True)
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    with _lock:
        if _lib is None:
            lib = ctypes.CDLL(build())
            dp = ctypes.POINTER(ctypes.c_double)
            ip = ctypes.POINTER(ctypes.c_int)
            lib.ctc_oracle.restype = ctypes.c_int
            lib.ctc_oracle.argtypes = [dp, ctypes.c_int, ctypes.c_int, ctypes.c_int, ip, ip, ip,
                                       ctypes.c_int, dp, dp, dp, dp, ctypes.c_int, ctypes.c_int]
            lib.ctc_oracle_max_threads.restype = ctypes.c_int
            lib.ctc_oracle_best_path.restype = ctypes.c_int
            lib.ctc_oracle_best_path.argtypes = [dp, ctypes.c_int, ctypes.c_int, ctypes.c_int, ip, ip, ip,
                                                 ctypes.c_int, dp, ip, ctypes.c_int]
            _lib = lib
    return _lib


def max_threads() -> int:
    return int(_load().ctc_oracle_max_threads())


def _dptr(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double)) if a is not None else None


def _iptr(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int))


def ctc_loss_and_grad(logits, flat_labels, label_lengths, input_lengths, blank=0, *,
                      want_grad=True, want_lattice=False, nthreads=0):
    """Costs [B] (nats) and gradients [T,B,A] w.r.t. the logits, in float64.

    logits: [T,B,A] array (any float dtype; converted to float64).
    With want_lattice, also returns ln alpha and ln beta as [B,T,S_max] arrays
    (entries outside an utterance's T_b x S_b block are NaN).
    """
    x = np.ascontiguousarray(logits, dtype=np.float64)
    if x.ndim != 3:
        raise ValueError("logits must be [T,B,A]")
    T, B, A = x.shape
    lab = np.ascontiguousarray(flat_labels, dtype=np.int32).reshape(-1)
    ll = np.ascontiguousarray(label_lengths, dtype=np.int32).reshape(-1)
    il = np.ascontiguousarray(input_lengths, dtype=np.int32).reshape(-1)
    if len(ll) != B or len(il) != B or int(ll.sum()) != len(lab):
        raise ValueError("length arrays do not match the batch")
    if len(lab) == 0:
        lab = np.zeros(1, dtype=np.int32)
    costs = np.empty(B, dtype=np.float64)
    grads = np.empty_like(x) if want_grad else None
    la = lb = None
    s_pad = 0
    if want_lattice:
        s_pad = int(2 * (ll.max() if B else 0) + 1)
        la = np.full((B, T, s_pad), np.nan)
        lb = np.full((B, T, s_pad), np.nan)
    rc = _load().ctc_oracle(_dptr(x), T, B, A, _iptr(lab), _iptr(ll), _iptr(il), int(blank),
                            _dptr(costs), _dptr(grads), _dptr(la), _dptr(lb), s_pad, int(nthreads))
    if rc == 2:
        raise ValueError("oracle: invalid arguments (lengths or label ids out of range)")
    if rc != 0:
        raise MemoryError("oracle: allocation failed")
    out = (costs, grads)
    if want_lattice:
        out = out + (la, lb)
    return out


def ctc_best_path(logits, flat_labels, label_lengths, input_lengths, blank=0, *, nthreads=0):
    """Most probable alignment per utterance (Section 5.1, alignment step).

    Returns (scores [B] float64: -ln of the alignment's probability, +inf if none exists;
    states [B,T] int32: lattice state per frame, index into the blank-interleaved label
    (even = blank, odd s = label[(s-1)//2]), -1 for padding frames and infeasible utterances).
    """
    x = np.ascontiguousarray(logits, dtype=np.float64)
    if x.ndim != 3:
        raise ValueError("logits must be [T,B,A]")
    T, B, A = x.shape
    lab = np.ascontiguousarray(flat_labels, dtype=np.int32).reshape(-1)
    ll = np.ascontiguousarray(label_lengths, dtype=np.int32).reshape(-1)
    il = np.ascontiguousarray(input_lengths, dtype=np.int32).reshape(-1)
    if len(ll) != B or len(il) != B or int(ll.sum()) != len(lab):
        raise ValueError("length arrays do not match the batch")
    if len(lab) == 0:
        lab = np.zeros(1, dtype=np.int32)
    scores = np.empty(B, dtype=np.float64)
    states = np.empty((B, T), dtype=np.int32)
    rc = _load().ctc_oracle_best_path(_dptr(x), T, B, A, _iptr(lab), _iptr(ll), _iptr(il), int(blank),
                                      _dptr(scores), _iptr(states), int(nthreads))
    if rc == 2:
        raise ValueError("oracle: invalid arguments (lengths or label ids out of range)")
    if rc != 0:
        raise MemoryError("oracle: allocation failed")
    return scores, states
