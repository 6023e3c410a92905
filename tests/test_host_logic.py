"""Host-side checks that need no GPU: the C-ABI library loads, exports what the header
declares, sizes workspaces and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_1512_02595_amd import ctc
from paper_1512_02595_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(ctc.LIB_PATH):
        from paper_1512_02595_amd import build
        build.build()
    return ctc.load()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "ctc_mi355x.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ctc_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert set(names) == set(ctc.EXPORTS), names
    for n in names:
        assert getattr(lib, n) is not None


def test_status_strings_and_kernel_names(lib):
    assert ctc.status_string(ctc.STATUS_SUCCESS) == "success"
    assert len({ctc.status_string(i) for i in range(6)}) == 6
    assert ctc.status_string(ctc.STATUS_NOT_READY) == "too many calls in flight"
    assert ctc.debug_staging_allocations() >= 0        # (callable without a GPU; counts pinned allocations)
    names = [ctc.kernel_name(i) for i in range(ctc.NUM_KERNELS)]
    assert names == ["ctc_softmax", "ctc_lattice", "ctc_gradient"]
    assert ctc.kernel_name(ctc.KERNEL_BACKTRACE) == "ctc_backtrace"
    assert ctc.kernel_name(ctc.KERNEL_BACKTRACE + 1) is None and ctc.kernel_name(-1) is None
    assert ctc.last_hip_error() == 0


def test_workspace_size_grows_with_the_lattice(lib):
    small = ctc.workspace_size(50, 4, 29, [5, 6, 7, 8], [30, 40, 50, 45])
    big = ctc.workspace_size(50, 4, 29, [15, 16, 17, 18], [30, 40, 50, 45])
    assert small % 256 == 0 and big % 256 == 0 and big > small > 0
    # alpha and beta of the label states in fp64 (L+1 entries per frame each) dominate for long
    # utterances; the fp32 emissions are one per label position and frame, or, for alphabets of at
    # most 64 symbols, the frame's whole row
    T, L = 1500, 500
    n = ctc.workspace_size(T, 1, 100, [L], [T])
    assert n >= 2 * T * (L + 1) * 8 + T * L * 4
    assert n <= 2 * T * (L + 1) * 8 + T * L * 4 + (1 << 20)
    n = ctc.workspace_size(T, 1, 29, [L], [T])
    assert n >= 2 * T * (L + 1) * 8 + T * 29 * 4
    assert n <= 2 * T * (L + 1) * 8 + T * 29 * 4 + (1 << 20)
    # zero-frame and zero-label utterances are fine
    assert ctc.workspace_size(10, 3, 5, [0, 0, 3], [0, 10, 0]) > 0


def test_workspace_size_of_the_five_configs(lib):
    expect_min = {0: 0, 1: 60e6, 3: 250e6, 4: 400e6}
    for idx in (0, 1, 3, 4):
        b = wl.make_config(idx)
        n = ctc.workspace_size(b.T, b.B, b.A, b.label_lengths, b.input_lengths)
        assert n >= 8 * b.lattice_cells and n >= expect_min[idx]


def test_workspace_size_rejects_bad_shapes(lib):
    ok_l, ok_i = [3, 4], [10, 10]
    cases = [
        (dict(T=0, B=2, A=5), ok_l, ok_i, ctc.STATUS_INVALID_VALUE),
        (dict(T=10, B=0, A=5), ok_l, ok_i, ctc.STATUS_INVALID_VALUE),
        (dict(T=10, B=2, A=0), ok_l, ok_i, ctc.STATUS_INVALID_VALUE),
        (dict(T=10, B=2, A=5), [3, -1], ok_i, ctc.STATUS_INVALID_VALUE),
        (dict(T=10, B=2, A=5), ok_l, [10, 11], ctc.STATUS_INVALID_VALUE),
        (dict(T=10, B=2, A=5), ok_l, [-1, 5], ctc.STATUS_INVALID_VALUE),
        (dict(T=10, B=2, A=5), [3, ctc.MAX_LABEL_LENGTH + 1], ok_i, ctc.STATUS_UNSUPPORTED),
        (dict(T=10, B=2, A=5, dtype=7), ok_l, ok_i, ctc.STATUS_INVALID_VALUE),
    ]
    for kw, ll, il, want in cases:
        st, _ = ctc.workspace_size_status(kw["T"], kw["B"], kw["A"], ll, il, kw.get("dtype", ctc.DTYPE_F32))
        assert st == want, (kw, ll, il, st)
    st, _ = ctc.workspace_size_status(10, 2, 5, None, ok_i)
    assert st == ctc.STATUS_INVALID_VALUE
    st = lib.ctc_workspace_size(10, 2, 5, (ctypes.c_int32 * 2)(3, 4), (ctypes.c_int32 * 2)(10, 10), 0, None)
    assert st == ctc.STATUS_INVALID_VALUE
    assert ctc.workspace_size_status(10, 2, 5, [3, ctc.MAX_LABEL_LENGTH], ok_i)[0] == ctc.STATUS_SUCCESS
    big = 65536
    assert ctc.workspace_size_status(4, big, 3, [1] * big, [4] * big)[0] == ctc.STATUS_UNSUPPORTED
    assert ctc.workspace_size_status(4, big - 1, 3, [1] * (big - 1), [4] * (big - 1))[0] == ctc.STATUS_SUCCESS


def test_loss_and_grad_validates_before_any_device_work(lib):
    """All of these must return from validation; the pointers are never dereferenced."""
    T, B, A = 10, 2, 5
    ll, il, lab = [2, 1], [10, 8], [1, 2, 3]
    x, g, c, ws = 0x10000, 0x200000, 0x300000, 0x400000       # fake, suitably aligned addresses
    n = ctc.workspace_size(T, B, A, ll, il)

    def call(**kw):
        a = dict(activations_ptr=x, flat_labels=lab, label_lengths=ll, input_lengths=il, T=T, B=B, A=A,
                 blank=0, dtype=ctc.DTYPE_F32, costs_ptr=c, grads_ptr=g, workspace_ptr=ws, workspace_bytes=n)
        a.update(kw)
        return ctc.loss_and_grad_status(**a)

    assert call(activations_ptr=0) == ctc.STATUS_INVALID_VALUE
    assert call(costs_ptr=0) == ctc.STATUS_INVALID_VALUE
    # no gradient buffer is the cost-only form: it passes validation (and, without a device, stops there)
    assert call(grads_ptr=None) == ctc.STATUS_HIP_ERROR
    assert call(grads_ptr=None, workspace_bytes=n - 1) == ctc.STATUS_WORKSPACE_TOO_SMALL
    assert call(workspace_ptr=0) == ctc.STATUS_INVALID_VALUE
    assert call(workspace_ptr=ws + 8) == ctc.STATUS_INVALID_VALUE          # not 256-byte aligned
    assert call(blank=-1) == ctc.STATUS_INVALID_VALUE
    assert call(blank=A) == ctc.STATUS_INVALID_VALUE
    assert call(flat_labels=[1, 0, 3]) == ctc.STATUS_INVALID_VALUE          # a label equal to blank
    assert call(flat_labels=[1, 2, A]) == ctc.STATUS_INVALID_VALUE          # outside the alphabet
    assert call(flat_labels=[1, 2, -3]) == ctc.STATUS_INVALID_VALUE
    assert call(input_lengths=[10, 11]) == ctc.STATUS_INVALID_VALUE
    assert call(label_lengths=[2, -1]) == ctc.STATUS_INVALID_VALUE
    assert call(grads_ptr=x + 16) == ctc.STATUS_INVALID_VALUE               # overlaps the activations
    assert call(workspace_bytes=n - 1) == ctc.STATUS_WORKSPACE_TOO_SMALL
    assert call(label_lengths=[ctc.MAX_LABEL_LENGTH + 1, 1]) == ctc.STATUS_UNSUPPORTED
    assert call(dtype=5) == ctc.STATUS_INVALID_VALUE
    kms = np.zeros(ctc.NUM_KERNELS, dtype=np.float32)
    assert call(workspace_bytes=n - 1, kernel_ms=kms) == ctc.STATUS_WORKSPACE_TOO_SMALL


def test_best_path_validates_before_any_device_work(lib):
    T, B, A = 10, 2, 5
    ll, il, lab = [2, 1], [10, 8], [1, 2, 3]
    x, al, c, ws = 0x10000, 0x200000, 0x300000, 0x400000
    n = ctc.workspace_size(T, B, A, ll, il)

    def call(**kw):
        a = dict(activations_ptr=x, flat_labels=lab, label_lengths=ll, input_lengths=il, T=T, B=B, A=A,
                 blank=0, dtype=ctc.DTYPE_F32, scores_ptr=c, alignment_ptr=al, workspace_ptr=ws,
                 workspace_bytes=n)
        a.update(kw)
        return ctc.best_path_status(**a)

    assert call(activations_ptr=0) == ctc.STATUS_INVALID_VALUE
    assert call(scores_ptr=0) == ctc.STATUS_INVALID_VALUE
    assert call(alignment_ptr=0) == ctc.STATUS_INVALID_VALUE
    assert call(alignment_ptr=al + 2) == ctc.STATUS_INVALID_VALUE           # not int32-aligned
    assert call(blank=A) == ctc.STATUS_INVALID_VALUE
    assert call(flat_labels=[1, 0, 3]) == ctc.STATUS_INVALID_VALUE
    assert call(input_lengths=[10, 11]) == ctc.STATUS_INVALID_VALUE
    assert call(workspace_bytes=n - 1) == ctc.STATUS_WORKSPACE_TOO_SMALL
    assert call(label_lengths=[ctc.MAX_LABEL_LENGTH + 1, 1]) == ctc.STATUS_UNSUPPORTED
    kms = np.zeros(ctc.NUM_KERNELS, dtype=np.float32)
    assert call(workspace_bytes=n - 1, kernel_ms=kms) == ctc.STATUS_WORKSPACE_TOO_SMALL


def test_workload_generator_is_seeded_and_feasible():
    a, b = wl.make_config(1), wl.make_config(1)
    assert np.array_equal(a.logits, b.logits) and np.array_equal(a.flat_labels, b.flat_labels)
    for idx in (0, 1, 3, 4, 5):
        c = wl.make_config(idx)
        assert c.logits.shape == (c.T, c.B, c.A) and c.logits.dtype == np.float32
        assert c.input_lengths.max() <= c.T and c.label_lengths.max() <= ctc.MAX_LABEL_LENGTH
        for i in range(c.B):
            lab = c.labels_of(i)
            assert lab.min() >= 1 and lab.max() < c.A
            assert len(lab) + wl.repeats(lab) <= c.input_lengths[i]
    e = wl.make_config(1)
    rep = np.mean([wl.repeats(e.labels_of(i)) / max(1, len(e.labels_of(i)) - 1) for i in range(e.B)])
    assert 0.05 < rep < 0.12          # forced 5 % plus the 1/28 chance repeats


def test_bf16_rounding_helpers():
    x = np.array([1.0, 1.00390625, 1.01171875, -3.1415926, 1e-30, 65504.0], dtype=np.float32)
    r = wl.to_bf16_grid(x)
    assert np.array_equal(wl.bf16_bits_to_f32(wl.bf16_bits(x)), r)
    assert r[0] == 1.0 and r[1] == 1.0 and r[2] == 1.015625      # ties to even, then up
    assert np.all(np.abs(r - x) <= np.abs(x) * 2.0 ** -8)


def test_device_metadata_call_validates_on_the_host_what_the_host_can_see(lib):
    T, B, A, Lmax = 10, 2, 5, 3
    st, n = ctc.workspace_size_device_status(T, B, A, Lmax)
    assert st == ctc.STATUS_SUCCESS
    exact = ctc.workspace_size(T, B, A, [Lmax] * B, [T] * B)
    assert n == exact                                   # the bound layout is the exact one of a full-size batch
    assert ctc.workspace_size_device_status(T, B, A, ctc.MAX_LABEL_LENGTH + 1)[0] == ctc.STATUS_UNSUPPORTED
    assert ctc.workspace_size_device_status(T, 4097, A, Lmax)[0] == ctc.STATUS_UNSUPPORTED
    assert ctc.workspace_size_device_status(T, B, 0, Lmax)[0] == ctc.STATUS_INVALID_VALUE
    assert ctc.workspace_size_device_status(T, B, A, -1)[0] == ctc.STATUS_INVALID_VALUE
    x, lab, ll, il, c, g, stw, ws = (0x10000 * (i + 1) for i in range(8))     # fake aligned addresses
    args = [x, lab, ll, il, Lmax, T, B, A, 0, ctc.DTYPE_F32, c, g, stw, ws, n]

    def call(i, v):
        a = list(args)
        a[i] = v
        return ctc.loss_and_grad_device_status(*a)

    for i in (0, 2, 3, 10, 12, 13):                     # activations, lengths, costs, status word, workspace
        assert call(i, None) == ctc.STATUS_INVALID_VALUE
    assert call(1, None) == ctc.STATUS_INVALID_VALUE    # labels missing although max_label_length > 0
    assert call(8, A) == ctc.STATUS_INVALID_VALUE
    assert call(9, 7) == ctc.STATUS_INVALID_VALUE
    assert call(14, n - 1) == ctc.STATUS_WORKSPACE_TOO_SMALL
    assert call(13, ws + 8) == ctc.STATUS_INVALID_VALUE
    assert call(11, x + 16) == ctc.STATUS_INVALID_VALUE
