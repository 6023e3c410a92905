"""GPU test of ctc_loss_and_grad_device_static, the entry point that allocates nothing: its workspace
is an array inside the library's device code.  Called through the C ABI and compared with
ctc_loss_and_grad_device (the same kernels on a caller-provided workspace): bitwise, on two calls
in a row, the second with a smaller batch whose blocks land on memory that still holds the first
call's contents; each also against the CPU oracle to the tolerances of the other parity tests.
"""
import numpy as np
import pytest
import torch

from oracle import ctc_oracle as orc
from paper_1512_02595_amd import ctc, harness
from paper_1512_02595_amd import workloads as wl

pytestmark = pytest.mark.gpu


def run_static(dm):
    st = ctc.loss_and_grad_device_static_status(
        dm.x.data_ptr(), dm.labels.data_ptr(), dm.label_lengths.data_ptr(), dm.input_lengths.data_ptr(),
        dm.max_label, dm.T, dm.B, dm.A, dm.blank, dm.dtype, dm.costs.data_ptr(), dm.grads.data_ptr(),
        dm.status.data_ptr(), torch.cuda.current_stream(dm.device).cuda_stream)
    assert st == ctc.STATUS_SUCCESS, ctc.status_string(st)


def one_call(batch, max_label):
    print(f"static-workspace case {batch.name} seed={batch.seed} T={batch.T} B={batch.B} A={batch.A} "
          f"max_label={max_label}", flush=True)
    dm = harness.DeviceMetaBatch(batch.T, batch.B, batch.A, max_label, batch.blank)
    assert dm.ws_bytes <= ctc.STATIC_WORKSPACE_BYTES
    dm.load(batch)
    dm.poison()
    dm.run()                                             # the existing entry point, caller's workspace
    status, ref_costs, ref_grads = dm.results()
    assert status == ctc.STATUS_SUCCESS
    dm.poison()
    run_static(dm)
    status, costs, grads = dm.results()
    assert status == ctc.STATUS_SUCCESS
    assert np.array_equal(costs, ref_costs, equal_nan=True)
    assert np.array_equal(grads, ref_grads)
    orc_c, orc_g = orc.ctc_loss_and_grad(batch.logits, batch.flat_labels, batch.label_lengths,
                                         batch.input_lengths, batch.blank)
    inf = np.isinf(orc_c)
    assert np.array_equal(np.isinf(costs) & (costs > 0), inf) and not np.isnan(costs).any()
    err_c = np.abs(costs[~inf] - orc_c[~inf]) / np.maximum(np.abs(orc_c[~inf]), 1e-2)
    assert err_c.size == 0 or err_c.max() <= 1e-4
    assert np.abs(grads - orc_g).max() <= 1e-4
    return dm


def test_two_calls_in_a_row_the_second_smaller():
    # several wavefronts per chain and some infeasible pairs, then a small batch of short utterances
    first = wl.make_random(401, T=300, B=12, A=29, max_label=150, min_input=120, sigma=2.0)
    second = wl.make_random(402, T=40, B=3, A=29, max_label=12, min_input=20, sigma=2.0)
    one_call(first, 150)
    one_call(second, 12)
    one_call(first, 150)                                 # and back again, over the small call's leftovers


def test_shapes_beyond_the_static_workspace_are_refused():
    T, B, A, max_label = 750, 64, 29, 250                # the English-shaped minibatch by bounds: about 200 MB
    assert ctc.workspace_size_device(T, B, A, max_label) > ctc.STATIC_WORKSPACE_BYTES
    dm = harness.DeviceMetaBatch(8, 2, 5, 3)
    st = ctc.loss_and_grad_device_static_status(
        dm.x.data_ptr(), dm.labels.data_ptr(), dm.label_lengths.data_ptr(), dm.input_lengths.data_ptr(),
        max_label, T, B, A, 0, ctc.DTYPE_F32, dm.costs.data_ptr(), dm.grads.data_ptr(), dm.status.data_ptr(), 0)
    assert st == ctc.STATUS_WORKSPACE_TOO_SMALL          # refused on sizes alone: nothing was enqueued
    torch.cuda.synchronize()
