"""GPU tests of ctc_loss_and_grad_device: lengths and labels on the device, nothing read from the host.

Every shape is compared with the CPU oracle, element by element, to the tolerances of the
host-metadata call (costs 1e-4 relative, gradients 1e-4 absolute; bf16: 2e-2 and 1e-2), and with
the host-metadata call itself: bitwise where both calls plan the same chains, within rounding
where the bounds make the device call plan otherwise.  Invalid entries are reported through the
device status word; and the call can be recorded into a HIP graph and replayed on new buffer
contents.
"""
import numpy as np
import pytest
import torch

from oracle import ctc_oracle as orc
from paper_1512_02595_amd import ctc, harness
from paper_1512_02595_amd import workloads as wl

pytestmark = pytest.mark.gpu


def both_paths(batch, dtype=ctc.DTYPE_F32, max_label=None, same_kernels=True):
    print(f"device-metadata case {batch.name} seed={batch.seed} T={batch.T} B={batch.B} A={batch.A}", flush=True)
    max_label = int(batch.label_lengths.max()) if max_label is None else max_label
    dm = harness.DeviceMetaBatch(batch.T, batch.B, batch.A, max_label, batch.blank, dtype)
    dm.load(batch)
    dm.poison()
    dm.run()
    status, costs, grads = dm.results()
    ref_costs, ref_grads = harness.run_batch(batch, dtype)
    assert status == ctc.STATUS_SUCCESS
    # against the oracle, as the host-metadata call is checked
    logits = batch.logits if dtype == ctc.DTYPE_F32 else wl.to_bf16_grid(batch.logits)
    orc_c, orc_g = orc.ctc_loss_and_grad(logits, batch.flat_labels, batch.label_lengths, batch.input_lengths,
                                         batch.blank)
    rtol, atol = (1e-4, 1e-4) if dtype == ctc.DTYPE_F32 else (2e-2, 1e-2)
    inf = np.isinf(orc_c)
    assert np.array_equal(np.isinf(costs) & (costs > 0), inf) and not np.isnan(costs).any()
    err_c = np.abs(costs[~inf] - orc_c[~inf]) / np.maximum(np.abs(orc_c[~inf]), 1e-2)
    err_g = np.abs(grads - orc_g).max()
    print(f"  against the oracle: max cost rel err {err_c.max() if err_c.size else 0.0:.3e}  "
          f"max grad abs err {err_g:.3e}", flush=True)
    assert err_c.size == 0 or err_c.max() <= rtol
    assert err_g <= atol
    for b in range(batch.B):
        assert not grads[batch.input_lengths[b]:, b, :].any()
        if inf[b]:
            assert not grads[:, b, :].any()
    if same_kernels:
        assert np.array_equal(costs, ref_costs, equal_nan=True)
        assert np.array_equal(grads, ref_grads)
    else:
        # a different recursion kernel: the same numbers up to rounding
        assert np.array_equal(np.isfinite(costs), np.isfinite(ref_costs))
        ok = np.isfinite(ref_costs)
        if ok.any():                                             # (a batch may hold no utterance with an alignment)
            assert np.abs(costs[ok] - ref_costs[ok]).max() <= 1e-5 * max(np.abs(ref_costs[ok]).max(), 1e-2)
        assert np.abs(grads - ref_grads).max() <= 2e-5
    return dm, costs, grads


def test_matches_the_host_metadata_call_bitwise_and_the_oracle():
    batch = wl.make_config(0)
    both_paths(batch, max_label=40)           # bound larger than any label


@pytest.mark.parametrize("maker", [
    lambda: wl.make_config(1),
    lambda: wl.make_config(5, B=16),
    lambda: wl.make_config(2, B=8),
    lambda: wl.make_random(2, T=40, B=9, A=9, max_label=30),                                   # infeasible pairs
    lambda: wl.make_random(4, T=300, B=7, A=5, max_label=290, min_input=250, feasible_only=True),  # several wavefronts
    lambda: wl.make_random(17, T=50, B=4, A=29, max_label=0),                                  # empty labels
    lambda: wl.make_random(81, T=120, B=6, A=7, max_label=40, min_input=90, sigma=60.0, feasible_only=True),  # emissions below the linear range
    lambda: wl.make_random(6, T=420, B=3, A=4, max_label=400, min_input=410, feasible_only=True),  # two pairs per lane
])
def test_matches_the_host_metadata_call_on_other_shapes(maker):
    both_paths(maker())


def test_bounds_far_above_the_actual_labels():
    """A label bound that only the barrier kernel serves, on a batch of short labels; and a bound that makes
    the launch as wide as sixteen wavefronts while the labels need one or two."""
    # (the barrier kernel recurs on logarithms, the host call's kernel for short labels on probabilities)
    both_paths(wl.make_random(31, T=60, B=3, A=5, max_label=20, min_input=30), max_label=ctc.MAX_LABEL_LENGTH,
               same_kernels=False)
    both_paths(wl.make_random(32, T=150, B=5, A=6, max_label=100, min_input=120, feasible_only=True), max_label=900)


def test_launch_of_more_chains_than_the_chip_runs_side_by_side():
    """The 512-utterance sweep at full size: from the bounds alone the call takes the launch for a crowded one
    (lengths spread evenly up to the bound would put more than two wavefronts on every SIMD) and plans its chains
    for total work, as the host-metadata call does from the actual lengths."""
    both_paths(wl.make_config(4), same_kernels=False)


def test_bf16_and_cost_only():
    batch = wl.make_config(4, B=32)
    both_paths(batch, ctc.DTYPE_BF16)
    dm = harness.DeviceMetaBatch(batch.T, batch.B, batch.A, int(batch.label_lengths.max()), batch.blank)
    dm.load(batch)
    dm.poison()
    dm.run(want_grad=False)
    status, costs, grads = dm.results()
    ref_costs, _ = harness.run_batch(batch)
    assert status == ctc.STATUS_SUCCESS and np.array_equal(costs, ref_costs)
    assert np.isnan(grads).all()                                 # untouched


def test_invalid_entries_are_reported_on_the_device():
    batch = wl.make_random(21, T=30, B=6, A=7, max_label=8, min_input=20, feasible_only=True)
    Lmax = 8
    dm = harness.DeviceMetaBatch(batch.T, batch.B, batch.A, Lmax, batch.blank)
    ref_costs, ref_grads = harness.run_batch(batch)
    pad = np.zeros((batch.B, Lmax), dtype=np.int32)
    off = 0
    for b in range(batch.B):
        L = int(batch.label_lengths[b])
        pad[b, :L] = batch.flat_labels[off:off + L]
        off += L
    bad = batch.label_lengths.argmax()                            # an utterance with at least one label
    cases = []
    p1 = pad.copy(); p1[bad, 0] = batch.blank; cases.append((p1, None, None, [bad]))          # blank in a label
    p2 = pad.copy(); p2[bad, 0] = batch.A; cases.append((p2, None, None, [bad]))              # outside the alphabet
    ll = batch.label_lengths.copy(); ll[1] = Lmax + 1; cases.append((pad, ll, None, [1]))     # longer than the bound
    il = batch.input_lengths.copy(); il[2] = batch.T + 1; il[3] = -1; cases.append((pad, None, il, [2, 3]))
    for raw, ll_, il_, which in cases:
        dm.load(batch, raw_labels=raw)
        if ll_ is not None:
            dm.label_lengths.copy_(torch.from_numpy(ll_.astype(np.int32)))
        if il_ is not None:
            dm.input_lengths.copy_(torch.from_numpy(il_.astype(np.int32)))
        dm.poison()
        dm.run()
        status, costs, grads = dm.results()
        assert status == ctc.STATUS_INVALID_VALUE
        for b in range(batch.B):
            if b in which:
                assert np.isnan(costs[b]) and not grads[:, b, :].any()
            else:
                assert costs[b] == ref_costs[b] and np.array_equal(grads[:, b, :], ref_grads[:, b, :])
    dm.load(batch)
    dm.poison()
    dm.run()
    status, costs, _ = dm.results()
    assert status == ctc.STATUS_SUCCESS and np.array_equal(costs, ref_costs)


def test_host_side_checks_of_the_device_call():
    assert ctc.workspace_size_device_status(10, 4, 5, ctc.MAX_LABEL_LENGTH + 1)[0] == ctc.STATUS_UNSUPPORTED
    assert ctc.workspace_size_device_status(10, 5000, 5, 3)[0] == ctc.STATUS_UNSUPPORTED
    assert ctc.workspace_size_device_status(0, 4, 5, 3)[0] == ctc.STATUS_INVALID_VALUE
    dm = harness.DeviceMetaBatch(10, 2, 5, 3)
    args = [dm.x.data_ptr(), dm.labels.data_ptr(), dm.label_lengths.data_ptr(), dm.input_lengths.data_ptr(),
            3, 10, 2, 5, 0, ctc.DTYPE_F32, dm.costs.data_ptr(), dm.grads.data_ptr(), dm.status.data_ptr(),
            dm.ws_ptr, dm.ws_bytes]
    def call(i, v):
        a = list(args); a[i] = v
        return ctc.loss_and_grad_device_status(*a)
    assert call(12, None) == ctc.STATUS_INVALID_VALUE            # no status word
    assert call(8, 5) == ctc.STATUS_INVALID_VALUE                # blank outside the alphabet
    assert call(14, dm.ws_bytes - 1) == ctc.STATUS_WORKSPACE_TOO_SMALL
    assert call(11, dm.x.data_ptr() + 16) == ctc.STATUS_INVALID_VALUE   # gradient overlaps the activations
    assert call(13, dm.ws_ptr + 8) == ctc.STATUS_INVALID_VALUE


def test_recorded_into_a_graph_and_replayed_on_new_contents():
    T, B, A, Lmax = 120, 12, 29, 40
    batches = [wl.make_random(100 + i, T=T, B=B, A=A, max_label=Lmax, min_input=30, sigma=2.0) for i in range(4)]
    dm = harness.DeviceMetaBatch(T, B, A, Lmax)
    dm.load(batches[0])
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                                # warm-up outside the capture
        dm.run(stream=side.cuda_stream)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        dm.run(stream=torch.cuda.current_stream().cuda_stream)
    # replays: each on fresh contents of the same buffers, with eager work of the program between them
    for rep, batch in enumerate(batches[1:] + batches[:2]):
        ref_costs, ref_grads = harness.run_batch(batch)          # eager, host-metadata call
        dm.load(batch)
        dm.poison()
        torch.cuda.synchronize()
        graph.replay()
        status, costs, grads = dm.results()
        print(f"  replay {rep}: status {status}", flush=True)
        assert status == ctc.STATUS_SUCCESS
        assert np.array_equal(costs, ref_costs, equal_nan=True)
        assert np.array_equal(grads, ref_grads)
