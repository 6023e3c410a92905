"""GPU tests of the gradient rows written inside the lattice launch (launches that leave compute
units idle: few utterances, alphabets of at most 64 symbols).  Whatever share of the utterances the
launch's workers take (none, some, all), costs and gradients are bitwise the same, and they match
the CPU oracle to the usual tolerances."""
import numpy as np
import pytest

from oracle import ctc_oracle as orc
from paper_1512_02595_amd import ctc, harness
from paper_1512_02595_amd import workloads as wl

pytestmark = pytest.mark.gpu


def run_with(batch, dtype, percent):
    ctc.debug_set_overlap(percent)
    try:
        db = harness.DeviceBatch(batch, dtype)
        db.run()
        return db.results()
    finally:
        ctc.debug_set_overlap(-1)


@pytest.mark.parametrize("maker,dtype", [
    (lambda: wl.make_config(0), ctc.DTYPE_F32),
    (lambda: wl.make_config(1), ctc.DTYPE_F32),
    (lambda: wl.make_config(1), ctc.DTYPE_BF16),
    (lambda: wl.make_config(3, B=8), ctc.DTYPE_F32),                                            # long labels, several wavefronts
    (lambda: wl.make_random(2, T=40, B=9, A=9, max_label=30), ctc.DTYPE_F32),                   # infeasible pairs, zero rows
    (lambda: wl.make_random(4, T=300, B=7, A=5, max_label=290, min_input=250, feasible_only=True), ctc.DTYPE_F32),
    (lambda: wl.make_random(81, T=120, B=6, A=7, max_label=40, min_input=90, sigma=60.0, feasible_only=True), ctc.DTYPE_F32),  # log domain
    (lambda: wl.make_random(17, T=50, B=4, A=29, max_label=0), ctc.DTYPE_F32),                  # empty labels
    (lambda: wl.make_random(33, T=90, B=100, A=20, max_label=30, min_input=10), ctc.DTYPE_F32), # 200 chains: just under the limit
])
def test_same_results_whatever_the_workers_share(maker, dtype):
    batch = maker()
    print(f"overlap case {batch.name} seed={batch.seed} T={batch.T} B={batch.B} A={batch.A} dtype={dtype}", flush=True)
    ref_c, ref_g = run_with(batch, dtype, 0)                     # the whole gradient in a launch of its own
    logits = batch.logits if dtype == ctc.DTYPE_F32 else wl.to_bf16_grid(batch.logits)
    orc_c, orc_g = orc.ctc_loss_and_grad(logits, batch.flat_labels, batch.label_lengths, batch.input_lengths,
                                         batch.blank)
    rtol, atol = (1e-4, 1e-4) if dtype == ctc.DTYPE_F32 else (2e-2, 1e-2)
    inf = np.isinf(orc_c)
    assert np.array_equal(np.isinf(ref_c) & (ref_c > 0), inf) and not np.isnan(ref_c).any()
    err = np.abs(ref_c[~inf] - orc_c[~inf]) / np.maximum(np.abs(orc_c[~inf]), 1e-2)
    assert err.size == 0 or err.max() <= rtol
    assert np.abs(ref_g - orc_g).max() <= atol
    for percent in (30, 60, 80, 100):
        c, g = run_with(batch, dtype, percent)
        assert np.array_equal(c, ref_c, equal_nan=True), percent
        assert np.array_equal(g, ref_g), percent


def test_repeated_calls_on_one_workspace():
    """The counters and marks of one call must not leak into the next: alternating batches through one set
    of buffers of the larger shape's size."""
    a = wl.make_random(501, T=200, B=20, A=29, max_label=60, min_input=40, sigma=2.0)
    b = wl.make_random(502, T=200, B=20, A=29, max_label=60, min_input=150, sigma=2.0)
    refs = [run_with(x, ctc.DTYPE_F32, 0) for x in (a, b)]
    dbs = [harness.DeviceBatch(x) for x in (a, b)]
    donor = max(dbs, key=lambda d: d.ws_bytes)                   # one workspace for both: the larger one
    for d in dbs:
        d.ws, d.ws_ptr = donor.ws, donor.ws_ptr
    for i in range(6):
        d, (rc, rg) = dbs[i % 2], refs[i % 2]
        d.run()
        c, g = d.results()
        assert np.array_equal(c, rc, equal_nan=True) and np.array_equal(g, rg), i


@pytest.mark.parametrize("maker", [
    lambda: wl.make_config(0),
    lambda: wl.make_config(1),
    lambda: wl.make_config(3, B=8),                                                             # several wavefronts per chain
    lambda: wl.make_random(81, T=120, B=6, A=7, max_label=40, min_input=90, sigma=60.0, feasible_only=True),  # log domain
    lambda: wl.make_random(7, T=60, B=12, A=80, max_label=20, min_input=30),                    # frame-major emissions
])
def test_recursions_one_after_the_other_give_the_same_results(maker):
    """The measurement switch that runs the forward chains' launch before the backward chains' (the order
    of the paper's GPU design, CTC appendix) changes when things run, not what they compute."""
    batch = maker()
    print(f"sequential case {batch.name} seed={batch.seed} T={batch.T} B={batch.B} A={batch.A}", flush=True)
    ref_c, ref_g = run_with(batch, ctc.DTYPE_F32, 0)
    ctc.debug_set_sequential_chains(True)
    try:
        db = harness.DeviceBatch(batch, ctc.DTYPE_F32)
        db.run()
        c, g = db.results()
    finally:
        ctc.debug_set_sequential_chains(False)
    assert np.array_equal(c, ref_c, equal_nan=True)
    assert np.array_equal(g, ref_g)
