"""GPU tests of the pinned staging memory of the host-metadata calls (Section 4.3: no allocation
on the training step): one allocation at the first call on a device, none afterwards; a caller
that enqueues further ahead of the GPU than there are slots is never made to wait."""
import time

import numpy as np
import pytest
import torch

from oracle import ctc_oracle as orc
from paper_1512_02595_amd import ctc, harness
from paper_1512_02595_amd import workloads as wl

pytestmark = pytest.mark.gpu


def test_one_allocation_then_none():
    batches = [wl.make_random(300 + i, T=60, B=5, A=29, max_label=20, min_input=30, sigma=2.0) for i in range(3)]
    dbs = [harness.DeviceBatch(b) for b in batches]
    dbs[0].run()
    torch.cuda.synchronize()
    after_first = ctc.debug_staging_allocations()
    assert after_first >= 1                                # (other tests of this process may have grown the pools)
    for i in range(40):                                    # five times round the slots, the stream drained now and then
        dbs[i % 3].run()
        if i % 6 == 5:
            torch.cuda.synchronize()
    torch.cuda.synchronize()
    assert ctc.debug_staging_allocations() == after_first
    for db, b in zip(dbs, batches):
        costs, grads = db.results()
        ref_c, ref_g = orc.ctc_loss_and_grad(b.logits, b.flat_labels, b.label_lengths, b.input_lengths, b.blank)
        fin = np.isfinite(ref_c)
        assert np.abs(costs[fin] - ref_c[fin]).max() <= 1e-4 * np.abs(ref_c[fin]).max()
        assert np.abs(grads - ref_g).max() <= 1e-4


def test_calls_enqueued_behind_a_long_kernel_never_wait():
    """Forty calls go out while the stream is held up by a kernel that spins for about 50 ms: every call
    returns at once (the pools of slots double instead of the host waiting for a free slot, once per
    doubling), and once the stream drains every call's results are right."""
    batch = wl.make_random(310, T=80, B=6, A=29, max_label=25, min_input=40, sigma=2.0, feasible_only=True)
    dbs = [harness.DeviceBatch(batch) for _ in range(4)]
    dbs[0].run()
    torch.cuda.synchronize()
    before = ctc.debug_staging_allocations()
    torch.cuda._sleep(int(0.05 * 2.0e9))
    t0 = time.perf_counter()
    worst = 0.0
    for i in range(40):
        c0 = time.perf_counter()
        dbs[i % 4].run()
        worst = max(worst, time.perf_counter() - c0)
    enqueue = time.perf_counter() - t0
    torch.cuda.synchronize()
    total = time.perf_counter() - t0
    grown = ctc.debug_staging_allocations() - before
    print(f"  40 calls enqueued in {enqueue * 1e3:.2f} ms (slowest {worst * 1e3:.2f} ms), stream drained after "
          f"{total * 1e3:.1f} ms, {grown} further pinned allocations", flush=True)
    assert enqueue < 0.03 < total                          # the host was done long before the GPU
    assert grown <= 2                                      # 8 -> 16 -> 32 slots: earlier pools drain, the last serves
    ref_c, ref_g = orc.ctc_loss_and_grad(batch.logits, batch.flat_labels, batch.label_lengths,
                                         batch.input_lengths, batch.blank)
    for db in dbs:
        costs, grads = db.results()
        assert np.abs(costs - ref_c).max() <= 1e-4 * np.abs(ref_c).max()
        assert np.abs(grads - ref_g).max() <= 1e-4
    # and from here on the last pool (32 slots after two doublings) serves as many calls in flight
    # without allocating
    torch.cuda._sleep(int(0.05 * 2.0e9))
    for i in range(30):
        dbs[i % 4].run()
    torch.cuda.synchronize()
    assert ctc.debug_staging_allocations() - before == grown


def test_two_threads_on_two_streams():
    """Calls from several threads are serialised while they prepare and enqueue, and share the pinned slots;
    with a stream, a workspace and output buffers of its own each thread gets the results it gets alone."""
    import threading
    batches = [wl.make_config(1, B=16), wl.make_random(320, T=120, B=24, A=29, max_label=50, min_input=60, sigma=2.0)]
    refs = []
    for b in batches:
        d = harness.DeviceBatch(b)
        d.run()
        refs.append(d.results())
    dbs = [harness.DeviceBatch(b) for b in batches]
    streams = [torch.cuda.Stream() for _ in batches]
    torch.cuda.synchronize()
    failures = []

    def work(i):
        try:
            for _ in range(25):
                dbs[i].run(streams[i].cuda_stream)
            streams[i].synchronize()
        except Exception as e:                              # (surfaces in the main thread below)
            failures.append((i, repr(e)))

    print("  two threads, 25 calls each", flush=True)
    threads = [threading.Thread(target=work, args=(i,)) for i in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join(60)
    assert not any(t.is_alive() for t in threads) and not failures, failures
    for d, (rc, rg) in zip(dbs, refs):
        c, g = d.results()
        assert np.array_equal(c, rc, equal_nan=True) and np.array_equal(g, rg)
