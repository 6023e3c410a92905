"""The lattice kernels read emissions ahead of the recursion without bounds checks (up to three chunks
past either end of an utterance's block); the workspace has margins for that.  A mismatch between the
two has faulted a GPU before, so it is checked here without one: the library replays, on the host, the
chains' own fetch schedule and address arithmetic (shared code, not a copy) against the workspace
layout and counts reads outside their region.  No GPU needed."""
import itertools

import numpy as np
import pytest

from paper_1512_02595_amd import ctc

FRAMES = list(range(1, 65)) + [750, 1500]
LABELS = [0, 1, 63, 64, 1023]


def batch_with(Tb, L, where, T):
    """Three utterances, the one under test first, in the middle or last; neighbours as small as can be."""
    frames = [1, 1, 1]
    labels = [0, 0, 0]
    frames[where], labels[where] = Tb, L
    return np.asarray(labels, dtype=np.int32), np.asarray(frames, dtype=np.int32)


@pytest.mark.parametrize("A", [29, 64, 65, 600])          # symbol-major emission block up to 64 symbols, gathered beyond
def test_every_emission_read_stays_inside_its_region(A):
    checked = 0
    for Tb, L, where in itertools.product(FRAMES, LABELS, (0, 1, 2)):
        T = max(Tb, 2)
        labels, frames = batch_with(Tb, L, where, T)
        for bound in (-1, int(labels.max()), ctc.MAX_LABEL_LENGTH):      # host layout; bounds layout, tight and widest
            bad, margin = ctc.debug_replay_emission_fetches(T, 3, A, labels, frames, bound)
            assert bad == 0, (A, Tb, L, where, bound, bad, margin)
            assert margin >= 0
            checked += 1
    assert checked == len(FRAMES) * len(LABELS) * 3 * 3


def test_the_five_workload_shapes():
    from paper_1512_02595_amd import workloads as wl
    for idx in range(6):
        b = wl.make_config(idx)
        for bound in (-1, int(b.label_lengths.max())):
            if bound >= 0 and b.B > 4096:
                continue
            bad, margin = ctc.debug_replay_emission_fetches(b.T, b.B, b.A, b.label_lengths, b.input_lengths, bound)
            assert bad == 0 and margin >= 0, (idx, bound, bad, margin)


def test_the_replay_notices_a_read_outside():
    """The checker itself: a batch whose lengths contradict the tensor is refused (-1), and the margin it
    reports for a single short utterance is what the fetch schedule implies -- the constants that lanes
    without a label state read sit 8 floats into the region and a fetch reads the 8 floats before them."""
    assert ctc.debug_replay_emission_fetches(10, 1, 29, [3], [11], -1)[0] == -1
    bad, margin = ctc.debug_replay_emission_fetches(40, 1, 29, [5], [40], -1)
    assert bad == 0 and margin == 0
