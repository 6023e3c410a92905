"""GPU parity of the cost-only call and of the most probable alignment, through the C ABI.

Cost-only (grads == NULL): costs against the oracle to the tolerances of the full call, and
bitwise equal to the full call's costs (same forward recursion).

Most probable alignment (Section 5.1, alignment step): the score is unique and is compared
with the oracle's (1e-4 relative for fp32 activations, 2e-2 for bf16); the alignment itself
need not be (ties, and near-ties within rounding), so it is checked for what must hold: it is
a legal walk over the blank-interleaved label from a start state to an end state, frames past
the end are -1, and its own probability, evaluated in float64, equals the best score within
the same tolerance.  How many utterances reproduce the oracle's alignment exactly is printed
and must be the large majority.
"""
import numpy as np
import pytest

from oracle import ctc_oracle as orc
from paper_1512_02595_amd import ctc, harness
from paper_1512_02595_amd import workloads as wl

pytestmark = pytest.mark.gpu


from parity_checks import check_best, check_loss, log_softmax  # noqa: F401


# ---------------------------------------------------------------- cost only

@pytest.mark.parametrize("index", [0, 1, 2, 3, 5])
def test_loss_only_configs(index):
    check_loss(wl.make_config(index))


def test_loss_only_sweep_bf16():
    check_loss(wl.make_config(4, B=128), ctc.DTYPE_BF16)


def test_loss_only_odd_shapes():
    check_loss(wl.make_random(2, T=40, B=9, A=9, max_label=30))                      # many infeasible
    check_loss(wl.make_random(4, T=300, B=7, A=5, max_label=290, min_input=250, feasible_only=True))
    check_loss(wl.make_random(11, T=9, B=3, A=2051, max_label=6, blank=2050))        # wide, scalar rows
    check_loss(wl.make_random(16, T=9, B=3, A=4104, max_label=6, blank=7))           # wide, vector rows


# ---------------------------------------------------------------- most probable alignment

@pytest.mark.parametrize("index", [0, 1, 2, 3, 5])
def test_best_path_configs(index):
    check_best(wl.make_config(index))


def test_best_path_sweep_fp32_and_bf16():
    check_best(wl.make_config(4, B=128))
    check_best(wl.make_config(4, B=128), ctc.DTYPE_BF16, min_same=0.3)   # bf16 logits tie often


@pytest.mark.parametrize("seed,kw", [
    (1, dict(T=12, B=5, A=6, max_label=4)),
    (2, dict(T=40, B=9, A=9, max_label=30)),
    (3, dict(T=70, B=6, A=3, max_label=69, min_input=60)),
    (4, dict(T=300, B=7, A=5, max_label=290, min_input=250, feasible_only=True)),
    (5, dict(T=33, B=4, A=2, max_label=20, blank=1)),
    (6, dict(T=25, B=8, A=40, max_label=12, blank=39, sigma=4.0)),
    (8, dict(T=64, B=5, A=64, max_label=63, feasible_only=True)),
    (12, dict(T=9, B=3, A=9000, max_label=5, min_input=6, blank=4000, feasible_only=True)),
    (17, dict(T=200, B=4, A=29, max_label=0)),                      # empty labels only
])
def test_best_path_random_shapes(seed, kw):
    check_best(wl.make_random(seed, **kw))


def test_best_path_longest_supported_label():
    T, A = 1100, 6
    rng = np.random.default_rng(31)
    L = ctc.MAX_LABEL_LENGTH
    # no adjacent repeats: each symbol is its predecessor moved on by 1..A-2 places among the A-1 symbols
    lab = (1 + np.cumsum(rng.integers(1, A - 1, size=L)) % (A - 1)).astype(np.int32)
    assert (lab[1:] != lab[:-1]).all() and lab.min() >= 1 and lab.max() < A
    x = (rng.standard_normal((T, 2, A)) * 2.0).astype(np.float32)
    batch = wl.CTCBatch(name="longest", T=T, B=2, A=A, blank=0, logits=x,
                        flat_labels=np.concatenate([lab, lab[:700]]).astype(np.int32),
                        label_lengths=np.asarray([L, 700], dtype=np.int32),
                        input_lengths=np.asarray([T, 900], dtype=np.int32), seed=31)
    check_best(batch)
    check_loss(batch)


def test_best_path_recovers_a_planted_alignment():
    """Logits that favour one legal walk by a wide margin: exactly that walk must come back."""
    rng = np.random.default_rng(41)
    T, B, A = 500, 5, 29
    labs, walks = [], []
    x = (rng.standard_normal((T, B, A)) * 0.5).astype(np.float32)
    tlen = np.asarray([500, 431, 377, 250, 64], dtype=np.int32)
    for b in range(B):
        L = int(rng.integers(20, 120)) if b < 4 else 30
        lab = rng.integers(1, A, size=L)
        S = 2 * L + 1
        # advance at the frames of a random subset, so that the walk ends on the last state
        t_adv = np.sort(rng.choice(np.arange(1, tlen[b]), size=S - 1, replace=False))
        s = np.zeros(tlen[b], dtype=np.int64)
        s[t_adv] = 1
        s = np.cumsum(s)
        sym = np.where(s % 2 == 0, 0, lab[np.maximum(s - 1, 0) // 2])
        x[np.arange(tlen[b]), b, sym] += 8.0
        labs.append(lab)
        walks.append(s)
    batch = wl.CTCBatch(name="planted", T=T, B=B, A=A, blank=0, logits=x,
                        flat_labels=np.concatenate(labs).astype(np.int32),
                        label_lengths=np.asarray([len(l) for l in labs], dtype=np.int32),
                        input_lengths=tlen, seed=41)
    _, states = check_best(batch, min_same=1.0)
    for b in range(B):
        assert np.array_equal(states[b, :tlen[b]], walks[b]), b


def test_best_path_repeats_bitwise_and_leaves_the_other_calls_intact():
    batch = wl.make_config(1)
    db = harness.DeviceBatch(batch)
    db.run_best_path()
    s1, a1 = db.best_path_results()
    db.run()                                     # the full call reuses the same workspace
    c_full, g_full = db.results()
    db.run_best_path()
    s2, a2 = db.best_path_results()
    assert np.array_equal(s1, s2) and np.array_equal(a1, a2)
    db2 = harness.DeviceBatch(batch)
    db2.run()
    c_ref, g_ref = db2.results()
    assert np.array_equal(c_full, c_ref) and np.array_equal(g_full, g_ref)
    assert (s1 >= c_ref - 1e-3).all()            # the best alignment cannot beat the sum over all


def test_a_lost_wavefront_exchange_is_reported_as_nan_cost():
    """With a poll budget of zero every wait between the wavefronts of a long label gives up at once:
    all kernels still run to their end, and the utterances concerned report NaN in all three calls,
    while labels that fit one wavefront are unaffected.  (The label of 400 symbols takes the recursion
    whose lanes own two state pairs each, those of 120 and 150 the one-pair recursion.)"""
    rng = np.random.default_rng(51)
    T, A = 420, 7
    lengths = np.asarray([150, 40, 400, 10, 120, 63], dtype=np.int32)
    # labels without adjacent repeats, so that every utterance has an alignment
    labs = [(1 + np.cumsum(rng.integers(1, A - 1, size=n)) % (A - 1)).astype(np.int32) for n in lengths]
    batch = wl.CTCBatch(name="lost-exchange", T=T, B=len(lengths), A=A, blank=0,
                        logits=(rng.standard_normal((T, len(lengths), A)) * 2.0).astype(np.float32),
                        flat_labels=np.concatenate(labs), label_lengths=lengths,
                        input_lengths=np.full(len(lengths), T, dtype=np.int32), seed=51)
    multi = lengths + 1 > 64
    ref = orc.ctc_loss_and_grad(batch.logits, batch.flat_labels, batch.label_lengths, batch.input_lengths,
                                batch.blank, want_grad=False)[0]
    assert np.isfinite(ref).all()
    try:
        ctc.debug_set_poll_budget(0)
        db = harness.DeviceBatch(batch)
        for run in (db.run, db.run_loss, db.run_best_path):
            db.poison()
            run()
            costs, _ = db.results()
            assert np.isnan(costs[multi]).all(), (run.__name__, costs)
            assert np.isfinite(costs[~multi]).all(), (run.__name__, costs)
        assert (db.alignment.cpu().numpy()[multi] == -1).all()
    finally:
        ctc.debug_set_poll_budget(-1)
    db = harness.DeviceBatch(batch)
    db.run()
    costs, _ = db.results()
    assert np.abs(costs - ref).max() <= 1e-4 * np.abs(ref).max()
