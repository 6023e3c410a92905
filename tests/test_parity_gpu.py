"""Parity of the HIP path against the CPU oracle, element by element, through the C ABI.

Tolerances (fp32 activations): costs within 1e-4 relative (floored at |ref| = 1e-2),
gradients within 1e-4 absolute.  bf16 activations: the oracle is fed the bf16-rounded
logits; costs within 2e-2 relative, gradients within 1e-2 absolute (the output itself is
rounded to bf16).  +inf costs must match exactly.
"""
import numpy as np
import pytest

from oracle import ctc_oracle as orc
from paper_1512_02595_amd import ctc, harness
from paper_1512_02595_amd import workloads as wl

pytestmark = pytest.mark.gpu

from parity_checks import BF16_COST_RTOL, BF16_GRAD_ATOL, COST_RTOL, GRAD_ATOL, check, check_best  # noqa: F401


def test_tiny_config():
    check(wl.make_config(0))


def test_english_config():
    check(wl.make_config(1))


def test_long_config():
    check(wl.make_config(3))


def test_mandarin_config():
    check(wl.make_config(2))


def test_sweep_config_fp32():
    check(wl.make_config(4))


def test_sweep_config_bf16():
    check(wl.make_config(4), ctc.DTYPE_BF16)


def test_bigram_alphabet_config():
    """Mid-size alphabet (Section 3.5: bigrams + unigrams, stride 3), fp32 and bf16."""
    check(wl.make_config(5))
    check(wl.make_config(5), ctc.DTYPE_BF16)


@pytest.mark.parametrize("seed,kw", [
    (1, dict(T=12, B=5, A=6, max_label=4)),
    (2, dict(T=40, B=9, A=9, max_label=30)),                       # many infeasible pairs
    (3, dict(T=70, B=6, A=3, max_label=69, min_input=60)),         # labels spanning two wavefronts
    (4, dict(T=300, B=7, A=5, max_label=290, min_input=250, feasible_only=True)),   # up to 5 wavefronts
    (5, dict(T=33, B=4, A=2, max_label=20, blank=1)),              # one non-blank symbol: all repeats
    (6, dict(T=25, B=8, A=40, max_label=12, blank=39, sigma=4.0)),
    (7, dict(T=20, B=3, A=1030, max_label=10, blank=517)),         # alphabet not a multiple of 4
    (8, dict(T=64, B=5, A=64, max_label=63, feasible_only=True)),
    (11, dict(T=9, B=3, A=2051, max_label=6, blank=2050)),          # wide alphabet, rows not 16-byte aligned
    (12, dict(T=9, B=3, A=9000, max_label=5, min_input=6, blank=4000, feasible_only=True)),          # wider than the register-resident path
    (13, dict(T=12, B=3, A=600, max_label=10, sigma=3.0)),          # mid-size alphabet (bigram-like)
])
def test_random_shapes(seed, kw):
    check(wl.make_random(seed, **kw))


@pytest.mark.parametrize("A", [63, 64, 65, 66])
def test_both_sides_of_the_emission_layouts(A):
    """Alphabets of up to 64 symbols keep the normalised rows, symbol-major, as the emission block; wider ones
    gather an emission per label position.  Same lengths on both sides of the switch, labels from one to three
    wavefronts wide (one and two state pairs per lane), utterances shorter than one fetch of eight frames
    included, fp32 and bf16."""
    rng = np.random.default_rng(640 + A)
    lengths = [0, 1, 3, 7, 30, 63, 64, 100, 150, 207, 208, 230, 260]
    frames = [1, 2, 5, 9, 40, 80, 70, 130, 170, 230, 215, 300, 300]
    T = max(frames)
    labs = []
    for n in lengths:                       # no adjacent repeats: every label fits its utterance
        lab = 1 + (np.cumsum(rng.integers(1, A - 2, size=n)) % (A - 1))
        labs.append(lab.astype(np.int32))
    batch = wl.CTCBatch(name="layouts", T=T, B=len(lengths), A=A, blank=0,
                        logits=(rng.standard_normal((T, len(lengths), A)) * 2.0).astype(np.float32),
                        flat_labels=np.concatenate(labs), label_lengths=np.asarray(lengths, dtype=np.int32),
                        input_lengths=np.asarray(frames, dtype=np.int32), seed=640 + A)
    costs, _, _, _ = check(batch)
    assert np.isfinite(costs).all()
    check(batch, ctc.DTYPE_BF16)


def test_random_shapes_bf16():
    check(wl.make_random(9, T=50, B=6, A=29, max_label=20, sigma=2.0, feasible_only=True), ctc.DTYPE_BF16)
    check(wl.make_random(10, T=30, B=3, A=1001, max_label=10), ctc.DTYPE_BF16)
    check(wl.make_random(14, T=8, B=2, A=4104, max_label=6), ctc.DTYPE_BF16)      # 16-byte vector path
    check(wl.make_random(15, T=8, B=2, A=4101, max_label=6), ctc.DTYPE_BF16)      # scalar wide path


def test_peaky_logits_like_a_trained_model():
    """Large-magnitude logits (per-frame probabilities from 1 - 1e-9 down to 1e-30): the mass sits on
    a thin band of the lattice, far below the maxima of alpha and of beta elsewhere."""
    rng = np.random.default_rng(77)
    T, B, A = 400, 6, 29
    lab_len = rng.integers(40, 120, size=B)
    labs = [rng.integers(1, A, size=n) for n in lab_len]
    x = rng.standard_normal((T, B, A)).astype(np.float32) * 2.0
    for b in range(B):                          # a plausible alignment gets +25, blanks elsewhere +20
        pos = np.sort(rng.choice(T, size=lab_len[b], replace=False))
        x[:, b, 0] += 20.0
        for i, t in enumerate(pos):
            x[t, b, 0] -= 20.0
            x[t, b, labs[b][i]] += 25.0
    batch = wl.CTCBatch(name="peaky", T=T, B=B, A=A, blank=0, logits=x,
                        flat_labels=np.concatenate(labs).astype(np.int32),
                        label_lengths=lab_len.astype(np.int32),
                        input_lengths=rng.integers(380, T + 1, size=B).astype(np.int32))
    check(batch)


def test_worst_case_spread_of_random_logits():
    """sigma = 6 logits without any structure: costs of several thousand nats per utterance."""
    check(wl.make_random(78, T=600, B=4, A=29, max_label=170, min_input=550, sigma=6.0, feasible_only=True))


def test_emissions_too_small_for_the_linear_domain():
    """Logit spreads of hundreds of nats: emissions below 2^-100 send an utterance's recursions to the
    log domain.  First every utterance (single- and multi-wavefront labels), then a launch in which one
    utterance of several has one such frame."""
    check(wl.make_random(81, T=120, B=6, A=7, max_label=40, min_input=90, sigma=60.0, feasible_only=True))
    check(wl.make_random(82, T=260, B=4, A=5, max_label=200, min_input=250, sigma=45.0, feasible_only=True))
    check(wl.make_random(83, T=30, B=3, A=900, max_label=12, min_input=20, sigma=40.0, feasible_only=True))
    batch = wl.make_random(84, T=90, B=5, A=29, max_label=30, min_input=70, sigma=2.0, feasible_only=True)
    lab = batch.labels_of(2)
    assert len(lab) > 0
    batch.logits[11, 2, lab[0]] = -300.0                # one label symbol at e^-300 in one frame of utterance 2
    check(batch)


def test_steep_fronts_just_inside_the_linear_domain():
    """Every label emission near 2^-90 (blank 62 nats above the symbols), labels of up to 200 symbols:
    neighbouring lattice states differ by ninety binary orders of magnitude at the fronts, close to
    the most that the linear-domain recursion's nine-pair exponent window is built for."""
    rng = np.random.default_rng(85)
    T, B, A = 500, 4, 4
    lab_len = np.array([200, 150, 63, 64])
    labs = [rng.integers(1, A, size=n) for n in lab_len]
    x = rng.standard_normal((T, B, A)).astype(np.float32)
    x[:, :, 0] += 62.0
    batch = wl.CTCBatch(name="steep", T=T, B=B, A=A, blank=0, logits=x,
                        flat_labels=np.concatenate(labs).astype(np.int32),
                        label_lengths=lab_len.astype(np.int32),
                        input_lengths=np.array([500, 480, 200, 450], dtype=np.int32))
    check(batch)


def test_renewals_put_off_in_single_wavefront_chains():
    """Batches whose labels all fit one wavefront run the chain that renews its lanes' exponents only
    when needed.  Long quiet stretches (most renewals skipped), steep fronts (every chunk shrinks the
    values by hundreds of binary orders), peaky rows (neighbouring lanes far apart) and stretches of
    likely and of nearly impossible label symbols in turn (values that grow again after shrinking)."""
    check(wl.make_random(91, T=1200, B=6, A=29, max_label=60, min_input=1000, sigma=2.0, feasible_only=True))
    rng = np.random.default_rng(92)
    T, B, A = 600, 5, 4
    lab_len = np.array([63, 40, 12, 1, 55])
    labs = [rng.integers(1, A, size=n) for n in lab_len]
    x = rng.standard_normal((T, B, A)).astype(np.float32)
    x[:, :, 0] += 62.0                                   # every label emission near 2^-90
    check(wl.CTCBatch(name="steep1", T=T, B=B, A=A, blank=0, logits=x,
                      flat_labels=np.concatenate(labs).astype(np.int32), label_lengths=lab_len.astype(np.int32),
                      input_lengths=np.array([600, 580, 300, 64, 590], dtype=np.int32)))
    x = rng.standard_normal((T, B, A)).astype(np.float32)
    for t0 in range(0, T, 50):                           # 25 frames of likely symbols, 25 of symbols near 2^-85
        x[t0:t0 + 25, :, 0] -= 8.0
        x[t0 + 25:t0 + 50, :, 0] += 58.0
    check(wl.CTCBatch(name="swing1", T=T, B=B, A=A, blank=0, logits=x,
                      flat_labels=np.concatenate(labs).astype(np.int32), label_lengths=lab_len.astype(np.int32),
                      input_lengths=np.array([600, 580, 300, 64, 590], dtype=np.int32)))
    T, B, A = 400, 6, 29
    lab_len = rng.integers(20, 64, size=B)
    labs = [rng.integers(1, A, size=n) for n in lab_len]
    x = rng.standard_normal((T, B, A)).astype(np.float32) * 2.0
    for b in range(B):                                   # (as in the peaky case above)
        pos = np.sort(rng.choice(T, size=lab_len[b], replace=False))
        x[:, b, 0] += 20.0
        for i, t in enumerate(pos):
            x[t, b, 0] -= 20.0
            x[t, b, labs[b][i]] += 25.0
    check(wl.CTCBatch(name="peaky1", T=T, B=B, A=A, blank=0, logits=x,
                      flat_labels=np.concatenate(labs).astype(np.int32), label_lengths=lab_len.astype(np.int32),
                      input_lengths=rng.integers(380, T + 1, size=B).astype(np.int32)))


def test_single_symbol_alphabet_long_repeats():
    """Every label position repeats its predecessor: each needs a blank in between."""
    check(wl.make_random(79, T=500, B=3, A=2, max_label=240, min_input=490, blank=0, sigma=3.0,
                         feasible_only=True))


def test_two_million_frames():
    """Utterances as long as the linear-domain recursion takes (2^21 frames; the lanes' exponents go down to
    minus several millions) and one frame longer, which the launcher sends to the log domain."""
    rng = np.random.default_rng(91)
    T, B, A = (1 << 21) + 1, 2, 3
    x = rng.standard_normal((T, B, A)).astype(np.float32)
    labs = [rng.integers(1, A, size=5), rng.integers(1, A, size=70)]
    batch = wl.CTCBatch(name="two-million-frames", T=T, B=B, A=A, blank=0, logits=x,
                        flat_labels=np.concatenate(labs).astype(np.int32),
                        label_lengths=np.array([5, 70], dtype=np.int32),
                        input_lengths=np.array([T, T - 1], dtype=np.int32), seed=91)
    check(batch)


def test_degenerate_lengths():
    """Empty labels, zero frames, single frames, the feasibility boundary."""
    rng = np.random.default_rng(0)
    T, A = 9, 5
    labels = [[], [], [1], [1], [2, 2], [2, 2], [1, 2, 3, 4], [3, 3, 3], [4]]
    in_len = [0, 9, 0, 1, 2, 3, 4, 5, 9]
    b = wl.CTCBatch(name="degenerate", T=T, B=len(labels), A=A, blank=0,
                    logits=rng.standard_normal((T, len(labels), A), dtype=np.float32),
                    flat_labels=np.array([k for l in labels for k in l], dtype=np.int32),
                    label_lengths=np.array([len(l) for l in labels], dtype=np.int32),
                    input_lengths=np.array(in_len, dtype=np.int32))
    costs, _, _, _ = check(b)
    assert costs[0] == 0.0 and np.isinf(costs[2]) and np.isinf(costs[4]) and np.isfinite(costs[5])


def test_smallest_shapes():
    """One frame, one utterance, one symbol (the blank alone), and a single all-padding tensor."""
    rng = np.random.default_rng(2)
    def one(T, B, A, labels, in_len, blank=0):
        return wl.CTCBatch(name="smallest", T=T, B=B, A=A, blank=blank,
                           logits=rng.standard_normal((T, B, A), dtype=np.float32),
                           flat_labels=np.array([k for l in labels for k in l], dtype=np.int32),
                           label_lengths=np.array([len(l) for l in labels], dtype=np.int32),
                           input_lengths=np.array(in_len, dtype=np.int32))
    costs, grads, _, _ = check(one(1, 1, 1, [[]], [1]))             # the blank is the whole alphabet
    assert abs(costs[0]) < 1e-6 and np.abs(grads).max() < 1e-6
    check(one(1, 1, 2, [[1]], [1]))
    check(one(1, 1, 2, [[1]], [1], blank=0))
    check(one(3, 2, 1, [[], []], [3, 0]))
    costs, grads, _, _ = check(one(4, 3, 5, [[1], [2, 2], []], [0, 0, 0]))   # no valid frame at all
    assert np.isinf(costs[0]) and np.isinf(costs[1]) and costs[2] == 0.0 and not grads.any()
    for b in (one(1, 1, 2, [[1]], [1]), one(5, 2, 3, [[1, 2], []], [5, 2])):
        db = harness.DeviceBatch(b)
        db.run_best_path()
        scores, states = db.best_path_results()
        ref_s, ref_a = orc.ctc_best_path(b.logits, b.flat_labels, b.label_lengths, b.input_lengths, b.blank)
        assert np.allclose(scores, ref_s, rtol=1e-5) and np.array_equal(states, ref_a)


def test_longest_supported_label():
    L = ctc.MAX_LABEL_LENGTH
    rng = np.random.default_rng(1)
    T, A = L + 40, 4
    lab = rng.integers(1, A, size=L)
    for i in range(1, L):                      # no adjacent repeats, so that T suffices
        if lab[i] == lab[i - 1]:
            lab[i] = 1 + (lab[i] % (A - 1))
    b = wl.CTCBatch(name="maxlabel", T=T, B=2, A=A, blank=0,
                    logits=rng.standard_normal((T, 2, A), dtype=np.float32),
                    flat_labels=np.concatenate([lab, lab[:100]]).astype(np.int32),
                    label_lengths=np.array([L, 100], dtype=np.int32),
                    input_lengths=np.array([T, 300], dtype=np.int32))
    check(b)


def test_padding_may_hold_nan_and_results_repeat_bitwise():
    b = wl.make_random(21, T=48, B=6, A=11, max_label=15, min_input=10, feasible_only=True)
    clean_c, clean_g, _, _ = check(b)
    x = b.logits.copy()
    for i in range(b.B):
        x[b.input_lengths[i]:, i, :] = np.nan
    b2 = wl.CTCBatch(**{**b.__dict__, "logits": x})
    db = harness.DeviceBatch(b2)
    db.run()
    c1, g1 = db.results()
    assert np.array_equal(c1, clean_c) and np.array_equal(g1, clean_g)
    db.poison()
    db.run()
    c2, g2 = db.results()
    assert np.array_equal(c1, c2) and np.array_equal(g1, g2)


def test_back_to_back_calls_with_different_batches():
    """Host arrays are consumed before the call returns: a second call may follow at once."""
    b1 = wl.make_random(31, T=60, B=8, A=7, max_label=20, feasible_only=True)
    b2 = wl.make_random(32, T=60, B=8, A=7, max_label=20, feasible_only=True)
    d1, d2 = harness.DeviceBatch(b1), harness.DeviceBatch(b2)
    for _ in range(3):
        d1.run()
        d2.run()
    for d, b in ((d1, b1), (d2, b2)):
        c, g = d.results()
        rc, rg = orc.ctc_loss_and_grad(b.logits, b.flat_labels, b.label_lengths, b.input_lengths, b.blank)
        assert np.abs(g - rg).max() <= GRAD_ATOL
        fin = np.isfinite(rc)
        assert (np.abs(c[fin] - rc[fin]) <= COST_RTOL * np.maximum(np.abs(rc[fin]), 1e-2)).all()


def test_runs_on_a_side_stream():
    import torch
    b = wl.make_random(41, T=30, B=4, A=8, max_label=8, feasible_only=True)
    db = harness.DeviceBatch(b)
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        db.run()
    s.synchronize()
    c, g = db.results()
    rc, rg = orc.ctc_loss_and_grad(b.logits, b.flat_labels, b.label_lengths, b.input_lengths, b.blank)
    assert np.abs(g - rg).max() <= GRAD_ATOL


def test_device_side_errors_are_reported_as_status():
    b = wl.make_random(51, T=10, B=2, A=5, max_label=3, feasible_only=True)
    db = harness.DeviceBatch(b)
    args = dict(T=b.T, B=b.B, A=b.A, blank=b.blank, dtype=ctc.DTYPE_F32)
    st = ctc.loss_and_grad_status(db.x.data_ptr(), b.flat_labels, b.label_lengths, b.input_lengths,
                                  costs_ptr=db.costs.data_ptr(), grads_ptr=db.grads.data_ptr(),
                                  workspace_ptr=db.ws_ptr, workspace_bytes=db.ws_bytes - 1, **args)
    assert st == ctc.STATUS_WORKSPACE_TOO_SMALL
    st = ctc.loss_and_grad_status(db.x.data_ptr(), b.flat_labels, b.label_lengths, b.input_lengths,
                                  costs_ptr=db.costs.data_ptr(), grads_ptr=db.x.data_ptr(),
                                  workspace_ptr=db.ws_ptr, workspace_bytes=db.ws_bytes, **args)
    assert st == ctc.STATUS_INVALID_VALUE


def plan_boundary_batch(lengths, seed, A=6, T=1040):
    rng = np.random.default_rng(seed)
    labs = [(1 + np.cumsum(rng.integers(1, A - 1, size=n)) % (A - 1)).astype(np.int32) for n in lengths]
    t_b = np.asarray([min(T, max(n + 3, int(n * rng.uniform(1.0, 1.3)) + 2)) for n in lengths], dtype=np.int32)
    return wl.CTCBatch(name="plan-boundaries", T=T, B=len(lengths), A=A, blank=0,
                       logits=(rng.standard_normal((T, len(lengths), A)) * 2.0).astype(np.float32),
                       flat_labels=np.concatenate(labs), label_lengths=np.asarray(lengths, dtype=np.int32),
                       input_lengths=t_b, seed=seed)


@pytest.mark.parametrize("lengths", [
    # one pair per lane while that takes at most 4 wavefronts with halos of 16 to 32 pairs (up to 207
    # symbols: the alphabet is small, so the emission block is symbol-major), two pairs per lane beyond
    # (2 to 9 wavefronts, halos of 4 to 16 lanes); the best path always has one pair per lane (up to 16
    # wavefronts)
    sorted({62, 63, 64, 65, 95, 96, 97, 119, 120, 121, 159, 160, 161, 183, 184, 199, 200, 201, 206, 207, 208,
            209, 215, 216, 223, 224, 225, 231, 232, 233,
            234, 235, 236, 237, 238, 239, 240, 253, 254, 255, 256, 271, 272, 287, 288, 327, 328, 343, 344, 345,
            346, 399, 400, 431, 432, 433, 455, 456, 511, 512, 519, 520, 521, 567, 568, 607, 608, 609, 623, 624,
            679, 680, 695, 696, 697, 735, 736, 783, 784, 785, 791, 792, 847, 848, 871, 872, 873, 895, 896,
            902, 903}),
    # labels for which no halo is left with one pair per lane: the launch uses the barrier kernel
    [100, 903, 904, 960, 1023],
])
def test_every_wavefront_plan_boundary(lengths):
    """Label lengths on both sides of every change of the wavefront plans, all three calls: the exchange
    between wavefronts is exercised in every configuration the planners can produce."""
    batch = plan_boundary_batch(lengths, 77)
    costs, grads, _, _ = check(batch)
    assert np.isfinite(costs).all()
    # the cost-only call and the best path run the same chains in their own modes
    db = harness.DeviceBatch(batch)
    db.run_loss()
    loss_only, _ = db.results()
    assert np.array_equal(loss_only, costs)
    # The most probable alignment runs the same chains in its own mode (one pair per lane, up to 16
    # wavefronts): every utterance's score against the oracle's with a tolerance of its own, and every
    # returned walk validated (legal, ends where it must, its own float64 probability equal to the best
    # score), whether or not it is the oracle's; how many are identical is asserted separately.
    check_best(batch, min_same=0.9)


def test_two_pairs_per_lane_in_a_crowded_launch():
    """Seven hundred utterances whose labels need two wavefronts with one pair per lane: the launcher plans
    such a launch for total work, which gives two pairs to every lane (one wavefront for up to 127 symbols,
    two beyond)."""
    rng = np.random.default_rng(88)
    B, T, A = 700, 150, 5
    lengths = rng.integers(64, 141, size=B)
    labs = [(1 + np.cumsum(rng.integers(1, A - 1, size=n)) % (A - 1)).astype(np.int32) for n in lengths]
    batch = wl.CTCBatch(name="crowded", T=T, B=B, A=A, blank=0,
                        logits=(rng.standard_normal((T, B, A)) * 2.0).astype(np.float32),
                        flat_labels=np.concatenate(labs), label_lengths=lengths.astype(np.int32),
                        input_lengths=np.minimum(T, lengths + rng.integers(1, 12, size=B)).astype(np.int32), seed=88)
    costs, _, _, _ = check(batch)
    assert np.isfinite(costs).all()
    db = harness.DeviceBatch(batch)
    db.run_loss()
    loss_only, _ = db.results()
    assert np.abs(loss_only - costs).max() <= 1e-5 * np.abs(costs).max()      # (the cost-only launch is not crowded)


def test_many_random_shapes():
    """Forty seeded shapes drawn over the ranges the kernels switch on (alphabet 2 .. 2500, labels 0 .. 400,
    frames 1 .. 450, both activation types, any blank id), each through the full call and the cost-only call."""
    rng = np.random.default_rng(2025)
    for case in range(40):
        A = int(rng.choice([2, 3, 5, 16, 29, 64, 65, 300, 513, 2048, 2049, 2500]))
        T = int(rng.integers(1, 450))
        B = int(rng.integers(1, 9))
        max_label = int(min(T, rng.choice([0, 3, 20, 63, 64, 130, 400])))
        blank = int(rng.integers(0, A))
        dtype = ctc.DTYPE_BF16 if case % 5 == 4 else ctc.DTYPE_F32
        batch = wl.make_random(5000 + case, T=T, B=B, A=A, blank=blank, max_label=max_label,
                               min_input=int(rng.integers(0, T + 1)), sigma=float(rng.choice([1.0, 2.0, 5.0])),
                               feasible_only=bool(case % 3))
        costs, _, _, _ = check(batch, dtype)
        db = harness.DeviceBatch(batch, dtype)
        db.run_loss()
        loss_only, _ = db.results()
        assert np.array_equal(loss_only, costs)


def test_hardly_a_frame_to_spare_and_widely_spread_logits():
    """Utterances with exactly as many frames as their labels need, under logits spread over tens of nats:
    the one alignment left runs along the front of the lattice, a thousand and more binary orders below
    the states behind it, whose mass can no longer reach the end.  Such utterances run in the log domain
    (fewer than 16 frames to spare), and the linear domain keeps a pair within 2^-150 of its lane's frame
    where its neighbours are up to 2^950 heavier."""
    # (seed 9117: an utterance of 408 frames, 399 symbols, 9 repeats; one of 396 frames with 50 to spare)
    check(wl.make_random(9117, T=417, B=19, A=29, blank=23, max_label=409, min_input=387, sigma=6.0, feasible_only=True))
    # (seed 9406: 138 frames, 91 symbols, 47 repeats, emissions down to 2^-95: the front 2^1900 below its neighbours)
    check(wl.make_random(9406, T=150, B=158, A=3, blank=1, max_label=128, min_input=120, sigma=20.0, feasible_only=True))
    # (one symbol only: 445 frames for 223 symbols and 222 repeats)
    check(wl.make_random(9192, T=452, B=31, A=2, blank=1, max_label=450, min_input=433, sigma=6.0, feasible_only=True))


@pytest.mark.parametrize("A,blank", [(29, 0), (130, 129), (256, 255), (257, 256), (700, 3)])
def test_metadata_upload_launch_with_byte_and_word_labels(A, blank):
    """Minibatches of more than 128 utterances (and every alphabet above 64 symbols) send their metadata in a
    launch of its own, which builds the label words from the labels' bytes where a symbol fits one (alphabets of
    at most 256 symbols) and copies the words otherwise: both sides of that limit, with the largest symbol id
    in use as a label or as the blank."""
    batch = wl.make_random(7300 + A, T=70, B=150, A=A, blank=blank, max_label=40, min_input=30, sigma=2.0)
    top = A - 1 if blank != A - 1 else A - 2                    # the largest symbol a label may hold
    labels = batch.flat_labels.copy()
    labels[::7] = top
    batch = wl.CTCBatch(batch.name, batch.T, batch.B, batch.A, batch.blank, batch.logits, labels,
                        batch.label_lengths, batch.input_lengths, seed=batch.seed)
    check(batch)
