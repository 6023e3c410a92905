"""Seeded synthetic CTC batches shaped like Deep Speech 2's training minibatches.

This module only draws inputs (lengths, label strings, logits).  It holds none of
the CTC arithmetic and is the one piece shared by the GPU path's tests, the
benchmark and the CPU oracle's tests, so that all of them see identical inputs.

Shapes follow the paper's workload statistics (Section 3.1 alphabet, Section 3.9
Mandarin output layer of about 6000 characters, Section 4.1 minibatch of 64
utterances per GPU and 512 overall, Section 5.1 utterances of about 7 seconds):

  index 0  tiny        B=4    A=29    T=50    quick oracle-sized check
  index 1  english     B=64   A=29    T=750   per-GPU English minibatch
  index 2  mandarin    B=64   A=6000  T=500   wide alphabet, Zipf symbols
  index 3  long        B=32   A=29    T=1500  lattices of up to 1001 states
  index 4  sweep       B=512  A=29    T=750   whole 512-utterance minibatch, unsorted

Draw order for every config is input_lengths, label_lengths, labels, logits, from
numpy.random.Generator(PCG64(BASE_SEED + index)).  "N(0,2)" means a standard
deviation of 2.0.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

BASE_SEED = 151202595
BLANK = 0

# Index 5 is not one of the five headline workloads: a bigram-alphabet minibatch
# (Section 3.5: non-overlapping bigrams plus unigrams as output symbols, time stride 3).
CONFIG_NAMES = ("tiny", "english", "mandarin", "long", "sweep", "bigram")


@dataclass
class CTCBatch:
    """One synthetic minibatch.  `logits` is [T, B, A] float32, A fastest."""
    name: str
    T: int
    B: int
    A: int
    blank: int
    logits: np.ndarray
    flat_labels: np.ndarray      # int32, concatenation of the B label strings
    label_lengths: np.ndarray    # int32 [B]
    input_lengths: np.ndarray    # int32 [B]
    seed: int = 0
    notes: dict = field(default_factory=dict)

    def labels_of(self, b: int) -> np.ndarray:
        off = int(self.label_lengths[:b].sum())
        return self.flat_labels[off:off + int(self.label_lengths[b])]

    @property
    def frames(self) -> int:
        return int(self.input_lengths.sum())

    @property
    def lattice_cells(self) -> int:
        return int((self.input_lengths.astype(np.int64)
                    * (2 * self.label_lengths.astype(np.int64) + 1)).sum())

    def compulsory_bytes(self, elem_bytes: int = 4) -> int:
        """Read every valid logit row once and write the whole gradient tensor."""
        return (self.frames * self.A + self.T * self.B * self.A) * elem_bytes


def repeats(label: np.ndarray) -> int:
    """Number of positions whose symbol equals its predecessor."""
    if len(label) < 2:
        return 0
    return int(np.count_nonzero(label[1:] == label[:-1]))


def _force_repeats(rng, lab, prob):
    for i in range(1, len(lab)):
        if rng.random() < prob:
            lab[i] = lab[i - 1]
    return lab


def _zipf_table(n_symbols: int, s: float) -> np.ndarray:
    k = np.arange(1, n_symbols + 1, dtype=np.float64)
    w = k ** (-s)
    return w / w.sum()


def _draw_logits(rng, T, B, A, sigma, blank_shift, blank):
    x = rng.standard_normal((T, B, A), dtype=np.float32)
    if sigma != 1.0:
        x *= np.float32(sigma)
    if blank_shift:
        x[:, :, blank] += np.float32(blank_shift)
    return x


def make_config(index: int, *, seed: int | None = None, B: int | None = None) -> CTCBatch:
    """Build config `index` (0-based position in the list above).

    `B` overrides the batch size (used for bounded CPU-baseline samples and
    reduced-size parity cases); everything else keeps the config's recipe.
    """
    if not 0 <= index < len(CONFIG_NAMES):
        raise ValueError("config index must be in 0..5")
    seed = BASE_SEED + index if seed is None else seed
    rng = np.random.Generator(np.random.PCG64(seed))
    name = CONFIG_NAMES[index]
    blank = BLANK

    if index == 0:
        Bn, A, T = B or 4, 29, 50
        in_len = rng.integers(30, 51, size=Bn)
        lab_len = rng.integers(5, 16, size=Bn)
        labs = []
        for b in range(Bn):
            while True:
                lab = rng.integers(1, A, size=lab_len[b])
                if len(lab) + repeats(lab) <= in_len[b]:
                    break
            labs.append(lab)
        sigma, shift = 1.0, 0.0
    elif index in (1, 4):
        Bn, A, T = B or (64 if index == 1 else 512), 29, 750
        in_len = rng.integers(100, 751, size=Bn)
        frac = rng.uniform(0.15, 0.30, size=Bn)
        lab_len = np.floor(frac * in_len).astype(np.int64)
        labs = [_force_repeats(rng, rng.integers(1, A, size=lab_len[b]), 0.05) for b in range(Bn)]
        sigma, shift = 2.0, 3.0
    elif index == 2:
        Bn, A, T = B or 64, 6000, 500
        in_len = rng.integers(100, 501, size=Bn)
        lab_len = rng.integers(5, 61, size=Bn)
        pz = _zipf_table(A - 1, 1.1)
        labs = [rng.choice(A - 1, size=lab_len[b], p=pz) + 1 for b in range(Bn)]
        sigma, shift = 1.0, 3.0
    elif index == 5:
        # 15 s of audio at 10 ms frames and stride 3 -> up to 500 frames; 14.1 characters per
        # second regrouped into bigrams and unigrams give about 0.25 symbols per frame; the
        # alphabet holds the bigrams seen in training plus the unigrams (about 750 symbols),
        # drawn here with Zipf-like frequencies.
        Bn, A, T = B or 64, 750, 500
        in_len = rng.integers(67, 501, size=Bn)
        frac = rng.uniform(0.15, 0.35, size=Bn)
        lab_len = np.floor(frac * in_len).astype(np.int64)
        pz = _zipf_table(A - 1, 1.0)
        labs = [rng.choice(A - 1, size=lab_len[b], p=pz) + 1 for b in range(Bn)]
        sigma, shift = 2.0, 3.0
    else:
        Bn, A, T = B or 32, 29, 1500
        in_len = rng.integers(1200, 1501, size=Bn)
        lab_len = rng.integers(300, 501, size=Bn)
        labs = [rng.integers(1, A, size=lab_len[b]) for b in range(Bn)]
        sigma, shift = 2.0, 3.0

    logits = _draw_logits(rng, T, Bn, A, sigma, shift, blank)
    flat = (np.concatenate(labs) if labs else np.zeros(0)).astype(np.int32)
    return CTCBatch(name=name, T=T, B=Bn, A=A, blank=blank, logits=logits,
                    flat_labels=flat,
                    label_lengths=np.asarray(lab_len, dtype=np.int32),
                    input_lengths=np.asarray(in_len, dtype=np.int32),
                    seed=seed, notes={"sigma": sigma, "blank_shift": shift})


def make_random(seed: int, T: int, B: int, A: int, *, blank: int = 0,
                max_label: int | None = None, min_input: int = 0,
                sigma: float = 1.0, feasible_only: bool = False) -> CTCBatch:
    """Free-form random batch for edge-case and small parity tests.

    Lengths are uniform in [min_input, T] and [0, max_label]; symbols are uniform
    over the non-blank ids.  With feasible_only, label strings are shortened until
    they fit their utterance.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    max_label = T if max_label is None else max_label
    in_len = rng.integers(min_input, T + 1, size=B)
    lab_len = rng.integers(0, max_label + 1, size=B)
    nonblank = np.array([k for k in range(A) if k != blank], dtype=np.int64)
    labs = []
    for b in range(B):
        lab = nonblank[rng.integers(0, len(nonblank), size=lab_len[b])] if len(nonblank) else nonblank[:0]
        if len(nonblank) == 0:
            lab_len[b] = 0
        if feasible_only:
            while len(lab) + repeats(lab) > in_len[b]:
                lab = lab[:-1]
            lab_len[b] = len(lab)
        labs.append(lab)
    logits = _draw_logits(rng, T, B, A, sigma, 0.0, blank)
    flat = (np.concatenate(labs) if B else np.zeros(0)).astype(np.int32)
    return CTCBatch(name=f"random{seed}", T=T, B=B, A=A, blank=blank, logits=logits,
                    flat_labels=flat, label_lengths=lab_len.astype(np.int32),
                    input_lengths=in_len.astype(np.int32), seed=seed,
                    notes={"sigma": sigma, "blank_shift": 0.0})


def to_bf16_grid(x: np.ndarray) -> np.ndarray:
    """Round float32 to the nearest bfloat16 (ties to even); returned as float32."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    rounded = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return rounded.astype(np.uint32).view(np.float32).reshape(x.shape)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """The uint16 bit patterns of `to_bf16_grid(x)`."""
    return (to_bf16_grid(x).view(np.uint32) >> 16).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << 16).view(np.float32)
