"""CTC by its definition: enumerate every alignment.  TEST INFRASTRUCTURE.

Independent of the dynamic-programming oracle: it walks all A**T frame-level
strings, applies the CTC operator (merge runs of equal symbols, then delete
blanks; Section 3.3, Eq. (ctc) with the operator of Graves et al.), and adds up
probabilities.  Usable only for tiny T and A.
"""
from __future__ import annotations

import itertools
import math

import numpy as np


def collapse(path, blank):
    """The CTC operator: merge repeats, then remove blanks."""
    out = []
    prev = None
    for k in path:
        if k != prev and k != blank:
            out.append(k)
        prev = k
    return tuple(out)


def softmax_rows(x):
    x = np.asarray(x, dtype=np.float64)
    e = np.exp(x - x.max(axis=-1, keepdims=True))
    return e / e.sum(axis=-1, keepdims=True)


def all_labelings(x, blank):
    """{labeling: probability} over every labeling reachable in T frames; x is [T,A] logits."""
    y = softmax_rows(x)
    T, A = y.shape
    table = {}
    for path in itertools.product(range(A), repeat=T):
        mass = 1.0
        for t, k in enumerate(path):
            mass *= y[t, k]
        key = collapse(path, blank)
        table[key] = table.get(key, 0.0) + mass
    return table


def cost_and_grad(x, label, blank):
    """(-ln p, d(-ln p)/dx) for one utterance by enumeration; x is [T,A] logits."""
    y = softmax_rows(x)
    T, A = y.shape
    label = tuple(int(k) for k in label)
    p = 0.0
    through = np.zeros((T, A))
    for path in itertools.product(range(A), repeat=T):
        if collapse(path, blank) != label:
            continue
        mass = 1.0
        for t, k in enumerate(path):
            mass *= y[t, k]
        p += mass
        for t, k in enumerate(path):
            through[t, k] += mass
    if T == 0:
        p = 1.0 if len(label) == 0 else 0.0
    if p == 0.0:
        return math.inf, np.zeros((T, A))
    return -math.log(p), y - through / p


def count_alignments(T, label, A, blank):
    """Number of length-T strings over A symbols that collapse to `label` (exact integer)."""
    label = tuple(int(k) for k in label)
    return sum(1 for path in itertools.product(range(A), repeat=T) if collapse(path, blank) == label)


def best_alignments(x, label, blank):
    """(max probability, [every alignment that attains it]) by enumeration; x is [T,A] logits.

    Section 5.1 (alignment step): l* = argmax over Align(x, y) of prod_t y_t(l_t).
    Alignments are tuples of frame-level symbols.  (0.0, []) when none exists.
    """
    y = softmax_rows(x)
    T, A = y.shape
    label = tuple(int(k) for k in label)
    best, arg = 0.0, []
    for path in itertools.product(range(A), repeat=T):
        if collapse(path, blank) != label:
            continue
        mass = 1.0
        for t, k in enumerate(path):
            mass *= y[t, k]
        if mass > best:
            best, arg = mass, [path]
        elif mass == best and mass > 0.0:
            arg.append(path)
    return best, arg
