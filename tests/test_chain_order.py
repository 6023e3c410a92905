"""The order in which the lattice launch takes its chains, checked on the CPU.

order_chains (paper_1512_02595_amd/csrc/ctc_internal.h) is host code; here it is compiled into a small
program and run on length mixes like those of the five configurations.  Whatever the dispatcher does with
the order, every chain must be launched exactly once; and under the placement model that the order is
built for (workgroup i on compute unit i mod n_cu, each further workgroup of a compute unit starting one
SIMD later) the busiest SIMD must carry no more than with the plain heaviest-first order.
"""
import os
import subprocess

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

PROGRAM = r"""
#include <cstdio>
#include <vector>
#include "ctc_internal.h"
int main()
{
    int n, dirs, n_cu;
    while (std::scanf("%d %d %d", &n, &dirs, &n_cu) == 3) {
        std::vector<int32_t> utt(n), frames(n), waves(n), order(static_cast<size_t>(n) * dirs + 1, -7);
        for (int i = 0; i < n; ++i)
            if (std::scanf("%d %d %d", &utt[i], &frames[i], &waves[i]) != 3) return 1;
        ctc::order_chains(utt.data(), frames.data(), waves.data(), n, dirs, n_cu, order.data());
        for (int i = 0; i <= n * dirs; ++i) std::printf("%d ", order[i]);
        std::printf("\n");
    }
    return 0;
}
"""


@pytest.fixture(scope="module")
def program(tmp_path_factory):
    d = tmp_path_factory.mktemp("order")
    src, exe = d / "order.cpp", d / "order"
    src.write_text(PROGRAM)
    subprocess.run(["g++", "-std=c++17", "-O1", "-I", os.path.join(ROOT, "include"),
                    "-I", os.path.join(ROOT, "paper_1512_02595_amd", "csrc"), str(src), "-o", str(exe)], check=True)
    return str(exe)


def run_order(exe, utt, frames, waves, dirs, n_cu):
    n = len(utt)
    text = "%d %d %d\n" % (n, dirs, n_cu) + "".join("%d %d %d\n" % t for t in zip(utt, frames, waves))
    out = subprocess.run([exe], input=text, check=True, capture_output=True, text=True).stdout.split()
    order = [int(v) for v in out]
    assert order[-1] == -7, "order_chains wrote past its n * dirs entries"
    return order[:-1]


def mix(seed, n, t_lo, t_hi, two_wave_from=127):
    """Utterances as the launcher passes them: heaviest (frames x wavefronts) first."""
    rng = np.random.default_rng(seed)
    frames = rng.integers(t_lo, t_hi + 1, n)
    labels = (frames * rng.uniform(0.15, 0.3, n)).astype(int)
    waves = np.where(labels >= two_wave_from, 2, 1)
    utt = rng.permutation(n)
    rank = np.argsort(-(frames * waves), kind="stable")
    return utt[rank].tolist(), frames[rank].tolist(), waves[rank].tolist()


def busiest_simd(order, frames_of, waves_of, n_cu):
    """Frames on the busiest SIMD under the placement model the order is built for."""
    load = np.zeros((n_cu, 4), dtype=np.int64)
    for i, entry in enumerate(order):
        c, s = i % n_cu, (i // n_cu) % 4
        for w in range(waves_of[entry >> 1]):
            load[c, (s + w) % 4] += frames_of[entry >> 1]
    return int(load.max())


@pytest.mark.parametrize("n,dirs,n_cu", [(1, 2, 256), (5, 1, 256), (64, 2, 256), (128, 2, 256), (129, 2, 256),
                                         (300, 1, 256), (512, 2, 256), (700, 2, 256), (2000, 2, 256),
                                         (37, 2, 4), (512, 2, 1)])
def test_every_chain_is_launched_exactly_once(program, n, dirs, n_cu):
    utt, frames, waves = mix(n, n, 100, 750)
    order = run_order(program, utt, frames, waves, dirs, n_cu)
    assert sorted(order) == sorted(u * 2 + d for u in utt for d in range(dirs))


def test_small_launches_keep_the_heaviest_first_in_blocks_per_direction(program):
    utt, frames, waves = mix(3, 40, 100, 750)
    order = run_order(program, utt, frames, waves, 2, 256)
    expect = []
    for i0 in range(0, 40, 16):
        for d in range(2):
            expect += [u * 2 + d for u in utt[i0:i0 + 16]]
    assert order == expect
    # the two chains of an utterance are a multiple of eight workgroups apart: same die
    where = {e: i for i, e in enumerate(order)}
    assert all((where[u * 2] - where[u * 2 + 1]) % 8 == 0 for u in utt)


@pytest.mark.parametrize("seed,n", [(0, 512), (1, 512), (2, 400), (3, 1000), (4, 2048)])
def test_busiest_simd_is_no_busier_than_with_the_plain_order(program, seed, n):
    utt, frames, waves = mix(seed, n, 100, 750)
    frames_of = dict(zip(utt, frames))
    waves_of = dict(zip(utt, waves))
    order = run_order(program, utt, frames, waves, 2, 256)
    plain = [u * 2 + d for d in range(2) for u in utt]          # all forward chains, then all backward ones
    ours, theirs = busiest_simd(order, frames_of, waves_of, 256), busiest_simd(plain, frames_of, waves_of, 256)
    assert ours <= theirs
    # no SIMD can carry less than the longest chain or the average
    total = sum(2 * f * w for f, w in zip(frames, waves))
    assert ours >= max(max(frames), total // (256 * 4))
    print("  n=%d: busiest SIMD %d frames (plain order %d, lower bound %d)"
          % (n, ours, theirs, max(max(frames), -(-total // 1024))))
