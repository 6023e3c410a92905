"""The wavefront plan of the lattice kernels, checked on the CPU for every label length.

plan_waves (paper_1512_02595_amd/csrc/ctc_internal.h) is plain C++ shared by the host launcher and the
device-side planner; here it is compiled into a small host program and its invariants are checked:
the kernels index lanes and LDS by them, so a plan outside them would read or write out of bounds.
"""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

PROGRAM = r"""
#include <cstdio>
#include "ctc_internal.h"
int main()
{
    for (int crowded = 0; crowded < 2; ++crowded)
        for (int L = 0; L <= CTC_MAX_LABEL_LENGTH; ++L) {
            const ctc::WavePlan p = ctc::plan_waves(L, crowded != 0);
            std::printf("%d %d %d %d %d\n", crowded, L, p.waves, p.halo, p.barrier ? 1 : 0);
            const ctc::WavePlan p2 = ctc::plan_waves2(L, crowded != 0);
            std::printf("two %d %d %d %d %d %d\n", crowded, L, p2.waves, p2.halo, p2.barrier ? 1 : 0,
                        ctc::two_pairs_per_lane(L, crowded != 0) ? 1 : 0);
            std::printf("sym %d %d %d\n", crowded, L, ctc::two_pairs_per_lane(L, crowded != 0, true) ? 1 : 0);
        }
    std::printf("chunk %d slack %d %d\n", ctc::kChunk, ctc::kBlankSlack, ctc::kLabelSlack);
    return 0;
}
"""


@pytest.fixture(scope="module")
def plans(tmp_path_factory):
    d = tmp_path_factory.mktemp("plan")
    src, exe = d / "plan.cpp", d / "plan"
    src.write_text(PROGRAM)
    subprocess.run(["g++", "-std=c++17", "-O1", "-I", os.path.join(ROOT, "include"),
                    "-I", os.path.join(ROOT, "paper_1512_02595_amd", "csrc"), str(src), "-o", str(exe)], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.splitlines()
    rows = [tuple(int(v) for v in line.split()) for line in out if line[0].isdigit()]
    rows2 = [tuple(int(v) for v in line.split()[1:]) for line in out if line.startswith("two")]
    consts = [line for line in out if line.startswith("chunk")][0].split()
    sym = {tuple(int(v) for v in line.split()[1:3]): int(line.split()[3]) for line in out if line.startswith("sym")}
    return rows, {"symbol_major": sym, "chunk": int(consts[1]), "blank_slack": int(consts[3]), "label_slack": int(consts[4]),
                  "two_pairs": rows2}


def test_every_label_length_has_a_plan_the_kernels_can_run(plans):
    rows, c = plans
    assert len(rows) == 2 * 1024
    for crowded, L, waves, halo, barrier in rows:
        pairs = L + 1
        assert 1 <= waves <= 16, (L, waves)
        if barrier:
            # 64 pairs per wavefront, one barrier per step: every pair needs a lane
            assert halo == 0 and waves * 64 >= pairs, (L, waves)
            continue
        if waves == 1:
            assert halo == 0 and pairs <= 64, (L, waves, halo)
            continue
        # halo exchange: hand-overs fall on chunk boundaries, the lanes handed up are exact lanes,
        # the exchange buffer holds two halves of 32 entries, and every pair has an exact lane
        assert halo % c["chunk"] == 0 and c["chunk"] <= halo <= 32, (L, waves, halo)
        assert halo <= 64 - halo
        assert waves * (64 - halo) + halo >= pairs, (L, waves, halo)
        # and no wavefront is idle: one fewer would not hold the pairs with this halo
        assert (waves - 1) * (64 - halo) + halo < pairs or waves == 2, (L, waves, halo)


def test_every_label_length_has_a_two_pairs_per_lane_plan(plans):
    """plan_waves2: lanes own two neighbouring pairs; a halo of h lanes lasts 2h steps."""
    _, c = plans
    rows = c["two_pairs"]
    assert len(rows) == 2 * 1024
    for crowded, L, waves, halo, barrier, chosen in rows:
        lanes = (L + 2) // 2                        # ceil((L + 1) / 2) lanes hold the L + 1 pairs
        assert not barrier and 1 <= waves <= 16, (L, waves)
        if waves == 1:
            assert halo == 0 and lanes <= 64, (L, halo)
            continue
        # hand-overs every 2 * halo steps fall on chunk boundaries; the exchange buffer holds 16 lanes
        assert (2 * halo) % c["chunk"] == 0 and 4 <= halo <= 16, (L, waves, halo)
        assert waves * (64 - halo) + halo >= lanes, (L, waves, halo)


def test_choice_between_one_and_two_pairs_per_lane(plans):
    """Two pairs per lane only for labels of more than 64 pairs; always when the one-pair plan would put
    several wavefronts on a SIMD or has no halo left, and always in crowded launches."""
    rows, c = plans
    one = {(crowded, L): (waves, barrier) for crowded, L, waves, halo, barrier in rows}
    for crowded, L, waves2, halo2, _, chosen in c["two_pairs"]:
        waves1, barrier1 = one[(crowded, L)]
        if L + 1 <= 64:
            assert not chosen, L
        else:
            assert bool(chosen) == bool(crowded or barrier1 or waves1 > 4), (crowded, L, waves1, chosen)
        if chosen:
            assert waves2 <= waves1, (crowded, L, waves1, waves2)
    # symbol-major emission block: also where the one-pair plan would hand over every chunk
    halo1 = {(crowded, L): halo for crowded, L, waves, halo, barrier in rows}
    for crowded, L, waves2, halo2, _, chosen in c["two_pairs"]:
        expect = bool(chosen) or (L + 1 > 64 and halo1[(crowded, L)] < 2 * c["chunk"])
        assert bool(c["symbol_major"][(crowded, L)]) == expect, (crowded, L)
    assert not c["symbol_major"][(0, 207)] and c["symbol_major"][(0, 208)] and c["symbol_major"][(0, 231)]


def test_plans_only_switch_to_the_barrier_kernel_when_no_halo_fits(plans):
    rows, _ = plans
    for crowded, L, waves, halo, barrier in rows:
        if barrier:
            assert 16 * 56 + 8 < L + 1, L


def test_emission_margins_cover_the_prefetch(plans):
    """The lattice kernel requests emissions up to 3 * chunk - 1 rows past an utterance's block."""
    _, c = plans
    assert c["label_slack"] >= (3 * c["chunk"] - 1) * 1024
    assert c["blank_slack"] >= 3 * c["chunk"] - 1 + c["chunk"] - 1


def test_the_two_pair_plan_is_the_cheapest_over_all_wavefront_counts(plans):
    """plan_waves2 only looks at four wavefront counts from the smallest feasible one (the planners run on the
    GPU per utterance); here its choice is compared with a search over all counts 2 .. 16 with the same cost
    model (restated: clocks per step and per hand-over as the header gives them)."""
    _, c = plans
    for crowded, L, waves, halo, barrier, _two in c["two_pairs"]:
        lanes = (L + 2) // 2
        if lanes <= 64:
            assert (waves, halo) == (1, 0)
            continue
        best, best_cost = None, float("inf")
        for w in range(2, 17):
            h = min((64 * w - lanes) // (w - 1), 16)
            h -= h % 4
            if h < 4:
                continue
            per_simd = (w + 3) // 4
            cost = w * (110.0 + 300.0 / h) if crowded else (150.0 if per_simd == 1 else per_simd * 110.0) + 300.0 / h + 4.0 * w
            if cost < best_cost - 1e-9:
                best, best_cost = (w, h), cost
        assert (waves, halo) == best, (crowded, L, (waves, halo), best)
