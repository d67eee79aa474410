"""Transfer schedule of a round (paper Sec. 4.2, "Scheduling parameter transfers"): pins of the oracle, and the
library's host-side planner against the oracle (no GPU needed: rp_plan_transfers is a pure host function)."""
import numpy as np
import pytest

from oracle import transfers as OT

RNG = np.random.default_rng(4242)


def test_lpt_on_the_classic_tight_instance():
    """Graham's worst case for three machines: jobs 5,5,4,4,3,3,3 -- LPT ends at 11, the optimum is 9 = 11 / (4/3 - 1/9)."""
    sizes = [5 * 256, 5 * 256, 4 * 256, 4 * 256, 3 * 256, 3 * 256, 3 * 256]
    plan = OT.lpt(sizes, 3, 1 << 30)
    assert OT.makespan(plan, 3) == 11 * 256
    assert OT.optimal_makespan(sizes, 3) == 9 * 256
    # descending sizes, each to the least loaded window, ties to the lower window
    assert [w for _, w, _, _ in plan] == [0, 1, 2, 2, 0, 1, 0]


def test_lpt_within_grahams_bound_of_the_brute_force_optimum():
    for trial in range(60):
        m = int(RNG.integers(1, 4))
        n = int(RNG.integers(1, 9))
        sizes = [int(RNG.integers(1, 40)) * 256 for _ in range(n)]
        plan = OT.lpt(sizes, m, 1 << 30)
        opt = OT.optimal_makespan(sizes, m)
        assert opt <= OT.makespan(plan, m) <= (4.0 / 3.0 - 1.0 / (3.0 * m)) * opt + 1e-9, (sizes, m)


def test_split_covers_every_byte_once_and_respects_the_piece_limit():
    sizes = [0, 100, 256, 70000, 1 << 20, (1 << 20) + 2, 3 * (1 << 20) + 4096]
    max_piece = 1 << 18
    plan = OT.lpt(sizes, 4, max_piece)
    for i, b in enumerate(sizes):
        mine = sorted((off, nb) for it, _, off, nb in plan if it == i)
        pos = 0
        for off, nb in mine:
            assert off == pos and 0 < nb <= max_piece
            assert off % 256 == 0
            pos += nb
        assert pos == b
    # one large tensor no longer dominates a window: loads differ by at most one piece
    load = [0] * 4
    for _, w, _, nb in plan:
        load[w] += nb
    assert max(load) - min(load) <= max_piece
    assert sum(load) == sum(sizes)


def test_single_window_and_empty_input():
    assert OT.lpt([], 3, 256) == []
    plan = OT.lpt([512, 256], 1, 256)
    assert [p[1] for p in plan] == [0, 0, 0] and sum(p[3] for p in plan) == 768


def test_library_planner_equals_oracle():
    from paper_2604_27085_amd import binding as B
    for trial in range(40):
        m = int(RNG.integers(1, 9))
        n = int(RNG.integers(0, 30))
        sizes = [int(RNG.integers(0, 5000)) * 16 for _ in range(n)]
        max_piece = int(RNG.integers(1, 64)) * 256
        assert B.rp_plan_transfers(sizes, m, max_piece) == OT.lpt(sizes, m, max_piece), (sizes, m, max_piece)
    # a stage's real tensor sizes: Qwen3-1.7B-shaped layer, 64 MiB pieces, 4 windows
    sizes = [2048 * 2, 4096 * 2048 * 2, 128 * 2, 128 * 2, 2048 * 2048 * 2, 2048 * 2, 12288 * 2048 * 2, 2048 * 6144 * 2,
             2048 * 2, 151936 * 2048 * 2]
    assert B.rp_plan_transfers(sizes, 4, 64 << 20) == OT.lpt(sizes, 4, 64 << 20)


def test_library_planner_rejects_bad_arguments():
    from paper_2604_27085_amd import binding as B
    with pytest.raises(B.RpError):
        B.rp_plan_transfers([256], 0, 256)
    with pytest.raises(B.RpError):
        B.rp_plan_transfers([256], 2, 100)
