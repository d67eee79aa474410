"""Automatic stage partitioning (paper Sec. 4.4): the oracle's algorithm against the brute-force definition, its
invariants, and the library's host function against the oracle (no GPU needed)."""
import time

import numpy as np
import pytest

from oracle import partition as OP

RNG = np.random.default_rng(31337)


def draw(L, heavy_last=True):
    tf = list(RNG.uniform(0.5, 1.5, L))
    tb = [f * RNG.uniform(2.5, 3.5) for f in tf]          # backward with recomputation is about three forwards (Sec. 3.3)
    if heavy_last:                                        # the LM head: an oversized last layer (Sec. 2.3)
        tf[-1] *= 3.0
        tb[-1] *= 3.0
    mf = list(RNG.uniform(1.0, 2.0, L))
    mb = [m * RNG.uniform(2.0, 4.0) for m in mf]
    return tf, tb, mf, mb


def test_algorithm_reaches_the_brute_force_optimum():
    for trial in range(40):
        L = int(RNG.integers(1, 8))
        tf, tb, mf, mb = draw(L, heavy_last=bool(trial & 1))
        mem = float(RNG.uniform(4.0, 30.0))
        n_gpus, n_micro = int(RNG.integers(1, 9)), int(RNG.integers(1, 33))
        want = OP.brute_force(tf, tb, mf, mb, mem, n_gpus, n_micro)
        got = OP.partition(tf, tb, mf, mb, mem, n_gpus, n_micro)
        if want is None:
            assert got is None
            continue
        fwd, bwd, t_max, cost = got
        assert cost == pytest.approx(want, rel=1e-12), (tf, tb, mem, n_gpus, n_micro)
        assert OP.evaluate(fwd, bwd, tf, tb, mf, mb, mem, n_gpus, n_micro) == pytest.approx(cost, rel=1e-12)


def test_partition_invariants_and_closed_forms():
    # uniform layers, no memory pressure, one GPU (no bubble term): cost = M * S * t_max is minimised by any exact
    # tiling; with backward = 3 x forward the total work is fixed: sum over stages >= (L - B1) f + L b
    L = 12
    tf, tb = [1.0] * L, [3.0] * L
    fwd, bwd, t_max, cost = OP.partition(tf, tb, [0.0] * L, [0.0] * L, 1.0, 1, 8)
    assert sum(bwd) == L and sum(fwd) + bwd[0] == L
    assert cost >= 8 * ((L - bwd[0]) * 1.0 + L * 3.0) - 1e-9       # stages x t_max covers all the work
    assert cost == pytest.approx(8 * ((L - bwd[0]) * 1.0 + L * 3.0))  # and here it is tight: perfectly balanced
    # many GPUs: the bubble term N (N-1) t_max favours short stages
    fwd2, bwd2, t2, _ = OP.partition(tf, tb, [0.0] * L, [0.0] * L, 1.0, 8, 8)
    assert t2 <= t_max
    # memory limit forces one layer per backward stage
    fwd3, bwd3, _, _ = OP.partition(tf, tb, [0.1] * L, [1.0] * L, 1.5, 2, 8)
    assert bwd3 == [1] * L
    # a layer that cannot fit at all
    assert OP.partition(tf, tb, [0.1] * L, [2.0] * L, 1.5, 2, 8) is None
    # the fused stage is as full as the winning bound allows: adding the next layer to it would exceed t_max or memory
    tf4, tb4, mf4, mb4 = draw(10)
    fwd4, bwd4, t4, _ = OP.partition(tf4, tb4, mf4, mb4, 1e9, 4, 16)
    if bwd4[0] < 10:
        assert sum(tb4[10 - bwd4[0] - 1:]) > t4


def test_library_partitioner_equals_oracle():
    from paper_2604_27085_amd import binding as B
    for trial in range(60):
        L = int(RNG.integers(1, 40))
        tf, tb, mf, mb = draw(L)
        mem = float(RNG.uniform(8.0, 60.0))
        n_gpus, n_micro = int(RNG.integers(1, 9)), int(RNG.integers(1, 65))
        want = OP.partition(tf, tb, mf, mb, mem, n_gpus, n_micro)
        if want is None:
            with pytest.raises(B.RpError) as e:
                B.rp_partition_stages(tf, tb, mf, mb, mem, n_gpus, n_micro)
            assert e.value.code == B.RP_EUNSUPPORTED
            continue
        fwd, bwd, t_max, cost = B.rp_partition_stages(tf, tb, mf, mb, mem, n_gpus, n_micro)
        assert (fwd, bwd) == (want[0], want[1]), (L, trial)
        assert t_max == want[2] and cost == want[3]          # same double arithmetic in the same order


def test_library_partitioner_is_fast_at_94_layers_and_rejects_bad_input():
    """The paper reports 1.47 s for its 94-layer model (Sec. 5.6); the O(L^3) loop in native code takes milliseconds."""
    from paper_2604_27085_amd import binding as B
    tf, tb, mf, mb = draw(95)
    t0 = time.perf_counter()
    fwd, bwd, t_max, cost = B.rp_partition_stages(tf, tb, mf, mb, 1e9, 8, 16)
    dt = time.perf_counter() - t0
    assert sum(bwd) == 95 and sum(fwd) + bwd[0] == 95
    assert dt < 0.5, dt
    with pytest.raises(B.RpError):
        B.rp_partition_stages([1.0, -1.0], [1.0, 1.0], [0.0, 0.0], [0.0, 0.0], 1.0, 2, 2)
    with pytest.raises(B.RpError):
        B.rp_partition_stages([1.0], [1.0], [0.0], [0.0], 1.0, 0, 2)
