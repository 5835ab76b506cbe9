"""Analytical model and greedy parameter search (section 6 of the paper).

CPU only.  First the oracle (`oracle/tuner.py`) is pinned to what the text fixes -- the printed
equations evaluated by hand, a trial sequence worked out by hand for a small latency table,
brute force over the whole grid on separable unimodal latencies, the "about ten trials" the
evaluation reports -- then the library's propose / report state machine must make exactly the
oracle's trials, in the oracle's order, on seeded random latency tables.
"""
import itertools

import numpy as np
import pytest

from oracle import tuner as otuner
from paper_2209_06800_amd import binding

POW2 = {32: [1, 2, 4, 8, 16, 32], 16: [1, 2, 4, 8, 16]}


# ------------------------------------------------------------------------------ oracle pins
def test_model_equations_by_hand():
    # section 6, equations (1)-(3), with ps 16, dist 4, wpb 8, D 64, IntS = FloatS = 4:
    #   WPW  = 2 * 16 * 64 * 4            = 8192
    #   SMEM = 16 * 8 * 4 + 2 * 8 * 64 * 4 = 512 + 4096 = 4608
    #   numWarps = max(1000, 2500) / 4 = 625; numBlocks = ceil(625 / 8) = 79; per unit 79 / 108
    m = otuner.model(1000, 2500, 16, 4, 8, 64, 108, 164 * 1024)
    assert m["wpw"] == 8192 and m["smem"] == 4608
    assert m["num_warps"] == 625 and m["num_blocks"] == 79
    assert m["blocks_per_unit"] == pytest.approx(79 / 108)
    assert m["feasible"]
    # the shared-memory constraint binds for wide rows and large blocks:
    #   ps 32, wpb 16, D 4096: 32*16*4 + 2*16*4096*4 = 2048 + 524288 > 164 KB
    assert not otuner.model(10, 10, 32, 1, 16, 4096, 108, 164 * 1024)["feasible"]


def test_search_order_worked_by_hand():
    # latency table (anything not listed is 100): the search must make exactly these trials.
    lat = {(1, 1, 1): 50, (2, 1, 1): 40, (4, 1, 1): 45,            # ps stops at 2
           (2, 2, 1): 30, (2, 4, 1): 35,                           # dist stops at 2
           (2, 2, 2): 25, (2, 2, 4): 26,                           # wpb stops at 2
           (1, 2, 1): 27, (1, 2, 2): 24, (1, 2, 4): 90}            # retreat: ps 2 -> 1, wpb from 1
    best, table = otuner.search(lambda k: lat.get(k, 100))
    assert [k for k, _ in table] == [(1, 1, 1), (2, 1, 1), (4, 1, 1), (2, 2, 1), (2, 4, 1), (2, 2, 2), (2, 2, 4),
                                     (1, 2, 1), (1, 2, 2), (1, 2, 4)]
    assert best == (1, 2, 2)
    assert len(table) == 10                                        # "about 10 iterations" (section 8.2)


def test_retreat_stops_at_the_third_lowest_latency():
    # upward sweeps: ps stops at 4, dist and wpb stay at 1; the three lowest latencies are then
    # 10, 20, 30.  Retreat to ps = 2: (2,1,1) is already in the table (20, within the three
    # lowest), its first wpb increase costs 31 > 30, which ends the whole search.
    lat = {(1, 1, 1): 30, (2, 1, 1): 20, (4, 1, 1): 10, (8, 1, 1): 50, (4, 2, 1): 60, (4, 1, 2): 70, (2, 1, 2): 31}
    best, table = otuner.search(lambda k: lat.get(k, 100))
    assert [k for k, _ in table] == [(1, 1, 1), (2, 1, 1), (4, 1, 1), (8, 1, 1), (4, 2, 1), (4, 1, 2), (2, 1, 2)]
    assert best == (4, 1, 1)
    # a retreat trial within the three lowest keeps the search alive: wpb goes on to 4 (stop)
    lat[(2, 1, 2)] = 15
    best, table = otuner.search(lambda k: lat.get(k, 100))
    assert [k for k, _ in table][-2:] == [(2, 1, 2), (2, 1, 4)] and best == (4, 1, 1)
    # ... and a retreat can win: the lowest latency of the lookup table is what is applied
    lat[(2, 1, 2)] = 5
    best, _ = otuner.search(lambda k: lat.get(k, 100))
    assert best == (2, 1, 2)


def test_separable_unimodal_latency_reaches_the_grid_minimum():
    # coordinate-wise search is exact when latency = f(ps) + g(dist) + h(wpb) with unimodal terms:
    # compare with brute force over the whole 6 x 5 x 5 grid
    rng = np.random.default_rng(7)
    for _ in range(50):
        opt = [rng.choice(POW2[32]), rng.choice(POW2[16]), rng.choice(POW2[16])]
        scale = rng.uniform(0.5, 2.0, size=3)

        def latency(k, opt=opt, scale=scale):
            return 1.0 + sum(s * abs(np.log2(v) - np.log2(o)) for s, v, o in zip(scale, k, opt))

        best, table = otuner.search(latency)
        brute = min(itertools.product(POW2[32], POW2[16], POW2[16]), key=latency)
        assert best == brute == tuple(opt)
        assert len(table) <= 6 + 5 + 5 + 6 * 5                     # never the whole grid of 150
        assert len({k for k, _ in table}) == len(table)            # no configuration measured twice


def test_search_respects_the_ranges():
    best, table = otuner.search(lambda k: 1.0 / (k[0] * k[1] * k[2]))    # always better when larger
    assert best == (32, 16, 16)
    assert all(1 <= ps <= 32 and 1 <= d <= 16 and 1 <= w <= 16 for (ps, d, w), _ in table)
    best, _ = otuner.search(lambda k: float(k[0] * k[1] * k[2]))         # always worse when larger
    assert best == (1, 1, 1)


def test_search_inside_the_models_constraint_worked_by_hand():
    # D = 64 and a shared-memory limit of 1200 bytes: SMEM = 4 ps wpb + 512 wpb allows wpb 1 for every ps,
    # wpb 2 up to ps 22, and never wpb 4.  Latency 1 + |log2 ps - 4| + 0.5 |log2 dist - 1| + 0.25 |log2 wpb - 3|
    # (lowest at ps 16, dist 2, wpb 8, which the constraint excludes).  By hand:
    #   ps:    (1,1,1) 6.25, (2,1,1) 5.25, (4,1,1) 4.25, (8,1,1) 3.25, (16,1,1) 2.25, (32,1,1) 3.25 -> ps 16
    #   dist:  (16,2,1) 1.75, (16,4,1) 2.25                                                        -> dist 2
    #   wpb:   (16,2,2) 1.5 [SMEM 1152], (16,2,4) infeasible [SMEM 2304]: not measured             -> wpb 2
    #   retreat: (8,2,1) 2.75 > third lowest (2.25): the search ends
    def latency(k):
        return 1 + abs(np.log2(k[0]) - 4) + 0.5 * abs(np.log2(k[1]) - 1) + 0.25 * abs(np.log2(k[2]) - 3)

    feasible = lambda k: otuner.model(1, 1, k[0], k[1], k[2], 64, 256, 1200)["feasible"]
    best, table = otuner.search(latency, feasible=feasible)
    assert [k for k, _ in table] == [(1, 1, 1), (2, 1, 1), (4, 1, 1), (8, 1, 1), (16, 1, 1), (32, 1, 1), (16, 2, 1), (16, 4, 1),
                                     (16, 2, 2), (8, 2, 1)]
    assert [v for _, v in table] == [6.25, 5.25, 4.25, 3.25, 2.25, 3.25, 1.75, 2.25, 1.5, 2.75]
    assert best == (16, 2, 2)
    # without the constraint the wpb sweep goes on to 8
    assert otuner.search(latency)[0] == (16, 2, 8)
    # nothing feasible at all: no trial is made
    assert otuner.search(latency, feasible=lambda k: False) == (None, [])


# ------------------------------------------------------------------------------ library vs oracle
def _drive(latency, limits=(32, 16, 16), constraint=None):
    t = binding.Tuner(*limits)
    if constraint is not None:
        t.set_constraint(*constraint)
    while True:
        k = t.next()
        if k is None:
            break
        assert t.next() == k                                       # asking twice proposes the same trial
        t.report(latency(k))
    table = t.table()
    if not table:                                                  # not even the starting point was feasible
        with pytest.raises(binding.MggError):
            t.result()
        t.destroy()
        return None, table
    best, best_lat, n = t.result()
    t.destroy()
    assert n == len(table) and best_lat == min(v for _, v in table)
    return best, table


def test_library_model_matches_oracle():
    rng = np.random.default_rng(11)
    for _ in range(200):
        nl, nr = int(rng.integers(0, 10**7)), int(rng.integers(0, 10**7))
        ps, dist, wpb = (int(rng.choice(POW2[32])), int(rng.choice(POW2[16])), int(rng.choice(POW2[16])))
        dim = int(rng.integers(1, 5000))
        units, limit = int(rng.choice([108, 256])), int(rng.choice([64, 160, 164])) * 1024
        assert binding.mgg_model_evaluate(nl, nr, ps, dist, wpb, dim, units, limit) == \
            otuner.model(nl, nr, ps, dist, wpb, dim, units, limit)
    assert binding.mgg_model_evaluate(1000, 2500, 16, 4, 8, 64, 108, 164 * 1024)["smem"] == 4608


@pytest.mark.parametrize("seed", range(40))
def test_library_search_makes_the_oracles_trials(seed):
    rng = np.random.default_rng(1000 + seed)
    grid = list(itertools.product(POW2[32], POW2[16], POW2[16]))
    if seed % 2:
        lat = {k: float(rng.uniform(1, 2)) for k in grid}                      # rough landscape
    else:                                                                      # bowl plus noise
        opt = np.log2([rng.choice(POW2[32]), rng.choice(POW2[16]), rng.choice(POW2[16])])
        lat = {k: float(1 + np.abs(np.log2(k) - opt).sum() + rng.uniform(0, 0.3)) for k in grid}
    want_best, want_table = otuner.search(lambda k: lat[k])
    best, table = _drive(lambda k: lat[k])
    assert table == want_table
    assert best == want_best


@pytest.mark.parametrize("seed", range(30))
def test_library_search_inside_the_models_constraint(seed):
    """With mgg_tuner_set_constraint the library skips what the model calls infeasible, exactly as the oracle does."""
    rng = np.random.default_rng(5000 + seed)
    grid = list(itertools.product(POW2[32], POW2[16], POW2[16]))
    opt = np.log2([rng.choice(POW2[32]), rng.choice(POW2[16]), rng.choice(POW2[16])])
    lat = {k: float(1 + np.abs(np.log2(k) - opt).sum() + rng.uniform(0, 0.3)) for k in grid}
    dim = int(rng.choice([16, 64, 602, 4096]))
    limit = int(rng.choice([8 * dim - 1, 8 * dim + 4, 20 * dim, 70 * dim, 160 * 1024]))
    feasible = lambda k: otuner.model(1, 1, k[0], k[1], k[2], dim, 256, limit)["feasible"]
    want_best, want_table = otuner.search(lambda k: lat[k], feasible=feasible)
    best, table = _drive(lambda k: lat[k], constraint=(dim, limit))
    assert table == want_table and best == want_best
    assert all(feasible(k) for k, _ in table)


def test_constraint_has_to_come_before_the_first_trial():
    t = binding.Tuner()
    t.set_constraint(64, 1200)
    t.next()
    t.report(1.0)
    with pytest.raises(binding.MggError):
        t.set_constraint(64, 4000)
    t.destroy()


def test_library_search_with_ties_and_small_ranges():
    for limits in ((1, 1, 1), (2, 1, 4), (32, 16, 16), (64, 1024, 16)):
        for const in (1.0,):
            want_best, want_table = otuner.search(lambda k: const, *limits)
            best, table = _drive(lambda k: const, limits)
            assert (best, table) == (want_best, want_table)


def test_tuner_argument_errors():
    lib = binding.lib()
    import ctypes
    h = ctypes.c_void_p()
    assert lib.mgg_tuner_create(0, 16, 16, ctypes.byref(h)) == binding.ERR_INVALID_ARG
    assert lib.mgg_tuner_create(32, 16, 17, ctypes.byref(h)) == binding.ERR_INVALID_ARG
    assert lib.mgg_tuner_create(32, 16, 16, None) == binding.ERR_INVALID_ARG
    t = binding.Tuner()
    with pytest.raises(binding.MggError):
        t.report(1.0)                                              # nothing proposed yet
    with pytest.raises(binding.MggError):
        t.result()                                                 # nothing measured yet
    t.next()
    with pytest.raises(binding.MggError):
        t.report(float("nan"))
    t.report(3.0)
    assert t.result() == ((1, 1, 1), 3.0, 1)
    lib.mgg_tuner_destroy(None)
    assert lib.mgg_model_evaluate(1, 1, binding.Knobs(0, 1, 1), 4, 256, 1, None) == binding.ERR_INVALID_ARG
