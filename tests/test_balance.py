"""Width balancer (Section 3.3.1, the balance formula and Algorithm 1): pins for the oracle, then the
C-ABI function against the oracle, bit-exact (the widths are integers)."""
import itertools
import math

import numpy as np
import pytest

from oracle import balance

BIG = 1e30


# ---- pins for the oracle ---------------------------------------------------------------------------

def test_three_to_one_capacity_gives_the_uneven_partition():
    # initial load ratios = DF_i / sum DF (Algorithm 1, initialisation): 3:1 -> 0.75 / 0.25
    assert balance.balance_widths(50_000, [3.0, 1.0], [BIG, BIG], 1.0, 1.0) == ([37_500, 12_500], True)
    w, ok = balance.balance_widths(100_000, [3, 1, 3, 1], [BIG] * 4, 1.0, 1.0)
    assert w == [37_500, 12_500, 37_500, 12_500] and ok


def test_equal_devices_get_equal_widths_and_remainders_go_to_low_indices():
    assert balance.balance_widths(12_500 * 8, [7.0] * 8, [BIG] * 8, 2.0, 3.0)[0] == [12_500] * 8
    assert balance.balance_widths(10, [1, 1, 1], [BIG] * 3, 1.0, 1.0)[0] == [4, 3, 3]
    assert balance.balance_widths(11, [1, 1, 1], [BIG] * 3, 1.0, 1.0)[0] == [4, 4, 3]
    assert balance.proportional_widths(7, [2, 1]) == [5, 2]          # 4.67, 2.33 -> floors 4, 2; extra to 0


def test_memory_cap_forces_a_shift_by_hand():
    # two devices 3:1, the fast one only holds half of the layer: (750, 250) -> (500, 500)
    w, ok = balance.balance_widths(1000, [3.0, 1.0], [0.5, 10.0], 1.0, 1.0)
    assert (w, ok) == ([500, 500], True)
    # three devices 2:1:1; device 0 fits 30 %.  All flop utilisations start equal, so the valley is
    # the device with the lowest memory utilisation: device 1 (0.25) before device 2 (0.5).
    w, ok = balance.balance_widths(1000, [2.0, 1.0, 1.0], [0.3, 1.0, 0.5], 5.0, 1.0)
    assert (w, ok) == ([300, 450, 250], True)


def test_failed_shift_drops_the_valley_and_infeasible_is_reported():
    # total memory 0.8 of the layer: no assignment fits.  Device 0 (500 columns, fits 200) is the peak;
    # device 1 takes its 50 spare columns, fails, is dropped; device 2 likewise; the loop ends.
    w, ok = balance.balance_widths(1000, [2.0, 1.0, 1.0], [0.2, 0.3, 0.3], 1.0, 1.0)
    assert (w, ok) == ([400, 300, 300], False)
    # with a roomy third device that one has the lowest memory utilisation (0.25 against 0.83), is the
    # first valley and absorbs all 300 excess columns
    w, ok = balance.balance_widths(1000, [2.0, 1.0, 1.0], [0.2, 0.3, 1.0], 1.0, 1.0)
    assert (w, ok) == ([200, 250, 550], True)


def test_peak_is_the_highest_memory_utilisation():
    # devices 0 and 1 both over memory; device 1 is worse (util 2.5 vs 1.25) and is served first by the
    # only valley, which then has room for just part of device 0's excess
    w, ok = balance.balance_widths(1000, [1.0, 1.0, 1.0, 1.0], [0.2, 0.1, 0.45, 0.25], 1.0, 1.0)
    # start (250, 250, 250, 250); utils 1.25, 2.5, 0.556, 1.0.  Valley = device 2 (0.556 < 1.0).
    # device 1 sheds 150 -> device 2 at 400 of 450; device 0 sheds 50 -> device 2 at 450.  Feasible.
    assert (w, ok) == ([200, 100, 450, 250], True)


def _feasible_exists(C, DM, TG_mem):
    return sum(balance.max_columns(C, TG_mem, d) for d in DM) >= C


def test_invariants_on_random_instances():
    r = np.random.Generator(np.random.PCG64(0))
    for _ in range(300):
        N = int(r.integers(1, 7))
        C = int(r.integers(1, 5000))
        DF = r.uniform(0.5, 8.0, N).tolist()
        TG_mem = float(r.uniform(1.0, 4.0))
        DM = (r.uniform(0.05, 1.2, N) * TG_mem).tolist()
        w, ok = balance.balance_widths(C, DF, DM, 3.0, TG_mem)
        assert sum(w) == C and min(w) >= 0
        fits = all(balance.mem_util(w[i], C, TG_mem, DM[i]) <= 1.0 for i in range(N))
        assert ok == fits
        # load only leaves over-memory devices and only enters devices with room, so the result is
        # feasible exactly when the devices' capacities add up to the layer
        assert ok == _feasible_exists(C, DM, TG_mem)
        if all(d >= TG_mem for d in DM):            # memory never binds: the proportional optimum
            assert w == balance.proportional_widths(C, DF)
            assert balance.objective(w, C, DF) <= N / C


def test_two_devices_reach_the_optimum_of_the_formula_by_brute_force():
    r = np.random.Generator(np.random.PCG64(1))
    for _ in range(60):
        C = int(r.integers(2, 40))
        DF = r.uniform(0.5, 4.0, 2).tolist()
        DM = r.uniform(0.2, 1.2, 2).tolist()
        w, ok = balance.balance_widths(C, DF, DM, 1.0, 1.0)
        cands = [(a, C - a) for a in range(C + 1)
                 if balance.mem_util(a, C, 1.0, DM[0]) <= 1.0 and balance.mem_util(C - a, C, 1.0, DM[1]) <= 1.0]
        assert ok == bool(cands)
        if cands:
            best = min(balance.objective(list(c), C, DF) for c in cands)
            assert balance.objective(w, C, DF) <= best + 1e-12


def _compositions(C, N):
    if N == 1:
        yield (C,)
        return
    for a in range(C + 1):
        for rest in _compositions(C - a, N - 1):
            yield (a,) + rest


def test_small_instances_against_enumeration_of_all_partitions():
    """Independent of the algorithm's steps: for up to four devices and a few dozen columns, list EVERY integer
    partition of the layer, keep those that satisfy the memory constraint of the formula in Section 3.3.1, and
    check the algorithm's result against that set: it reports feasibility exactly when the set is non-empty,
    its result lies in the set, and its value of the formula's objective is within rounding (one column per
    device, counted on both sides of a shift) of the best value in the set.  When nothing fits, no device is
    left over its memory while another still has room (load is conserved and only moves off over-memory
    devices)."""
    r = np.random.Generator(np.random.PCG64(7))
    n_feasible = n_shifted = 0
    for _ in range(150):
        N = int(r.integers(2, 5))
        C = int(r.integers(N, 25))
        DF = r.uniform(0.5, 6.0, N).tolist()
        TG_mem = float(r.uniform(1.0, 3.0))
        DM = (r.uniform(0.1, 0.9, N) * TG_mem).tolist()
        w, ok = balance.balance_widths(C, DF, DM, 2.0, TG_mem)
        assert sum(w) == C and min(w) >= 0
        fits = lambda part: all(part[i] / C * TG_mem <= DM[i] for i in range(N))
        total = sum(DF)
        value = lambda part: sum(abs(part[i] / C - DF[i] / total) for i in range(N))
        feasible = [part for part in _compositions(C, N) if fits(part)]
        assert ok == bool(feasible)
        if feasible:
            n_feasible += 1
            assert tuple(w) in set(feasible)
            best = min(value(part) for part in feasible)
            assert value(w) <= best + 2.0 * N / C + 1e-12, (C, DF, DM, w, best)
            n_shifted += w != balance.proportional_widths(C, DF)
        else:
            over = [i for i in range(N) if w[i] / C * TG_mem > DM[i]]
            room = [i for i in range(N) if (w[i] + 1) / C * TG_mem <= DM[i]]
            assert over and not room, (C, DF, DM, w)
    assert n_feasible > 20 and n_shifted > 10        # the memory constraint was binding in many of them


def test_ties_go_to_the_lower_device_index():
    # two identical valleys: device 1 takes the whole excess of device 0 (it can), device 2 stays
    w, ok = balance.balance_widths(900, [1.0, 1.0, 1.0], [0.2, 1.0, 1.0], 1.0, 1.0)
    assert (w, ok) == ([180, 420, 300], True)
    # two identical over-memory devices: device 0 is served first and gets the roomier valley
    w, ok = balance.balance_widths(800, [1.0, 1.0, 1.0, 1.0], [0.125, 0.125, 0.375, 0.5], 1.0, 1.0)
    assert ok and w[0] == 100 and w[1] == 100 and sum(w) == 800


# ---- the library against the oracle ------------------------------------------------------------------

@pytest.fixture(scope="module")
def ws():
    from paper_2011_09208_amd import buildlib
    if buildlib.is_stale():
        buildlib.build()
    from paper_2011_09208_amd import binding
    return binding


def test_library_matches_oracle_bit_exact(ws):
    r = np.random.Generator(np.random.PCG64(2))
    cases = [(100_000, [3, 1, 3, 1], [BIG] * 4, 1.0, 1.0), (1000, [2.0, 1.0, 1.0], [0.2, 0.3, 0.3], 1.0, 1.0),
             (1, [1.0], [1.0], 1.0, 1.0), (10, [1, 1, 1], [BIG] * 3, 1.0, 1.0)]
    for _ in range(500):
        N = int(r.integers(1, 9))
        C = int(r.integers(1, 200_000))
        TG_mem = float(r.uniform(0.5, 64.0))
        cases.append((C, r.uniform(0.5, 20.0, N).tolist(), (r.uniform(0.03, 1.0, N) * TG_mem).tolist(),
                      float(r.uniform(1.0, 1e3)), TG_mem))
    n_infeasible = 0
    for C, DF, DM, TG_flop, TG_mem in cases:
        got = ws.balance_widths(C, DF, DM, TG_flop, TG_mem)
        ref = balance.balance_widths(C, list(map(float, DF)), list(map(float, DM)), TG_flop, TG_mem)
        assert got == ref, (C, DF, DM)
        n_infeasible += not ref[1]
    assert 0 < n_infeasible < len(cases)          # both outcomes are exercised


def test_library_rejects_bad_arguments(ws):
    import ctypes
    f = ws.lib.ws_balance_widths
    d2 = (ctypes.c_double * 2)(1.0, 1.0)
    w2 = (ctypes.c_int32 * 2)()
    ok = ctypes.c_int32()
    assert f(2, None, d2, 1.0, 1.0, 10, w2, ctypes.byref(ok)) == 1
    assert f(2, d2, d2, 1.0, 1.0, 10, None, ctypes.byref(ok)) == 1
    assert f(0, d2, d2, 1.0, 1.0, 10, w2, ctypes.byref(ok)) == 2
    assert f(2, d2, d2, 1.0, 1.0, 0, w2, ctypes.byref(ok)) == 2
    assert f(2, d2, d2, 0.0, 1.0, 10, w2, ctypes.byref(ok)) == 4
    assert f(2, d2, d2, 1.0, float("nan"), 10, w2, ctypes.byref(ok)) == 4
    bad = (ctypes.c_double * 2)(1.0, -1.0)
    assert f(2, bad, d2, 1.0, 1.0, 10, w2, ctypes.byref(ok)) == 4
    assert f(2, d2, bad, 1.0, 1.0, 10, w2, ctypes.byref(ok)) == 4
