"""Scheduler arithmetic (Sec. 3.4, Algorithm 1, Eq. 1-3) and graph choice (Sec. 3.2.2): the oracle
against cases worked by hand from the paper's text, then the library against the oracle."""
import math
import random
from fractions import Fraction

import pytest

import paper_2503_20552_amd as adr
from oracle import sched_oracle as O


# ---- the oracle, pinned by hand-worked cases ---------------------------------------------------

def test_bounds_worked_examples():
    # two prefill instances lending 20 and 30 GB at 400 and 500 GB/s to a decode instance with 80 GB, 1500 GB/s:
    # capacity ratio 50/80 = 0.625, bandwidth ratio 900/1500 = 0.6 -> Eq. 1 gives 0.6
    assert O.offload_bound_mem([20, 30], [400, 500], 80, 1500) == Fraction(3, 5)
    # more bandwidth than capacity: the capacity ratio binds
    assert O.offload_bound_mem([20, 30], [800, 1000], 80, 1500) == Fraction(5, 8)
    # Eq. 2: memory-bound up to batch 120, TPOT allows 80 without offloading -> (120-80)/80 = 0.5
    assert O.offload_bound_comp(120, 80) == Fraction(1, 2)
    assert O.offload_bound_comp(80, 80) == 0
    # Eq. 3
    assert O.offload_bound(Fraction(3, 5), Fraction(1, 2)) == Fraction(1, 2)
    # the paper's evaluation runs at an offloading ratio of 70 % (Sec. 4.2 captions): a bound of 0.7
    # lets 7 requests' worth of tokens be offloaded per 10 local ones
    assert O.offload_bound(Fraction(7, 10), Fraction(9, 10)) == Fraction(7, 10)


LOCAL = [(2048, 1000)] * 10          # decode_used_tokens = 10 000
HALF = Fraction(1, 2)                # budget = 5 000 tokens, batch bound = 5 requests


@pytest.mark.parametrize("req,offloaded,expect,why", [
    ((1500, 300), [(2048, 1000)] * 3, 1, "C1: 3000 + 1500 = 4500 < 5000"),
    ((2000, 300), [(2048, 1000)] * 3, 1, "C1 fails at exactly 5000 (strict); C2: 3300 < 5000 and 4 < 5"),
    ((2001, 300), [(2048, 1000)] * 3, 1, "C1 fails (5001); C2 holds"),
    ((2001, 300), [(2048, 800)] * 4, 0, "C1: 3200+2001 > 5000; C2: tokens 3500 < 5000 but batch 5 < 5 is false"),
    ((2001, 2000), [(2048, 1000)] * 3, 0, "C2 fails on tokens at exactly 5000 (strict)"),
    ((2001, 1999), [(2048, 1000)] * 3, 1, "C2: 4999 < 5000 and 4 < 5"),
    ((100, 50), [(2048, 700)] * 7, 0, "tokens 4900 + 100 = 5000 is not < 5000; batch 8 < 5 false"),
    ((99, 50), [(2048, 700)] * 7, 1, "C1 alone suffices (4999 < 5000) whatever the batch size"),
    ((10, 5), [], 1, "empty executor"),
])
def test_algorithm_1_truth_table(req, offloaded, expect, why):
    assert O.need_offload(req, LOCAL, offloaded, HALF) == expect, why


def test_algorithm_1_degenerate_cases():
    assert O.need_offload((10, 5), [], [], Fraction(7, 10)) == 0       # nothing runs locally: budget 0
    assert O.need_offload((10, 5), LOCAL, [], 0) == 0                  # bound 0: never
    # the offloaded requests' maximal lengths do not matter (computed, unused)
    assert O.need_offload((1500, 300), LOCAL, [(10 ** 9, 1000)] * 3, HALF) == 1


def test_graph_capacity_worked_examples():
    assert [O.graph_capacity(n, 8, 64) for n in (0, 1, 8, 9, 63, 64, 65)] == [8, 8, 8, 16, 64, 64, -1]
    assert O.graph_capacity(5, 0, 64) == -1 and O.graph_capacity(-1, 8, 64) == -1
    assert O.graph_capacity(3, 8, 4) == -1


# ---- the library against the oracle -----------------------------------------------------------------

def test_library_bounds_match_oracle():
    rng = random.Random(7)
    for _ in range(200):
        n = rng.randint(0, 6)
        hbm = [rng.randint(1, 80) for _ in range(n)]
        bw = [rng.randint(100, 3000) for _ in range(n)]
        hd, bd = rng.randint(16, 288), rng.randint(500, 8000)
        got = adr.adr_offload_bound_mem(hbm, bw, hd, bd)
        assert got == pytest.approx(float(O.offload_bound_mem(hbm, bw, hd, bd)), rel=1e-15, abs=0)
        bmax, bt = rng.randint(1, 512), rng.randint(1, 256)
        comp = adr.adr_offload_bound_comp(bmax, bt)
        assert comp == pytest.approx(float(O.offload_bound_comp(bmax, bt)), rel=1e-15, abs=0)
        assert adr.adr_offload_bound(got, comp) == min(got, comp)
    assert math.isnan(adr.adr_offload_bound_mem([1], [1], 0, 1)) and math.isnan(adr.adr_offload_bound_comp(4, 0))


def test_library_decision_matches_oracle_including_ties():
    rng = random.Random(11)
    bounds = [Fraction(1, 2), Fraction(7, 10), Fraction(1, 4), Fraction(1), Fraction(3, 2), Fraction(0)]
    for trial in range(3000):
        ob = rng.choice(bounds)
        nl, no = rng.randint(0, 12), rng.randint(0, 12)
        local = [(rng.randint(100, 4096), rng.randint(1, 2000)) for _ in range(nl)]
        off = [(rng.randint(100, 4096), rng.randint(1, 2000)) for _ in range(no)]
        used = rng.randint(1, 2000)
        req = (used + rng.randint(0, 2000), used)
        if trial % 3 == 0 and nl:      # put the new request exactly on a boundary of C1 or C2
            budget = sum(u for _, u in local) * ob
            if budget.denominator == 1:
                target = int(budget) - sum(u for _, u in off)
                if target > 1:
                    req = (target, min(used, target)) if trial % 2 else (target + 500, target)
        want = O.need_offload(req, local, off, ob)
        # a binary fraction as the bound keeps the library's double arithmetic exact; 7/10 is the
        # paper's ratio and is checked too, away from exact ties
        if ob == Fraction(7, 10):
            budget = sum(u for _, u in local) * ob
            s1, s2 = sum(u for _, u in off) + req[0], sum(u for _, u in off) + req[1]
            if budget in (s1, s2) or Fraction(len(off) + 1) == len(local) * ob:
                continue
        assert adr.adr_need_offload(req, local, off, float(ob)) == bool(want), (req, local, off, ob)


def test_library_graph_capacity_matches_oracle():
    for interval in (1, 4, 8, 32):
        for cap in (interval, 64, 256):
            for n in range(-1, 300, 7):
                assert adr.adr_graph_capacity(n, interval, cap) == O.graph_capacity(n, interval, cap)
