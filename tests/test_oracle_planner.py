"""Pins for the oracle's brute-force placement cost (orc_min_link_bytes): hand-worked cases, a closed
form for a constant budget, and properties any correct minimum has.  None of them re-types the brute
force: the cases were worked by listing the alternatives by hand (tests/golden/min_link_bytes.txt),
the closed form follows from an exchange argument."""
import os

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "min_link_bytes.txt")


def golden_cases():
    out = []
    for line in open(GOLDEN):
        if not line.startswith("case "):
            continue
        name, used, budget, start, want = [f.strip() for f in line[5:].split("|")]
        ints = lambda s: [int(x) for x in s.split()]
        out.append((name, ints(used), ints(budget), ints(start), int(want)))
    return out


def test_golden_file_covers_the_cases_it_must():
    cases = {c[0]: c for c in golden_cases()}
    assert len(cases) >= 8
    assert any(all(s == 0 for s in c[3]) for c in cases.values())                 # an all-host start
    assert any(min(c[2]) >= len(c[1]) for c in cases.values())                    # budget >= n
    assert any(int(np.argmax(c[1])) != 0 for c in cases.values())                 # fullest chunk is not chunk 0
    assert any(c[2] != sorted(c[2]) for c in cases.values()) and any(c[2] != sorted(c[2], reverse=True) for c in cases.values())


@pytest.mark.parametrize("name,used,budget,start,want", golden_cases(), ids=[c[0] for c in golden_cases()])
def test_hand_worked_cases(orc, name, used, budget, start, want):
    assert orc.min_link_bytes(used, budget, start) == want


def test_constant_budget_from_an_all_host_start_has_a_closed_form(orc):
    """With room for b chunks at every step and everything on the host at the start, the best plan reads
    every chunk once in step 0, keeps the b fullest for good and streams the rest in and out at every
    step: 12*sum(top b) + 24*T*sum(rest).  (Exchange argument: swapping a kept chunk for a fuller one
    never costs more.)"""
    rng = np.random.default_rng(77)
    for _ in range(60):
        n = int(rng.integers(1, 6))
        T = int(rng.integers(1, min(4, 24 // n) + 1))
        used = [int(x) for x in rng.integers(0, 50, size=n)]
        b = int(rng.integers(0, n + 2))
        top = sorted(used, reverse=True)[:b]
        want = 12 * sum(top) + 24 * T * (sum(used) - sum(top))
        assert orc.min_link_bytes(used, [b] * T, [0] * n) == want


def test_properties_of_a_minimum(orc):
    rng = np.random.default_rng(78)
    for _ in range(40):
        n = int(rng.integers(1, 5))
        T = int(rng.integers(1, min(4, 20 // n) + 1))
        used = [int(x) for x in rng.integers(0, 30, size=n)]
        budget = [int(x) for x in rng.integers(0, n + 1, size=T)]
        start = [int(x) for x in rng.integers(0, 2, size=n)]
        base = orc.min_link_bytes(used, budget, start)
        # bounds: never below "whatever starts on the host is read once", never above "stream everything"
        lo = 12 * sum(u for u, s in zip(used, start) if not s)
        hi = lo + 12 * sum(used) * T + 12 * sum(used) * (T - 1)
        assert lo <= base <= hi
        # more room never costs more; room for everything costs exactly the first reads
        more = [x + 1 for x in budget]
        assert orc.min_link_bytes(used, more, start) <= base
        assert orc.min_link_bytes(used, [n] * T, start) == lo
        # no room: every chunk is written at every step and read at every step but possibly the first
        none = orc.min_link_bytes(used, [0] * T, start)
        assert none == 12 * sum(used) * T + 12 * sum(used) * (T - 1) + lo
        # scaling every fill scales the cost; chunk order is irrelevant
        assert orc.min_link_bytes([3 * u for u in used], budget, start) == 3 * base
        perm = rng.permutation(n)
        assert orc.min_link_bytes([used[i] for i in perm], budget, [start[i] for i in perm]) == base
