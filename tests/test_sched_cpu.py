"""Host-side schedule model against what the paper states: the worked six-device example
(tests/golden/paper_schedule_examples.txt), the mapping formula, the closed forms of the
Theoretical Analysis, and structural invariants of the step table."""
import itertools
import os

import pytest

import paper_2511_09741_amd.binding as taw

FWD, BWD, IDLE = 1, 2, 0


def _golden():
    """(key, value, citation) of every line of tests/golden/paper_schedule_examples.txt"""
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "paper_schedule_examples.txt")
    out = []
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            lhs, cite = line.split(";", 1)
            key, val = lhs.split("=")
            out.append((key.split(), int(val), cite.strip()))
    return out


def test_worked_example_of_the_paper():
    """Every value the paper states for its six-device example (two groups of three, six layers), read from the
    golden file, against the schedule model."""
    P, D, L = 6, 2, 6
    lines = _golden()
    assert len(lines) >= 16
    kinds = set()
    for key, val, cite in lines:
        kinds.add(key[0])
        if key[0] == "owner":
            got = taw.taw_sched_owner(P, D, L, int(key[1]))[0]
        elif key[0] == "step":
            got = taw.taw_sched_step(P, D, L, int(key[1][1:]), int(key[2][1:]))[key[3]]
        elif key[0] == "update":
            got = taw.taw_sched_update_step(P, D, L, int(key[1]))
        else:
            raise AssertionError(f"unknown key {key}")
        assert got == val, (key, got, val, cite)
    assert kinds == {"owner", "step", "update"}


@pytest.mark.parametrize("P,D", [(6, 2), (8, 1), (24, 3), (16, 4), (4, 4)])
def test_mapping_formula_is_a_balanced_bijection(P, D):
    """Device i of group k holds W_((D i + k) mod P): every device exactly one shard per P layers."""
    L = 2 * P
    per = P // D
    for k, i in itertools.product(range(D), range(per)):
        layer = (D * i + k) % P
        assert taw.taw_sched_owner(P, D, L, layer) == (k * per + i, k)
        assert taw.taw_sched_owner(P, D, L, layer + P) == (k * per + i, k)      # the pattern repeats
    assert sorted(taw.taw_sched_owner(P, D, L, j)[0] for j in range(P)) == list(range(P))


@pytest.mark.parametrize("P,D,L", [(6, 2, 6), (24, 3, 48), (8, 4, 16)])
def test_step_table_invariants(P, D, L):
    per = P // D
    for g in range(D):
        seen_f, seen_b = [], []
        for t in range(2 * L + D - 1):
            s = taw.taw_sched_step(P, D, L, g, t)
            if s["phase"] == IDLE:
                assert t < g or t >= 2 * L + g
                continue
            (seen_f if s["phase"] == FWD else seen_b).append(s["layer"])
            assert g * per <= s["master"] < (g + 1) * per                        # the master is a member of the group
            owner, og = taw.taw_sched_owner(P, D, L, s["layer"])
            assert (s["master"] == owner) == (og == g)
            nxt = taw.taw_sched_step(P, D, L, g, t + 1) if t + 1 <= 2 * L + D - 2 else None
            if s["prefetch_from"] >= 0:                                          # exactly the remote shards are prefetched, from their owner
                assert nxt and taw.taw_sched_owner(P, D, L, nxt["layer"]) == (s["prefetch_from"], s["prefetch_from"] // per)
                assert s["prefetch_from"] // per != g
            elif nxt and nxt["phase"] != IDLE and nxt["layer"] != s["layer"]:
                assert taw.taw_sched_owner(P, D, L, nxt["layer"])[1] == g
        assert seen_f == list(range(L)) and seen_b == list(reversed(range(L)))    # every layer once, in order
    # an owner updates after the last group delivered, one step after that group's backward of the layer
    for j in range(L):
        last = [t for t in range(2 * L + D - 1) if taw.taw_sched_step(P, D, L, D - 1, t)["phase"] == BWD
                and taw.taw_sched_step(P, D, L, D - 1, t)["layer"] == j]
        assert taw.taw_sched_update_step(P, D, L, j) == last[0]


def test_closed_forms_of_the_theoretical_analysis():
    a, b = taw.taw_sched_bubble_ratio(24, 3, 48, 64)
    assert a == pytest.approx((2 * 24 + 64) / ((3 * 64 + 2) * 24 + 64)) and b == pytest.approx(23 / (64 + 23))
    assert a < b                                                                 # fewer idle slots than 1F1B / ring passing
    # one group: the expression reduces to N / (3 N P + N) = 1 / (3 P + 1)
    a1, _ = taw.taw_sched_bubble_ratio(8, 1, 8, 5)
    assert a1 == pytest.approx(1 / 25)
    t, w, f = taw.taw_sched_comm_elems(24, 4, 16384, 4096)
    assert t == 24 * 4096**2 and w == 36 * 4096**2 and f == 2 * 24 * 4 * 16384 * 4096
    assert 1 - t / w == pytest.approx(1 / 3)                                      # the stated 33 % reduction
    assert t < f                                                                 # weights are cheaper to move than long-context activations


def test_bad_arguments_are_rejected():
    for args in [(6, 4, 6, 0), (6, 2, 7, 0), (6, 2, 6, 6), (6, 2, 6, -1)]:
        with pytest.raises(ValueError):
            taw.taw_sched_owner(*args)
    with pytest.raises(ValueError):
        taw.taw_sched_step(6, 2, 6, 2, 0)
    with pytest.raises(ValueError):
        taw.taw_sched_step(6, 2, 6, 0, 13)
