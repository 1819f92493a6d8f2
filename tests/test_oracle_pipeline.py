"""Pins of the multi-stage schedule oracle (oracle/pipeline_oracle.py): what the paper and
arithmetic fix, none of it computed by the oracle itself."""
import os
import random

import pytest

from oracle import pipeline_oracle as P
from oracle.stage_oracle import EARLY_BACKWARD, GPIPE

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "pipeline_two_stage_timeline.txt")


def test_hand_worked_two_stage_timeline():
    rows = [l.split() for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    K = P.warmup_depths(2, 3, "A")
    assert K == [2, 1]
    sim = P.simulate([1, 1], [2, 2], 3, P.stage_lists(2, 3, K))
    assert len(rows) == 12 == len(sim["start"])
    for kind, st, mb, t0, t1 in rows:
        key = (kind, int(st), int(mb))
        assert sim["start"][key] == float(t0) and sim["end"][key] == float(t1), key
    assert sim["makespan"] == 12 and sim["peak_live"] == [2, 1]


def test_warmup_depths_of_both_policies():
    # K_i = min(S - i, D) and min(2(S - i) - 1, D)   (section V-C)
    assert P.warmup_depths(4, 16, "A") == [4, 3, 2, 1]
    assert P.warmup_depths(4, 16, "B") == [7, 5, 3, 1]
    assert P.warmup_depths(4, 16, "B", D=4) == [4, 4, 3, 1]
    assert P.warmup_depths(4, 2, "A") == [2, 2, 2, 1]      # never more than the M there are


@pytest.mark.parametrize("S,M", [(1, 1), (1, 5), (2, 2), (3, 8), (4, 16), (5, 3)])
def test_equal_stages_closed_form_and_same_bubbles_as_gpipe_order(S, M):
    f, b = 1.5, 2.75
    want = (M + S - 1) * (f + b)
    for order in (EARLY_BACKWARD, GPIPE):
        for policy in ("A", "B"):
            sim = P.simulate([f] * S, [b] * S, M, P.stage_lists(S, M, P.warmup_depths(S, M, policy), order))
            assert sim["makespan"] == pytest.approx(want, rel=1e-12)
            # every stage idles for the time of S - 1 micro-batches: the bubble of section III-A
            assert sim["bubble"] == pytest.approx([(S - 1) * (f + b)] * S, rel=1e-12)
    assert P.latency_model([f] * S, [b] * S, M) == pytest.approx(want, rel=1e-12)
    assert P.pivot_stage([f] * S, [b] * S, M) == S - 1


def test_residency_is_K_i_for_the_early_backward_order_and_M_for_gpipe():
    S, M = 4, 9
    F, B = [1.0, 0.7, 1.3, 0.9], [2.0, 1.4, 2.6, 1.8]
    for policy in ("A", "B"):
        K = P.warmup_depths(S, M, policy)
        assert P.simulate(F, B, M, P.stage_lists(S, M, K))["peak_live"] == K
    assert P.simulate(F, B, M, P.stage_lists(S, M, None, GPIPE))["peak_live"] == [M] * S


def test_model_is_a_lower_bound_and_exact_when_the_last_stage_is_slowest():
    rng = random.Random(20200701)
    for _ in range(400):
        S, M = rng.randint(1, 5), rng.randint(1, 9)
        F = [rng.uniform(0.5, 2.0) for _ in range(S)]
        B = [rng.uniform(1.0, 4.0) for _ in range(S)]
        sim = P.simulate(F, B, M, P.stage_lists(S, M, P.warmup_depths(S, M, "A")))
        # F_0..F_Q, M x (F_Q + B_Q) on the pivot, B_Q..B_0 is a chain of dependent tasks for any Q
        for Q in range(S):
            assert P.latency_model(F, B, M, Q) <= sim["makespan"] + 1e-9
        gp = P.simulate(F, B, M, P.stage_lists(S, M, None, GPIPE))
        assert sim["makespan"] <= gp["makespan"] + 1e-9          # early backward never costs time
        F[-1], B[-1] = max(F) + 0.1, max(B) + 0.1
        sim = P.simulate(F, B, M, P.stage_lists(S, M, P.warmup_depths(S, M, "A")))
        assert P.pivot_stage(F, B, M) == S - 1
        assert P.latency_model(F, B, M) == pytest.approx(sim["makespan"], rel=1e-12)


def test_hand_worked_unequal_stages():
    # F = (1, 2), B = (2, 4), M = 3: the second stage never waits after its first forward,
    # so the iteration is F_0 + 3 (F_1 + B_1) + B_0 = 1 + 18 + 2 = 21 = T_w + T_s + T_e = 3 + 12 + 6
    sim = P.simulate([1, 2], [2, 4], 3, P.stage_lists(2, 3, [2, 1]))
    assert sim["makespan"] == 21 == P.latency_model([1, 2], [2, 4], 3)
    assert sim["bubble"] == [21 - 9, 21 - 18]


def test_pivot_moves_to_a_dominant_early_stage():
    # stage 0 alone needs (M-1)(F_0+B_0) = 7 x 9 = 63 > 7 x 3 + (F_1 + B_1) = 24
    F, B, M = [3, 1, 1], [6, 2, 2], 8
    assert P.pivot_stage(F, B, M) == 0
    # and not when it is only slightly slower than the last: 7 x 3.3 = 23.1 < 24
    assert P.pivot_stage([1.1, 1, 1], [2.2, 2, 2], M) == 2
    # a one-stage pipeline is M (F + B)
    assert P.latency_model([2.0], [3.0], 5) == 25.0


def test_depths_that_grow_along_the_pipeline_deadlock():
    # stage 1 wants micro-batch 1 before its first backward, stage 0 will not send it before that
    with pytest.raises(RuntimeError):
        P.simulate([1, 1], [1, 1], 3, P.stage_lists(2, 3, [1, 2]))


def test_transfer_time_delays_every_hop():
    # one micro-batch through S stages and back: 2 (S - 1) hops
    S = 3
    sim = P.simulate([1] * S, [2] * S, 1, P.stage_lists(S, 1, [1] * S), comm=0.25)
    assert sim["makespan"] == pytest.approx(S * 3 + 2 * (S - 1) * 0.25)
