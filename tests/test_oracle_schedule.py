"""Pins for the oracle's schedule generator: the paper's worked two-stage
example and control-edge rules (section V-C), the memory behaviour of section
III-B and Table VI, and brute-force validity for every small (M, K)."""
import os

import pytest

from oracle import stage_oracle as O

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _fmt(ops):
    return " ".join(f"{k}{m}" for k, m in ops)


def test_worked_two_stage_example():
    n = 0
    for line in open(os.path.join(GOLD, "schedule_worked_example.txt")):
        if line.startswith("#") or not line.strip():
            continue
        S, i, M, K, *want = line.split()
        S, i, M, K = int(S), int(i), int(M), int(K)
        assert O.warmup_depth("A", S, i, D=99) == K
        assert _fmt(O.schedule_ops(M, K, O.EARLY_BACKWARD)) == " ".join(want)
        n += 1
    assert n == 6


def test_warmup_depth_policies():
    # K_i = min(S - i, D) and min(2(S - i) - 1, D)
    assert [O.warmup_depth("A", 4, i, 8) for i in range(4)] == [4, 3, 2, 1]
    assert [O.warmup_depth("B", 4, i, 8) for i in range(4)] == [7, 5, 3, 1]
    assert O.warmup_depth("A", 4, 0, 2) == 2 and O.warmup_depth("B", 4, 0, 3) == 3


@pytest.mark.parametrize("M", range(1, 10))
@pytest.mark.parametrize("K", range(1, 10))
def test_edges_and_validity(M, K):
    ops = O.schedule_ops(M, K, O.EARLY_BACKWARD)
    pos = {op: i for i, op in enumerate(ops)}
    assert len(ops) == 2 * M and len(pos) == 2 * M
    Kp = min(K, M)
    for m in range(M):
        assert pos[("F", m)] < pos[("B", m)]
    for k in range(1, Kp):                        # warm-up edges F_{k-1} -> F_k
        assert pos[("F", k - 1)] < pos[("F", k)]
    for m in range(M):                            # steady edges B_m -> F_{m+K}
        if m + Kp < M:
            assert pos[("B", m)] < pos[("F", m + Kp)]
            assert pos[("F", m + Kp)] == pos[("B", m)] + 1      # strict alternation
    assert [m for k, m in ops if k == "B"] == list(range(M))    # ascending backwards
    assert [m for k, m in ops if k == "F"] == list(range(M))
    trace = O.live_trace(ops)
    assert max(trace) == Kp and trace[-1] == 0
    # rises like GPipe's until K are injected, then never exceeds K
    assert trace[:Kp] == list(range(1, Kp + 1))
    assert all(t in (Kp, Kp - 1) for t in trace[Kp - 1:2 * M - Kp])


@pytest.mark.parametrize("M", [1, 2, 5, 16])
def test_gpipe_order(M):
    ops = O.schedule_ops(M, 3, O.GPIPE)
    assert ops == [("F", m) for m in range(M)] + [("B", m) for m in range(M)]
    assert max(O.live_trace(ops)) == M


def test_k_at_least_m_degenerates_to_gpipe_order():
    assert O.schedule_ops(3, 3, O.EARLY_BACKWARD) == O.schedule_ops(3, 3, O.GPIPE)
    assert O.schedule_ops(3, 7, O.EARLY_BACKWARD) == O.schedule_ops(3, 3, O.GPIPE)


def test_peak_independent_of_M_like_table6():
    rows = [l.split() for l in open(os.path.join(GOLD, "table6_memory.txt"))
            if l.strip() and not l.startswith("#")]
    dapple = [(int(r[1]), r[3]) for r in rows if r[0] == "DAPPLE"]
    assert len({mem for _, mem in dapple}) == 1            # the paper's constant peak
    K = 2
    peaks = {M: max(O.live_trace(O.schedule_ops(M, K, O.EARLY_BACKWARD))) for M, _ in dapple}
    assert set(peaks.values()) == {K}
    gp = [max(O.live_trace(O.schedule_ops(M, K, O.GPIPE))) for M in (2, 3, 8, 16)]
    assert gp == [2, 3, 8, 16]


def test_bad_arguments():
    with pytest.raises(ValueError):
        O.schedule_ops(0, 1, O.GPIPE)
    with pytest.raises(ValueError):
        O.schedule_ops(2, 0, O.EARLY_BACKWARD)
    with pytest.raises(ValueError):
        O.schedule_ops(2, 1, 7)
