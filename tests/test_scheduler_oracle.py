"""Pins for the run-bookkeeping oracle: queue contents and decisions worked by hand from the
paper's rules (Sections "State tracking", "Invalidation detection", "Cancellation
back-propagation", "Reactive speculation")."""
import pytest

from oracle.scheduler import OracleScheduler, SUPERFLUOUS, INVALIDATED


def test_chain_of_runs_worked_by_hand():
    s = OracleScheduler(0.25, 0.125, 0.0625)
    assert s.accept_tokens([5, 6, 7], run_completed=False) == []          # prompt: positions 0..2
    r_ns = s.begin_run(False, [], 0, [7], [-1], [2])                      # evaluates the last accepted token
    r0 = s.begin_run(True, [], 0, [10, 11], [-1, 0], [3, 4])              # speculates positions 3, 4
    r1 = s.begin_run(True, [10, 11], 3, [12, 13], [-1, 0], [5, 6])        # builds on r0's tokens
    assert (r_ns, r0, r1) == (0, 1, 2)
    # position 3 becomes 10, as r0 guessed: the non-speculative run has nothing new to say
    # (its highest position, 2, is below the accepted end, 3); it is marked, not signalled
    assert s.accept_tokens([10]) == [(r_ns, SUPERFLUOUS, False)]
    # position 4 becomes 99: r0's second token and r1's assumption are wrong
    assert s.accept_tokens([99]) == [(r0, INVALIDATED, True), (r1, INVALIDATED, True)]
    assert s.accept_tokens([1]) == []                                     # each run is reported once
    assert [rec.id for rec in s.fifo] == [0, 1, 2]
    assert s.complete_run(r_ns) == SUPERFLUOUS and s.complete_run(r0) == INVALIDATED
    assert [rec.id for rec in s.fifo] == [2]
    with pytest.raises(KeyError):
        s.complete_run(r0)
    # accepted now holds positions 0..5; a run for positions 6, 7 that guessed right lives until
    # the accepted end has passed its highest position, and not one token earlier
    r3 = s.begin_run(True, [], 0, [2, 3], [-1, 0], [6, 7])
    assert s.accept_tokens([2]) == []
    assert s.accept_tokens([3]) == []                                     # end 7 == highest position: still useful
    assert s.accept_tokens([4]) == [(r3, SUPERFLUOUS, True)]
    assert s.complete_run(r1) == INVALIDATED and s.complete_run(r3) == SUPERFLUOUS
    assert s.fifo == []


def test_assumed_tokens_beyond_the_accepted_end_are_not_judged():
    s = OracleScheduler(0.5, 0.0, 0.0)
    s.accept_tokens([1, 2], run_completed=False)
    r = s.begin_run(True, [7, 8], 2, [9], [-1], [4])
    assert s.accept_tokens([7]) == []                                     # position 3 not known yet
    assert s.accept_tokens([5]) == [(r, INVALIDATED, True)]               # position 3 is 5, not 8


def test_tree_run_follows_any_branch():
    def fresh():
        s = OracleScheduler(0.5, 0.0, 0.0)
        s.accept_tokens([1, 2], run_completed=False)
        # roots 4 and 5 at position 2; 6 under 4; 7 and 8 under 5; 9 under 7 (position 4)
        r = s.begin_run(True, [], 0, [4, 5, 6, 7, 8, 9], [-1, -1, 0, 1, 1, 3], [2, 2, 3, 3, 3, 4])
        return s, r
    s, r = fresh()
    assert s.accept_tokens([5]) == [] and s.accept_tokens([8]) == []      # 5 -> 8 is a branch
    assert s.accept_tokens([3]) == []                                     # the branch ended: nothing to contradict
    assert s.accept_tokens([3]) == [(r, SUPERFLUOUS, True)]               # end 5 > highest position 4
    s, r = fresh()
    assert s.accept_tokens([5, 7, 9]) == []
    s, r = fresh()
    assert s.accept_tokens([5, 6]) == [(r, INVALIDATED, True)]            # 6 hangs under 4, not under 5
    s, r = fresh()
    assert s.accept_tokens([3]) == [(r, INVALIDATED, True)]               # no root matches
    s, r = fresh()
    assert s.accept_tokens([5, 7, 1]) == [(r, INVALIDATED, True)]


def test_cutoff_rises_falls_and_resets():
    s = OracleScheduler(0.25, 0.125, 0.0625)                              # dyadic: exact in binary
    assert s.want_speculation(0.25) and not s.want_speculation(0.2)
    for _ in range(3):
        s.on_speculated()
    assert s.cutoff == 0.625 and not s.want_speculation(0.5)
    s.on_speculation_stopped(logits_waiting=True)
    assert s.cutoff == 0.625
    s.on_speculation_stopped(logits_waiting=False)
    assert s.cutoff == 0.5625
    s.accept_tokens([1], run_completed=False)
    assert s.cutoff == 0.5625
    s.accept_tokens([2], run_completed=True)
    assert s.cutoff == 0.25
    for _ in range(8):
        s.on_speculation_stopped(False)
    assert s.cutoff == -0.25                                              # not clamped
