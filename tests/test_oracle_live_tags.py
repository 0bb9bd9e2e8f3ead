"""Pins of the oracle's count of tags alive at once (Section 5.1: a frame lives from the Call that
creates it to the Return that deallocates it)."""
import oracle
from oracle import programs as oprog
from live_model import fib_peak_live


def _fib_peak(ns):
    it = oracle.Interpreter(oracle.transform(oprog.fib_program()))
    out = it.run({("in", 0): list(ns)}, len(ns), track_live=True)[("out", 0)]
    return it, out


def test_fib_live_tags_follow_the_interval_model():
    # breadth-first expansion in synchronous rounds: the peak is that of overlapping lifetimes
    for n in range(0, 14):
        it, _ = _fib_peak([n])
        assert it.peak_live_tags == fib_peak_live([n], 3, 2, 1), n
        assert it.peak_live_tags <= len(it.tags)
    it, out = _fib_peak([5, 9, 12])                       # a batch: instances expand side by side
    assert out == [5, 34, 144]
    assert it.peak_live_tags == fib_peak_live([5, 9, 12], 3, 2, 1)


def test_a_single_call_chain_keeps_every_frame_alive():
    # fact(n) = n * fact(n-1): nothing returns before the innermost call does: all n tags alive
    it = oracle.Interpreter(oracle.transform(oprog.fact_program()))
    it.run({}, 1, track_live=True)
    assert it.peak_live_tags == len(it.tags) == 3          # fact(3): tags [0], [1,0], [1,1,0]


def test_loops_keep_a_bounded_number_of_tags_alive():
    # an iteration's frame is dead once its Next tokens have left: O(1) per loop instance,
    # whatever the trip count
    prog = oracle.transform(oprog.sum_loop_program())
    peaks = []
    for n in (3, 30, 300):
        it = oracle.Interpreter(prog)
        assert it.run({("in", 0): [n]}, 1, track_live=True)[("out", 0)] == [n * (n + 1) // 2]
        assert len(it.iter_tags) == n + 1
        peaks.append(it.peak_live_tags)
    assert peaks[0] == peaks[1] == peaks[2] <= 2
    it = oracle.Interpreter(oracle.transform(oprog.gcd_loop_program()))
    it.run({("in", 0): [1000, 7, 300], ("in", 1): [3, 7, 299]}, 3, track_live=True)
    assert len(it.iter_tags) > 600 and it.peak_live_tags <= 2 * 3
