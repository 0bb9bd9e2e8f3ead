"""Peak number of call-context tags alive at once when fib is expanded breadth first in synchronous
time steps: a plain interval count, independent of both implementations.

A frame of fib(k) entered at time s is alive during [s, s + L(k)); the frames of its two calls are
entered at s + c; L(k) = A for k < 2 (a base case) and L(k) = c + L(k-1) + r otherwise (the deeper
call returns after L(k-1), the caller needs r more to add and return).  The constants are the time
steps of an executor: the oracle's synchronous rounds give A : c : r = 3 : 2 : 1 (pinned in
tests/test_oracle_live_tags.py); an executor that sweeps a whole frame per step, creates the callee
frames in the step after the caller's and frees a frame in the step that finds it complete gives
2 : 1 : 1.
"""
from collections import Counter


def fib_peak_live(ns, A, c, r):
    """Largest number of frames alive at once for the batch fib(n), n in ns, all started together."""
    life = {0: A, 1: A}
    for k in range(2, max(list(ns) + [1]) + 1):
        life[k] = c + life[k - 1] + r
    events = Counter()
    for n in ns:
        level = Counter({n: 1})            # frames entered at depth d, by argument
        d = 0
        while level:
            nxt = Counter()
            for k, cnt in level.items():
                events[d * c] += cnt
                events[d * c + life[k]] -= cnt
                if k >= 2:
                    nxt[k - 1] += cnt
                    nxt[k - 2] += cnt
            level, d = nxt, d + 1
    cur = best = 0
    for t in sorted(events):
        cur += events[t]
        best = max(best, cur)
    return best
