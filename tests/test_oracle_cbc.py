"""Pins of the confidence-breach-counter oracle (Sec. 3.3.3, Algorithm 1 of the paper)."""
import numpy as np

from oracle.ee_cbc import CBC


def recount(flags, window, cbc_max):
    """The same rule stated without a queue: at token t (1-based) count the breaches among the
    tokens max(last re-assessment + 1, t - window + 1) .. t of the whole history."""
    flags = [1 if f else 0 for f in flags]
    fired, last = [], 0
    for t in range(1, len(flags) + 1):
        lo = max(last + 1, t - window + 1)
        if sum(flags[lo - 1:t]) > cbc_max:
            fired.append(t)
            last = t
    return fired


def test_matches_a_recount_from_the_whole_history_on_random_streams():
    rng = np.random.default_rng(5)
    for window, cbc_max, p in ((100, 50, 0.5), (100, 50, 0.6), (10, 3, 0.4), (7, 0, 0.1), (1, 0, 0.5), (64, 63, 0.99)):
        flags = (rng.random(3000) < p).astype(np.uint8)
        c = CBC(window, cbc_max)
        got = []
        at = 0
        while at < len(flags):                  # fed in uneven pieces, like decode steps of a shrinking batch
            n = int(rng.integers(1, 300))
            got += c.push(flags[at:at + n])
            at += n
        assert got == recount(flags, window, cbc_max) == c.triggers
        assert c.tokens_seen == len(flags)


def test_default_tolerates_fifty_breaches_in_a_hundred_tokens():
    # the paper's default: up to 50 breaches in 100 consecutive tokens are tolerated
    c = CBC()
    assert c.push([1, 0] * 500) == []           # every window of 100 holds exactly 50
    assert c.count == 50


def test_fifty_first_breach_in_the_window_fires_and_the_counter_restarts():
    c = CBC()
    assert c.push([1] * 50) == []
    assert c.push([0] * 49) == []               # 99 tokens, 50 breaches
    assert c.push([1]) == [100]                 # the 51st breach among the last 100 tokens
    assert c.count == 0 and len(c.recent) == 0  # re-assessment empties the window (Algorithm 1: CBC <- 0)
    assert c.push([1] * 50) == []               # the old breaches do not count again
    assert c.push([1]) == [151]


def test_breaches_leave_the_window_after_a_hundred_tokens():
    c = CBC()
    assert c.push([1] * 50 + [0] * 50) == []    # 50 breaches, now 50..99 tokens old
    assert c.push([1] * 1) == []                # the oldest breach has just left: still 50
    assert c.push([0, 1] * 200) == []           # one breach every other token: 50 per 100, never more
    assert c.count == 50
    assert c.push([1]) == [502]                 # two breaches in a row make it 51


def test_all_breaching_stream_fires_every_cbc_max_plus_one_tokens():
    for window, cbc_max in ((100, 50), (10, 3), (5, 9)):
        c = CBC(window, cbc_max)
        fired = c.push([1] * 1000)
        if cbc_max >= window:                   # the window can never hold more than `window` breaches
            assert fired == []
        else:
            assert fired == list(range(cbc_max + 1, 1001, cbc_max + 1))


def test_no_breach_never_fires_and_zero_tolerance_fires_on_every_breach():
    assert CBC().push([0] * 1000) == []
    c = CBC(100, 0)
    flags = [0, 1, 0, 0, 1, 1, 0]
    assert c.push(flags) == [2, 5, 6]
