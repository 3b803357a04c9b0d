"""CPU oracle of the confidence-breach counter (CBC).  TEST INFRASTRUCTURE ONLY:
nothing on a product path may import this module.

What the paper fixes (HELIOS, Sec. 3.3.3 "Amortizing Loading Overheads with CBC",
Algorithm 1): a counter goes up by one for every emitted token that did not meet
the confidence threshold; when it exceeds CBC_max the serving loop re-assesses
(load more layers or switch model) and the counter starts again from zero; by
default at most 50 breaches are tolerated in a window of 100 consecutive tokens.

Reading taken where the text is silent: tokens are ordered
by (decode step, row id); the window is the most recent `window` tokens emitted
since the last re-assessment, so a re-assessment empties it; the test is made
after every token; "exceeds" is strictly greater.

The code below is the definition written out token by token with a queue; it is
pinned in tests/test_oracle_cbc.py against a recount from the whole history, closed
forms and hand-made streams.
"""
from collections import deque


class CBC:
    def __init__(self, window=100, cbc_max=50):
        assert window >= 1 and cbc_max >= 0
        self.window = window
        self.cbc_max = cbc_max
        self.recent = deque()        # breach bits of the tokens in the window, oldest first
        self.tokens_seen = 0
        self.triggers = []           # 1-based ordinals of the tokens at which a re-assessment fired

    @property
    def count(self):
        return sum(self.recent)

    def push(self, breach_flags):
        """Feeds the breach flags of the next tokens (in stream order); returns the ordinals of
        the tokens at which the counter exceeded CBC_max."""
        fired = []
        for f in breach_flags:
            self.tokens_seen += 1
            self.recent.append(1 if f else 0)
            if len(self.recent) > self.window:
                self.recent.popleft()
            if sum(self.recent) > self.cbc_max:
                fired.append(self.tokens_seen)
                self.recent.clear()
        self.triggers.extend(fired)
        return fired
