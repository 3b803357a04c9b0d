"""CPU oracle of the per-window serving statistics that make up a row of the
Performance History Table (PHT), and of the load-or-switch branch that reads them.
TEST INFRASTRUCTURE ONLY: nothing on a product path may import this module.

What the paper fixes (HELIOS): the PHT keeps, per model, the request-specific
performance data (throughput, accuracy) and the early-exit profile, i.e. the
distribution of the exit layers that tokens took (Sec. 3.3.2, "Performance History
Table", and the exit-layer histograms of Sec. 3.3.3).  Accuracy is estimated at inference time by the
perplexity of the generated tokens, computed from the token probabilities alone
(Sec. 4.4, Appendix A).  When the breach counter fires, the full version of the
chosen model is taken if its PHT figure is below that of every other candidate's
low-exit version, otherwise the next best candidate's low-exit version (Algorithm 1).

Readings taken where the text is silent: perplexity of a
window = exp of the mean of -ln p over its emitted tokens, p being the probability
the exit head gave the emitted token (the standard definition; the paper prints no
formula); the PHT figure compared in Algorithm 1 is a cost (lower is better); the
comparison is strict as printed there ("<"; Sec. 3.3.3: loading more layers pays only
while its overall resource usage "remains lower" than the other option's), so on a tie
the else branch is taken and the next best candidate's low-exit version is served; throughput is tokens divided by the wall time the caller
measured, so it is not part of the device-side row.

Plain definitions written out; pinned in tests/test_oracle_pht.py.
"""
import math


class PHTRow:
    def __init__(self, exit_layers):
        self.exit_layers = list(exit_layers)      # layers of the resident exits, ascending
        self.tokens = 0
        self.exits = [0] * len(self.exit_layers)  # tokens that left at each of them
        self.breaches = 0
        self.nll = 0.0                            # sum of -ln p over the tokens

    def push(self, out_layer, out_conf, out_breach):
        """One finished decode step: per row, the layer it left at, the probability of the
        token it emitted, and whether it stopped below its threshold."""
        for l, p, b in zip(out_layer, out_conf, out_breach):
            self.tokens += 1
            self.exits[self.exit_layers.index(int(l))] += 1
            self.breaches += 1 if b else 0
            self.nll += -math.log(float(p))

    @property
    def exit_profile(self):
        return [c / self.tokens for c in self.exits]

    @property
    def perplexity(self):
        return math.exp(self.nll / self.tokens)


def load_or_switch(cost_full_chosen, cost_low_exit_others):
    """Algorithm 1, the branch taken when the breach counter exceeds its limit.
    cost_low_exit_others: {candidate: cost of its low-exit version}.  Returns
    ("load", None) or ("switch", candidate)."""
    if not cost_low_exit_others:
        return ("load", None)
    best = min(cost_low_exit_others, key=lambda k: (cost_low_exit_others[k], str(k)))
    if cost_full_chosen < cost_low_exit_others[best]:
        return ("load", None)
    return ("switch", best)
