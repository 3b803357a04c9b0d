"""Pins of the oracle of a Performance History Table row (Sec. 3.3.2; perplexity:
Sec. 4.4, Appendix A) and of Algorithm 1's load-or-switch branch.  No GPU."""
import numpy as np
import scipy.stats

from oracle.ee_pht import PHTRow, load_or_switch


def _stream(seed, n, exits=(20, 40, 60, 80)):
    g = np.random.default_rng(seed)
    layer = g.choice(exits, size=n, p=[0.4, 0.1, 0.1, 0.4])
    conf = g.uniform(0.05, 1.0, size=n).astype(np.float32)
    breach = (layer == exits[-1]) & (conf < 0.5)
    return layer, conf, breach


def test_exit_profile_is_the_histogram_of_exit_layers():
    exits = (20, 40, 60, 80)
    layer, conf, breach = _stream(0, 5000)
    r = PHTRow(exits)
    r.push(layer, conf, breach)
    want = np.array([(layer == l).sum() for l in exits])
    assert r.exits == want.tolist() and r.tokens == 5000 and r.breaches == int(breach.sum())
    assert abs(sum(r.exit_profile) - 1.0) < 1e-12


def test_perplexity_is_the_geometric_mean_of_inverse_probabilities():
    layer, conf, breach = _stream(1, 3000)
    r = PHTRow((20, 40, 60, 80))
    r.push(layer, conf, breach)
    want = scipy.stats.gmean(1.0 / conf.astype(np.float64))
    assert abs(r.perplexity - want) <= 1e-10 * want


def test_closed_forms():
    r = PHTRow((2, 4))
    r.push([2] * 10, [1.0] * 10, [0] * 10)
    assert r.perplexity == 1.0 and r.nll == 0.0            # certain tokens: perplexity 1
    r = PHTRow((2, 4))
    r.push([4] * 7, [0.25] * 7, [1] * 7)
    assert abs(r.perplexity - 4.0) < 1e-12                  # uniform over 4 choices: perplexity 4
    assert r.exit_profile == [0.0, 1.0] and r.breaches == 7
    r = PHTRow((2, 4))
    r.push([2, 4], [0.5, 0.125], [0, 0])
    assert abs(r.perplexity - 4.0) < 1e-12                  # sqrt(2 * 8)


def test_steps_add_up():
    layer, conf, breach = _stream(2, 1000)
    whole, parts = PHTRow((20, 40, 60, 80)), PHTRow((20, 40, 60, 80))
    whole.push(layer, conf, breach)
    for lo in range(0, 1000, 64):
        parts.push(layer[lo:lo + 64], conf[lo:lo + 64], breach[lo:lo + 64])
    assert parts.exits == whole.exits and parts.breaches == whole.breaches
    assert abs(parts.nll - whole.nll) < 1e-9


def test_load_or_switch_branch():
    # Algorithm 1: the full chosen model wins only if its figure is below the others' low-exit versions
    assert load_or_switch(1.0, {"b": 1.5, "c": 2.0}) == ("load", None)
    assert load_or_switch(1.8, {"b": 1.5, "c": 2.0}) == ("switch", "b")
    assert load_or_switch(3.0, {"b": 2.5, "c": 2.0}) == ("switch", "c")
    # the printed condition is strict: on a tie the else branch (next best candidate) is taken
    assert load_or_switch(2.0, {"b": 2.0}) == ("switch", "b")
    assert load_or_switch(2.0, {"b": 2.0, "c": 2.0}) == ("switch", "b")
    assert load_or_switch(np.nextafter(2.0, 0.0), {"b": 2.0}) == ("load", None)
    assert load_or_switch(9.0, {}) == ("load", None)                # nobody to switch to
