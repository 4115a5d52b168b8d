"""Pins for the oracle's acceptance under random sampling (Table 2, Temperature = 0.7).

The paper states no rule, so the rule itself is a reading (see the oracle's docstring) and stays "parity
unpinned" with respect to the paper.  What these tests pin is that the oracle computes THAT rule: closed forms
(uniform and two-point distributions), the limit of a vanishing temperature (= the greedy rule), library routines
(scipy's entropy, numpy's searchsorted on a cumulative sum), monotonicity in the two thresholds, and the
empirical distribution of the drawn token."""
import numpy as np
import pytest
import scipy.stats

import synth_inputs as si
from oracle import amphista_oracle as orc


def small_tree(T=16, caps=(4, 2, 2, 2)):
    paths = si.tree_paths(T, caps)
    return orc.tree_from_paths(paths, len(caps))


def random_case(seed, T=16, V=50, peak=4.0):
    rng = np.random.default_rng(seed)
    tree = small_tree(T)
    logits = rng.standard_normal((T, V)) * peak
    tok = rng.integers(0, V, size=T).astype(np.int32)
    return tree, tok, logits, rng


def test_vanishing_temperature_is_the_greedy_rule():
    """p -> one-hot at the argmax: a child passes iff it carries the argmax, and the drawn token is the argmax."""
    for seed in range(20):
        tree, tok, logits, rng = random_case(seed)
        tgt = np.array([orc.row_argmax(r) for r in logits], dtype=np.int32)
        # plant a partly correct path so that accept lengths above zero occur
        for i in range(1, tree.T):
            if rng.random() < 0.6:
                tok[i] = tgt[tree.parent[i]]
        g = orc.accept_greedy(tree, tok, tgt)
        t = orc.accept_typical(tree, tok, logits, 1e-6, 0.3, 0.5, float(rng.random()))
        assert t[0] == g[0] and t[3] == g[3] and t[2] == g[2]
        np.testing.assert_array_equal(t[1], g[1])


@pytest.mark.parametrize("delta,expect_all", [(0.5, True), (0.999, True), (1.001, False), (3.0, False)])
def test_uniform_distribution_closed_form(delta, expect_all):
    """p = 1/V everywhere, H = ln V, threshold = min(eps, delta / V): every candidate passes iff delta < 1
    (eps well above 1/V), whatever the temperature."""
    V = 40
    tree = small_tree()
    tok = np.arange(tree.T, dtype=np.int32) % V
    logits = np.full((tree.T, V), 1.7)
    a, path, nxt, best, margin, _ = orc.accept_typical(tree, tok, logits, 0.7, 0.5, delta, 0.0)
    if expect_all:
        deepest = int(np.max(tree.depth))
        assert a == deepest and best == int(np.nonzero(tree.depth == deepest)[0][0])
        np.testing.assert_allclose(margin[1:], 1.0 / V - delta / V, rtol=1e-9)
    else:
        assert a == 0 and best == 0 and list(path) == [0] + [-1] * tree.K
    assert nxt == 0                      # u = 0: the first token of non-zero probability


def test_eps_caps_the_threshold():
    """A peaked distribution has exp(-H) near 1, so delta * exp(-H) exceeds eps and eps decides."""
    V = 30
    tree = small_tree(T=5, caps=(1, 1, 1, 1))          # a chain
    logits = np.full((tree.T, V), -20.0)
    logits[:, 3] = 0.0                                  # p(3) ~ 1 - 3e-8 ... at T = 1
    logits[:, 7] = np.log(0.05)                         # p(7) ~ 0.0476
    tok = np.array([0, 7, 7, 7, 7], dtype=np.int32)
    assert orc.accept_typical(tree, tok, logits, 1.0, 0.04, 0.9, 0.5)[0] == 4     # 0.0476 > eps = 0.04
    assert orc.accept_typical(tree, tok, logits, 1.0, 0.06, 0.9, 0.5)[0] == 0     # 0.0476 < eps = 0.06


def test_two_point_entropy_and_threshold():
    """Two tokens with probabilities q and 1 - q: H = -q ln q - (1-q) ln(1-q) in nats; the temperature scales
    the logit gap."""
    V, temp = 12, 0.7
    tree = small_tree(T=2, caps=(1, 1, 1, 1))
    for q in (0.1, 0.35, 0.5):
        gap = np.log((1 - q) / q) * temp                # after dividing by temp the odds are (1-q)/q
        logits = np.full((2, V), -1e9)
        logits[:, 2], logits[:, 5] = gap, 0.0
        H = -(q * np.log(q) + (1 - q) * np.log(1 - q))
        tok = np.array([0, 5], dtype=np.int32)
        for delta in (0.2, 0.6, 0.95):
            margin = orc.accept_typical(tree, tok, logits, temp, 10.0, delta, 0.0)[4]
            np.testing.assert_allclose(margin[1], q - delta * np.exp(-H), rtol=1e-9, atol=1e-12)


def test_entropy_and_probabilities_against_scipy():
    for seed in range(5):
        tree, tok, logits, rng = random_case(100 + seed, V=64)
        temp, delta = 0.7, 0.3
        margin = orc.accept_typical(tree, tok, logits, temp, 1e9, delta, 0.0)[4]
        for i in range(1, tree.T):
            j = tree.parent[i]
            p = scipy.special.softmax(logits[j] / temp)
            H = scipy.stats.entropy(p)                   # natural logarithm
            np.testing.assert_allclose(margin[i], p[tok[i]] - delta * np.exp(-H), rtol=1e-9, atol=1e-14)


def test_accept_length_never_grows_with_the_thresholds():
    for seed in range(10):
        tree, tok, logits, rng = random_case(200 + seed, V=20, peak=1.0)
        prev = None
        for eps, delta in [(0.001, 0.01), (0.02, 0.1), (0.05, 0.3), (0.09, 0.6), (0.5, 0.9), (0.9, 5.0)]:
            a = orc.accept_typical(tree, tok, logits, 0.7, eps, delta, 0.3)[0]
            assert prev is None or a <= prev
            prev = a


def test_a_rejected_parent_rejects_its_descendants():
    V = 10
    tree = small_tree(T=5, caps=(1, 1, 1, 1))          # chain 0-1-2-3-4
    logits = np.zeros((5, V))
    logits[:, 1] = 5.0                                  # token 1 is typical everywhere
    tok = np.array([0, 1, 9, 1, 1], dtype=np.int32)     # node 2 carries an improbable token
    a, path, nxt, best, margin, _ = orc.accept_typical(tree, tok, logits, 1.0, 0.09, 0.3, 0.0)
    assert a == 1 and best == 1 and list(path) == [0, 1, -1, -1, -1]
    assert margin[3] > 0 and margin[4] > 0              # they would pass on their own


def test_drawn_token_inverts_the_cumulative_distribution():
    rng = np.random.default_rng(7)
    V = 37
    tree = small_tree(T=1, caps=(1, 1, 1, 1))
    logits = rng.standard_normal((1, V)) * 2.0
    tok = np.zeros(1, dtype=np.int32)
    temp = 0.7
    p = scipy.special.softmax(logits[0] / temp)
    cdf = np.cumsum(p)
    for u in list(rng.random(200)) + [0.0, float(cdf[0]) * 0.999, float(cdf[5]) + 1e-12, 1.0 - 1e-12]:
        nxt = orc.accept_typical(tree, tok, logits, temp, 0.09, 0.3, float(u))[2]
        assert nxt == min(int(np.searchsorted(cdf, u, side="right")), V - 1)


def test_drawn_tokens_follow_the_target_distribution():
    """Uniform u in, p_best out: the empirical frequencies over 20000 draws stay within five standard errors."""
    rng = np.random.default_rng(11)
    V = 8
    tree = small_tree(T=1, caps=(1, 1, 1, 1))
    logits = rng.standard_normal((1, V))
    tok = np.zeros(1, dtype=np.int32)
    p = scipy.special.softmax(logits[0] / 0.7)
    n = 20000
    counts = np.zeros(V)
    for u in rng.random(n):
        counts[orc.accept_typical(tree, tok, logits, 0.7, 0.09, 0.3, float(u))[2]] += 1
    assert np.all(np.abs(counts / n - p) < 5 * np.sqrt(p * (1 - p) / n))


def test_zero_probability_tokens_are_never_drawn():
    V = 6
    tree = small_tree(T=1, caps=(1, 1, 1, 1))
    logits = np.array([[-np.inf, 0.0, -np.inf, 0.0, -np.inf, -np.inf]])
    tok = np.zeros(1, dtype=np.int32)
    assert orc.accept_typical(tree, tok, logits, 0.7, 0.09, 0.3, 0.0)[2] == 1
    assert orc.accept_typical(tree, tok, logits, 0.7, 0.09, 0.3, 0.49)[2] == 1
    assert orc.accept_typical(tree, tok, logits, 0.7, 0.09, 0.3, 0.51)[2] == 3
    assert orc.accept_typical(tree, tok, logits, 0.7, 0.09, 0.3, 1.0)[2] == 3     # u = 1 (out of range): last live token
