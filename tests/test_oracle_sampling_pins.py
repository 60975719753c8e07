"""Pins for the oracle's nucleus sampler (CPU only): its integer probability masses against the library exponential,
hand-computed distributions, the limits in which it must turn into arg-max, exact frequencies on a grid of uniforms,
an independent formulation of the nucleus with exact rationals, and the property the paper claims for it -- decoding
with drafts emits what plain sampling emits."""
import math
from fractions import Fraction

import numpy as np
import pytest

import oracle
import synth


def logits_of(probs):
    return np.log(np.asarray(probs, dtype=np.float64)).astype(np.float32)


def test_hand_distribution_boundaries():
    # probabilities 1/2, 1/4, 1/8, 1/16, 1/16 at tokens 3, 0, 4, 1, 2
    probs = np.zeros(5)
    probs[[3, 0, 4, 1, 2]] = [0.5, 0.25, 0.125, 0.0625, 0.0625]
    lg = logits_of(probs)
    # top_p 0.8: cumulative .5, .75, .875 -> nucleus {3, 0, 4} with mass .875; draw boundaries at 4/7 and 6/7
    want = {0.0: 3, 0.3: 3, 0.57: 3, 0.58: 0, 0.85: 0, 0.86: 4, 0.999: 4}
    for u, tok in want.items():
        assert oracle.nucleus_sample(lg, 1.0, 0.8, u)[0] == tok, u
    # top_p just under / over the mass 0.75 of the first two tokens (the logits are float32 roundings of log p, so the
    # sum is 0.75 only to about 1e-7)
    assert {oracle.nucleus_sample(lg, 1.0, 0.7499, u)[0] for u in np.linspace(0, 0.999, 50)} == {3, 0}
    assert {oracle.nucleus_sample(lg, 1.0, 0.7501, u)[0] for u in np.linspace(0, 0.999, 50)} == {3, 0, 4}
    # top_p 1: everything; the two equal tails are ordered by token id
    assert oracle.nucleus_sample(lg, 1.0, 1.0, 0.88)[0] == 1
    assert oracle.nucleus_sample(lg, 1.0, 1.0, 0.95)[0] == 2
    # temperature 1/2 squares the probabilities: 256, 64, 16, 4, 4 over 344
    assert oracle.nucleus_sample(lg, 0.5, 1.0, 255.9 / 344)[0] == 3
    assert oracle.nucleus_sample(lg, 0.5, 1.0, 256.1 / 344)[0] == 0
    assert oracle.nucleus_sample(lg, 0.5, 1.0, 336.1 / 344)[0] == 1


def test_boundaries_hit_exactly():
    """Four equal logits: every probability is exactly 1/4 and every cumulative sum exact, so both inequalities of the
    definition show: the nucleus is the shortest prefix whose mass is >= top_p (not >), and the draw is the first
    token whose cumulative mass exceeds (not reaches) u times the nucleus mass."""
    lg = np.full(4, 1.5, dtype=np.float32)
    # top_p = 1/2 is reached by two tokens: nucleus {0, 1}, mass 1/2.  A nucleus of three would give token 2 at u = 0.7.
    assert oracle.nucleus_sample(lg, 1.0, 0.5, 0.7)[0] == 1
    assert {oracle.nucleus_sample(lg, 1.0, 0.5, u)[0] for u in np.linspace(0, 0.999, 40)} == {0, 1}
    # u = 1/2: the target 1/4 equals the first cumulative sum, which does not exceed it: token 1
    assert oracle.nucleus_sample(lg, 1.0, 0.5, 0.5)[0] == 1
    assert oracle.nucleus_sample(lg, 1.0, 0.5, 0.4999)[0] == 0
    # top_p = 1: all four; targets on the cumulative sums go to the next token
    assert [oracle.nucleus_sample(lg, 1.0, 1.0, u)[0] for u in (0.0, 0.25, 0.5, 0.75)] == [0, 1, 2, 3]


def test_limits_are_argmax_with_lowest_id_on_ties():
    rng = np.random.default_rng(0)
    for _ in range(20):
        lg = rng.standard_normal(200).astype(np.float32)
        best = int(np.argmax(lg))
        for u in (0.0, 0.5, 0.999):
            # a vanishing temperature puts all mass on the single largest logit
            assert oracle.nucleus_sample(lg, 1e-4, 0.9, u)[0] == best
        lg[rng.integers(200)] = lg.max()                  # maybe a tie for the maximum
        best = int(np.argmax(lg))                         # numpy returns the first maximum
        for u in (0.0, 0.5, 0.999):
            # a vanishing top_p keeps one token: the most probable, lowest id among equals
            assert oracle.nucleus_sample(lg, 1.0, 1e-9, u)[0] == best


def test_frequencies_on_a_uniform_grid_equal_renormalised_probabilities():
    rng = np.random.default_rng(1)
    probs = rng.dirichlet(np.ones(12) * 0.7)
    lg = logits_of(probs)
    p = np.exp(lg.astype(np.float64))
    p /= p.sum()
    top_p = 0.9
    order = sorted(range(12), key=lambda i: (-p[i], i))
    acc, nucleus = 0.0, []
    for i in order:
        nucleus.append(i)
        acc += p[i]
        if acc >= top_p:
            break
    N = 20000
    counts = np.zeros(12, dtype=int)
    for i in range(N):
        counts[oracle.nucleus_sample(lg, 1.0, top_p, (i + 0.5) / N)[0]] += 1
    assert set(np.nonzero(counts)[0]) == set(nucleus)
    for i in nucleus:
        assert abs(counts[i] - N * p[i] / acc) <= 1.0 + 1e-9


@pytest.mark.parametrize("seed", range(6))
def test_nucleus_against_exact_rationals(seed):
    """Probabilities that are exact dyadic rationals: the nucleus and the draw computed with Fractions."""
    rng = np.random.default_rng(seed)
    V = 9
    w = rng.integers(1, 64, size=V)
    w[rng.integers(V)] = w[rng.integers(V)]              # a tie now and then
    total = int(w.sum())
    # scale so that the probabilities are w / 2^k: pad one extra token with the remainder
    k = int(np.ceil(np.log2(total + 1)))
    w = np.append(w, 2 ** k - total)
    probs = [Fraction(int(x), 2 ** k) for x in w]
    lg = logits_of([float(x) for x in probs])
    order = sorted(range(V + 1), key=lambda i: (-probs[i], i))
    for top_p in (Fraction(1, 3), Fraction(7, 10), Fraction(19, 20)):
        acc, cut = Fraction(0), []
        for i in order:
            cut.append(i)
            acc += probs[i]
            if acc >= top_p:
                break
        for u in (Fraction(1, 97), Fraction(30, 97), Fraction(61, 97), Fraction(96, 97)):
            run, want = Fraction(0), None
            for i in cut:
                run += probs[i]
                if run > u * acc:
                    want = i
                    break
            got, margin = oracle.nucleus_sample(lg, 1.0, float(top_p), float(u))
            assert margin > 1e-9          # the thresholds above never sit on a boundary
            assert got == want


def test_rest_decoding_with_sampled_acceptance_equals_plain_sampling():
    """With the uniform number tied to the position in the sequence, REST's draft/verify/accept loop must emit
    exactly the tokens of one-token-at-a-time nucleus sampling ("Sampling strategies")."""
    corp = synth.make_corpus(20000, 3, 40)
    V = 64
    table = np.random.default_rng(5).standard_normal((V, V, 16)).astype(np.float32)
    us = np.random.default_rng(6).random(4096)

    def next_token(seq):
        a, b = int(seq[-1]) % V, int(seq[-2]) % V
        lg = np.full(32000, -30.0, dtype=np.float32)
        # a corpus-aware toy model: strong preference for what followed the last token in the stream somewhere
        hits = np.nonzero(corp.tokens[:-1] == seq[-1])[0][:16]
        lg[corp.tokens[hits + 1]] = 2.0 + table[a, b, :hits.size]
        lg[(a * 7 + b) % 32000] = 1.0
        return oracle.nucleus_sample(lg, 0.8, 0.95, us[len(seq)])[0]

    prompt = [int(x) for x in corp.tokens[1000:1040]]
    plain = oracle.greedy_decode(next_token, prompt, 48)
    fast, steps = oracle.rest_decode(next_token, prompt, 48, corp.tokens, max_matches=200, cont_len=8, max_nodes=24)
    assert fast == plain
    assert steps < 48


def test_weights_are_the_library_exponential_cut_to_integers():
    """w_i = floor(2^36 * 2^((x_i - x_max) * log2(e) / T)) with the exponential evaluated by the oracle's fixed
    polynomial: against math.exp it may differ by the floor's one unit plus a relative 1e-12."""
    rng = np.random.default_rng(3)
    for T in (1.0, 0.8, 0.7, 0.05, 5.0):
        x = (rng.standard_normal(4000) * rng.choice([0.5, 3.0, 30.0])).astype(np.float32)
        x[7] = -np.inf
        x[11] = x.max()
        w = oracle.nucleus_weights(x, T)
        assert w.dtype == np.uint64 and int(w.max()) == 2 ** 36 and int(w[11]) == 2 ** 36 and int(w[7]) == 0
        t32, top = float(np.float32(T)), float(x.max())
        for i in rng.integers(0, x.size, 600):
            if np.isfinite(x[i]):
                ref = 2.0 ** 36 * math.exp((float(x[i]) - top) / t32)
                assert abs(int(w[i]) - ref) <= 1.0 + 1e-12 * ref, (T, i)
    # a token far below the top one weighs nothing; weights never grow as the logit falls by a visible step
    x = np.array([0.0, -24.0, -25.0, -26.0, -1000.0], dtype=np.float32)
    w = oracle.nucleus_weights(x, 1.0)
    assert int(w[1]) == math.floor(2 ** 36 * math.exp(-24.0)) and int(w[3]) == 0 and int(w[4]) == 0
    assert int(w[2]) == math.floor(2 ** 36 * math.exp(-25.0)) == 0
    # halving the temperature squares the ratios: 2^-3 -> 2^-6 (the logit step is a float32 rounding of 3 ln 2, so the
    # masses are 2^33 and 2^30 only to about 2^-24 of themselves)
    x = np.array([0.0, -3.0 * math.log(2.0)], dtype=np.float32)
    assert abs(int(oracle.nucleus_weights(x, 1.0)[1]) - 2 ** 33) <= 2 ** 33 * 2.0 ** -22
    assert abs(int(oracle.nucleus_weights(x, 0.5)[1]) - 2 ** 30) <= 2 ** 30 * 2.0 ** -21


def test_masses_add_exactly_whatever_the_order():
    """The point of integer masses: any order of summation gives the same totals, so the decisions do not depend on
    how an implementation groups its sums."""
    rng = np.random.default_rng(4)
    x = (rng.standard_normal(131072) * 2).astype(np.float32)
    w = oracle.nucleus_weights(x, 0.8)
    total = int(w.sum())
    assert total < 2 ** 53
    for _ in range(3):
        perm = rng.permutation(w.size)
        assert int(w[perm].reshape(512, 256).sum(axis=1).sum()) == total
        assert float(np.float64(total)) == total                        # and the sum is a float64 exactly
