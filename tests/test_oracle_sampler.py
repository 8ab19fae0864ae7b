"""Pins for the CPU oracle's integer sampler and Philox generator (no GPU)."""
import itertools
import math
import os

import numpy as np
import pytest

from conftest import GOLDEN
from oracle import philox, sampler as S


# ---------------------------------------------------------------- Philox
def test_philox_known_answer_vectors():
    n = 0
    with open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")) as fh:
        for line in fh:
            if line.startswith("#") or not line.strip():
                continue
            v = [int(x, 16) for x in line.split()]
            assert philox.philox4x32(v[:4], v[4:6]) == tuple(v[6:])
            n += 1
    assert n == 3


def test_philox_counter_and_key_matter():
    base = philox.rollout_uniform(3, 10, 4)
    assert base == philox.philox4x32((10, 0, 4, 0), (3, 0))[0]
    assert philox.rollout_uniform((7 << 32) | 3, (5 << 32) | 10, 4) == \
        philox.philox4x32((10, 5, 4, 0), (3, 7))[0]
    words = {philox.rollout_uniform(s, i, t) for s in (3, 4) for i in range(20) for t in range(20)}
    assert len(words) == 800                                  # no collisions among 800 draws
    xs = np.array([philox.rollout_uniform(1, i, 0) for i in range(4000)], dtype=np.float64)
    assert abs(xs.mean() / 2 ** 32 - 0.5) < 0.02              # roughly uniform


# ---------------------------------------------------------------- FIXEXP
def test_fixexp_tracks_exp_and_is_order_independent():
    rng = np.random.default_rng(0)
    logits = (3.0 * rng.standard_normal(5000)).astype(np.float32)
    w = S.fixexp_weights(logits, 1.0)
    d = (logits - logits.max()).astype(np.float64)
    ref = np.exp(d)
    big = ref > 1e-6                                          # truncation to 2^-40 is < 1e-6 there
    rel = np.abs(w / 2.0 ** 40 - ref) / ref
    # fp32 rounding of t = d log2(e) costs up to |t| 2^-24 ln 2 relative: 2e-6 at the cutoff
    assert np.max(rel[big]) < 3e-6 and np.max(rel[d > -1.0]) < 2.5e-7
    assert int(w[np.argmax(logits)]) == 1 << 40               # the arg-max weighs exactly 2^40
    perm = rng.permutation(5000)
    assert sum(int(v) for v in w) == sum(int(v) for v in S.fixexp_weights(logits[perm], 1.0))
    assert np.array_equal(S.fixexp_weights(logits[perm], 1.0), w[perm])


def test_fixexp_cutoff_and_minus_infinity():
    log2e = float(S.LOG2E_F32)
    logits = np.array([0.0, -39.5 / log2e, -40.5 / log2e, -np.inf, -1000.0], dtype=np.float32)
    w = S.fixexp_weights(logits, 1.0)
    assert w[0] == 1 << 40 and w[1] >= 1 and w[2] == 0 and w[3] == 0 and w[4] == 0


def test_temperature_is_one_fp32_multiply():
    logits = np.array([1.0, 2.0, -3.0, 0.5], dtype=np.float32)
    assert np.array_equal(S.fixexp_weights(logits, 0.5), S.fixexp_weights(logits * np.float32(0.5), 1.0))
    assert S.inv_temperature(0.99) == np.float32(1.0) / np.float32(0.99)


# ---------------------------------------------------------------- nucleus
def nucleus_by_threshold(w, top_p):
    """Selection form: largest tau with sum_{w >= tau} w >= theta; all above tau, then ties
    at tau in ascending id until theta is reached."""
    w_int = [int(v) for v in w]
    theta = S.nucleus_threshold(sum(w_int), top_p)
    tau = max(t for t in set(w_int) if t > 0 and sum(v for v in w_int if v >= t) >= theta)
    mask = np.array([v > tau for v in w_int])
    acc = sum(v for v in w_int if v > tau)
    for i, v in enumerate(w_int):
        if acc >= theta:
            break
        if v == tau:
            mask[i] = True
            acc += v
    return mask


@pytest.mark.parametrize("seed", range(6))
def test_nucleus_sorted_form_equals_selection_form(seed):
    rng = np.random.default_rng(seed)
    for _ in range(40):
        v = int(rng.integers(2, 24))
        logits = rng.choice(np.array([-2.0, -1.0, 0.0, 0.5, 1.0, 3.0], dtype=np.float32), v)  # many ties
        if rng.random() < 0.5:
            logits = logits + rng.standard_normal(v).astype(np.float32)
        w = S.fixexp_weights(logits, 1.0)
        top_p = float(rng.choice([0.0, 0.1, 0.5, 0.9, 0.999]))
        a, b = S.nucleus(w, top_p), nucleus_by_threshold(w, top_p)
        assert np.array_equal(a, b)
        # minimal and greedy: reaches theta, would not without its last member, and no
        # outsider outweighs a member
        theta = S.nucleus_threshold(sum(int(x) for x in w), top_p)
        inside = [int(x) for x, k in zip(w, a) if k]
        assert sum(inside) >= theta and sum(inside) - min(inside) < theta
        outside = [int(x) for x, k in zip(w, a) if not k]
        assert not outside or max(outside) <= min(inside)


def test_nucleus_brute_force_smallest_set():
    """On tiny vocabularies the nucleus is a smallest-cardinality set reaching theta."""
    rng = np.random.default_rng(11)
    for _ in range(30):
        logits = rng.standard_normal(6).astype(np.float32)
        w = [int(x) for x in S.fixexp_weights(logits, 1.0)]
        theta = S.nucleus_threshold(sum(w), 0.7)
        best = min(r for r in range(1, 7)
                   for c in itertools.combinations(range(6), r) if sum(w[i] for i in c) >= theta)
        assert int(S.nucleus(np.array(w, dtype=np.uint64), 0.7).sum()) == best


def test_top_p_limits():
    logits = np.array([0.1, 2.0, 2.0, -1.0], dtype=np.float32)
    for x in (0, 123456789, 2 ** 32 - 1):
        assert S.sample(logits, 1.0, 1e-9, x)[0] == 1        # arg-max, lowest id on ties
        assert S.sample(logits, 1.0, 0.0, x)[0] == 1
    w = S.fixexp_weights(logits, 1.0)
    assert S.nucleus(w, 1.0).all()
    assert S.top_p_fixed(0.9) == int(math.floor(float(np.float32(0.9)) * 2 ** 24))


# ---------------------------------------------------------------- draw
def test_draw_edge_uniforms_and_dominant_logit():
    logits = np.array([-1.0, 0.0, 1.0, 0.5, -60.0], dtype=np.float32)
    assert S.sample(logits, 1.0, 1.0, 0)[0] == 0                              # x = 0: lowest id
    assert S.sample(logits, 1.0, 1.0, 2 ** 32 - 1)[0] == 3                    # last token with w > 0
    assert S.sample(logits, 1.0, 0.6, 0)[0] == 2                              # lowest id *in the nucleus*
    hot = np.zeros(50, dtype=np.float32); hot[17] = 100.0
    assert all(S.sample(hot, 1.0, 1.0, x)[0] == 17 for x in (0, 2 ** 31, 2 ** 32 - 1))


def test_draw_is_monotone_inverse_cdf_and_matches_softmax():
    rng = np.random.default_rng(5)
    logits = rng.standard_normal(8).astype(np.float32)
    w = S.fixexp_weights(logits, 1.0)
    mask = S.nucleus(w, 1.0)
    xs = np.sort(rng.integers(0, 2 ** 32, 20000, dtype=np.uint64))
    toks = np.array([S.draw(w, mask, int(x)) for x in xs])
    assert np.all(np.diff(toks) >= 0)                                         # monotone in x
    p = np.exp(logits.astype(np.float64) - logits.max()); p /= p.sum()
    counts = np.bincount(toks, minlength=8)
    chi2 = np.sum((counts - 20000 * p) ** 2 / (20000 * p))
    assert chi2 < 24.3                                                        # 7 dof, p = 0.001
    # exact: the share of the 2^32 words that maps to token j is its weight share
    edges = np.concatenate([[0], np.cumsum([int(v) for v in w])])
    total = int(edges[-1])
    for j in range(8):
        lo = -(-int(edges[j]) * 2 ** 32 // total)           # first x with floor(S x / 2^32) >= edge
        hi = -(-int(edges[j + 1]) * 2 ** 32 // total)
        assert abs((hi - lo) / 2 ** 32 - p[j]) < 1e-6
        if hi > lo:
            assert S.draw(w, mask, lo) == j and S.draw(w, mask, hi - 1) == j


def test_log_prob_is_full_vocab_log_softmax():
    rng = np.random.default_rng(6)
    logits = rng.standard_normal(12).astype(np.float32)
    inv_t = S.inv_temperature(0.8)
    lps = [S.log_prob(logits, inv_t, j) for j in range(12)]
    assert abs(sum(math.exp(v) for v in lps) - 1.0) < 1e-12
    tok, lp = S.sample(logits, inv_t, 0.3, 12345)                            # not renormalised to the nucleus
    assert lp == lps[tok]
    z = (logits * inv_t).astype(np.float64)
    assert abs(lps[3] - (z[3] - np.log(np.sum(np.exp(z))))) < 1e-12
