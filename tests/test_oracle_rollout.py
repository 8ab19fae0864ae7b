"""Pins for the CPU oracle's generation loop (no GPU)."""
import numpy as np
import pytest

import workloads
from oracle import philox, rollout, sampler
from oracle import transformer as T

NANO = workloads.ModelShape("nano", 2, 24, 4, 2, 8, 40, 50, dtype="fp32", rope_theta=10000.0)


def model():
    w = workloads.make_weights(NANO, 1)
    for k in w:
        if w[k].ndim > 1:
            w[k] = (w[k] * np.float32(8.0)).astype(np.float32)
    return T.Model(NANO, w)


def prompts():
    return workloads.make_prompts(3, 4, 9, NANO.vocab, seed=2)


def test_lengths_ids_and_determinism():
    m = model()
    toks, offs = prompts()
    limits = np.array([5, 1, 3, 4, 2, 6], np.int32)
    a = rollout.generate(m, toks, offs, 2, limits, -1, 1.0, 0.9, seed=3)
    b = rollout.generate(m, toks, offs, 2, limits, -1, 1.0, 0.9, seed=3)
    assert [t.sample_id for t in a] == list(range(6))
    assert [len(t.tokens) for t in a] == list(limits)
    assert [t.tokens for t in a] == [t.tokens for t in b]
    c = rollout.generate(m, toks, offs, 2, limits, -1, 1.0, 0.9, seed=4)
    assert [t.tokens for t in a] != [t.tokens for t in c]


def test_first_token_uses_prompt_logits_and_own_uniform():
    m = model()
    toks, offs = prompts()
    tr = rollout.generate(m, toks, offs, 2, np.full(6, 2, np.int32), -1, 1.0, 1.0, seed=9,
                          keep_logits=True)
    for p in range(3):
        last = T.forward_full(m, toks[offs[p]:offs[p + 1]])[-1].astype(np.float32)
        for j in range(2):
            t = tr[p * 2 + j]
            assert np.array_equal(t.logits[0], last)
            tok, lp = sampler.sample(last, np.float32(1.0), 1.0, philox.rollout_uniform(9, t.sample_id, 0))
            assert (tok, lp) == (t.tokens[0], t.logprobs[0])


def test_samples_are_independent_of_batch_composition():
    m = model()
    toks, offs = prompts()
    limits = np.full(6, 4, np.int32)
    whole = rollout.generate(m, toks, offs, 2, limits, -1, 1.0, 0.95, seed=5)
    for p in range(3):
        alone = rollout.generate(m, toks[offs[p]:offs[p + 1]], np.array([0, offs[p + 1] - offs[p]]),
                                 2, limits[:2], -1, 1.0, 0.95, seed=5, first_prompt_index=p)
        assert [t.tokens for t in alone] == [t.tokens for t in whole[2 * p:2 * p + 2]]
        assert [t.sample_id for t in alone] == [2 * p, 2 * p + 1]


def test_eos_terminates_and_is_kept():
    m = model()
    toks, offs = prompts()
    free = rollout.generate(m, toks, offs, 2, np.full(6, 8, np.int32), -1, 1.0, 1.0, seed=6)
    eos = free[0].tokens[2]
    cut = rollout.generate(m, toks, offs, 2, np.full(6, 8, np.int32), eos, 1.0, 1.0, seed=6)
    for f, c in zip(free, cut):
        stop = f.tokens.index(eos) + 1 if eos in f.tokens else len(f.tokens)
        assert c.tokens == f.tokens[:stop]
    assert cut[0].tokens[-1] == eos and len(cut[0].tokens) <= 3


def test_teacher_forced_log_probs_reproduce_rollout_log_probs():
    m = model()
    toks, offs = prompts()
    tr = rollout.generate(m, toks, offs, 2, np.full(6, 5, np.int32), -1, 0.8, 0.9, seed=7)
    for t in tr:
        p = t.sample_id // 2
        seq = np.concatenate([toks[offs[p]:offs[p + 1]], t.tokens])
        lp = T.packed_log_probs(m, seq, [0, len(seq)], temperature=float(np.float32(1) / sampler.inv_temperature(0.8)))
        assert np.allclose(lp[-5:], t.logprobs, atol=1e-6)
    forced = {t.sample_id: t.tokens for t in tr}
    again = rollout.generate(m, toks, offs, 2, np.full(6, 5, np.int32), -1, 0.8, 0.9, seed=99,
                             forced_tokens=forced)
    for a, b in zip(tr, again):
        assert a.tokens == b.tokens and np.allclose(a.logprobs, b.logprobs, atol=1e-12)


def test_batched_slice_emits_expected_count():
    m = model()
    toks, offs = prompts()
    assert rollout.decode_slice_batched(m, toks[:offs[1]], 3, 4, 1.0, 1.0, 1) == 12


@pytest.mark.parametrize("temperature,top_p", [(1.0, 1.0), (0.7, 0.9)])
def test_batched_slice_draws_the_tokens_of_the_per_sample_rollout(temperature, top_p):
    """The function the benchmark times as the CPU baseline stacks the samples' rows into one
    matrix per step; `generate` runs one sample at a time.  Same prompt, same seed, sample ids
    0..n-1, no end-of-sequence token: the two must emit the same tokens."""
    m = model()
    toks, offs = prompts()
    prompt = toks[:offs[1]]
    n, n_new = 4, 9
    got = []
    assert rollout.decode_slice_batched(m, prompt, n, n_new, temperature, top_p, 11, out_tokens=got) == n * n_new
    ref = rollout.generate(m, prompt, [0, len(prompt)], n, np.full(n, n_new, np.int32), -1, temperature, top_p, 11)
    assert [t.sample_id for t in ref] == list(range(n))
    assert got == [t.tokens for t in ref]
    assert len({tuple(g) for g in got}) > 1      # the samples do differ from one another
