"""GPU tests of rollout_extend (multi-turn continuation): tokens the model did not generate are
appended to live samples' contexts between decode steps.  The oracle knows only sequences: a
sample's logits after any mix of prefill, decode steps and appended tokens must be those of
the causal model on the concatenated sequence."""
import numpy as np
import pytest

import paper_2506_06122_amd as R
import workloads
from gpu_util import make_engine, oracle_model, scaled_weights
from oracle import philox, sampler
from oracle import transformer as T

pytestmark = pytest.mark.gpu

CASES = {
    "c1-fp32": (workloads.C1_TINY, 1.0, 0, 1e-4),
    "small-bf16": (workloads.SMALL_BF16, 1.0, 0, 2e-2),
    "small-bf16-plain": (workloads.SMALL_BF16, 1.0, 1, 2e-2),
    "small-moe-bf16": (workloads.SMALL_MOE_BF16, 1.5, 2, 2e-2),
}


@pytest.mark.parametrize("name", list(CASES))
def test_multi_turn_extend_matches_oracle(name):
    """3 prompts x 2 samples, teacher-forced.  After decode step 2 three samples get 1, 37 and 80
    appended tokens (one token; a page boundary; more than one 64-row attention tile), after step
    5 two samples get 33 and 5; decoding goes on to 12 response tokens each.  Every logits row -
    prefill, decode steps, the rows after the appended tokens - is compared with the oracle's
    incremental forward on the same token sequence, every log-prob with the oracle's."""
    shape, scale, flags, tol = CASES[name]
    w = scaled_weights(shape, seed=1, scale=scale)
    model = oracle_model(shape, w)
    fwd = T.KVForward(model)
    moe = bool(shape.n_experts)
    P, n, steps = 3, 2, 12
    toks, offs = workloads.make_prompts(P, 5, 70, shape.vocab, seed=61)
    rng = np.random.default_rng(62)
    forced = rng.integers(0, shape.vocab, (P * n, steps)).astype(np.int32)
    eng = make_engine(shape, w, max_live_samples=8, max_context=256, max_batch_tokens=512, flags=flags)
    inv_t = np.float32(1.0)
    worst = worst_lp = 0.0

    def check(gpu_row, ref_row, lp, tok):
        nonlocal worst, worst_lp
        worst = max(worst, float(np.max(np.abs(gpu_row - ref_row))))
        worst_lp = max(worst_lp, abs(sampler.log_prob(ref_row.astype(np.float32), inv_t, int(tok)) - float(lp)))

    def set_routing(rows, pick=None):
        """MoE: the oracle takes the GPU's expert choices of the last forward (all rows, or the
        row range `pick` of them)."""
        if moe:
            routing = eng.rollout_debug_routing(rows)
            model.routing_override = {l: routing[l] if pick is None else routing[l][pick[0]:pick[1]]
                                      for l in range(shape.n_layers)}

    ids, tk, lps, fin = eng.rollout_prefill(toks, offs, n, np.full(P * n, steps + 3, np.int32), forced_first=forced[:, 0])
    gpu = eng.rollout_debug_logits()
    caches = []
    for p in range(P):
        set_routing(int(offs[-1]), (int(offs[p]), int(offs[p + 1])))
        c = fwd.new_cache()
        ref = fwd.extend([c], [toks[offs[p]:offs[p + 1]]])[0][-1]
        for j in range(n):
            check(gpu[p], ref, lps[p * n + j], forced[p * n + j, 0])
            caches.append(c.fork())
    last = forced[:, 0].copy()
    appended = {2: ([0, 3, 4], [1, 37, 80]), 5: ([1, 3], [33, 5])}
    emitted = np.ones(P * n, int)
    for t in range(1, steps):
        ids2, tk, lps, fin = eng.rollout_decode_step(forced_tokens=forced[:, t])
        assert np.array_equal(ids2, ids) and not fin.any()
        gpu = eng.rollout_debug_logits()
        set_routing(P * n)
        ref = fwd.extend(caches, [[int(x)] for x in last])
        for i in range(P * n):
            check(gpu[i], ref[i][0], lps[i], forced[i, t])
        last = forced[:, t].copy()
        emitted += 1
        if t in appended:
            who, lens = appended[t]
            obs = [rng.integers(0, shape.vocab, m).astype(np.int32) for m in lens]
            nxt = rng.integers(0, shape.vocab, len(who)).astype(np.int32)
            o = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
            tk, lps, fin = eng.rollout_extend(ids[who], np.concatenate(obs), o, forced_next=nxt)
            assert np.array_equal(tk, nxt) and not fin.any()
            gpu = eng.rollout_debug_logits()
            assert gpu.shape[0] == len(who)
            row0 = 0
            for k, i in enumerate(who):
                set_routing(int(sum(lens)) + len(who), (row0, row0 + lens[k] + 1))
                row0 += lens[k] + 1
                ref = fwd.extend([caches[i]], [[int(last[i])] + [int(x) for x in obs[k]]])[0][-1]
                check(gpu[k], ref, lps[k], nxt[k])
                last[i] = nxt[k]
                emitted[i] += 1
    model.routing_override = {}
    st = eng.rollout_get_stats()
    print(f"{name}: max |dlogits| = {worst:.3e}, max |dlogp| = {worst_lp:.3e}")
    assert worst <= tol and worst_lp <= tol
    assert st["matrix_core_path"] == int(flags != 1 and shape.dtype == "bf16")
    assert st["live_samples"] == P * n and emitted.max() == steps + 2   # sample 3 took both turns
    eng.close()


def test_extend_draws_with_the_samples_own_stream_and_budget():
    """Free-running: the token after appended tokens is the oracle sampler's choice on the GPU's
    logits row with the Philox word of (seed, sample id, response position) - appended tokens do
    not advance the response position - and the sample ends when its max_new_tokens are out,
    freeing its pages."""
    shape = workloads.C1_TINY
    w = scaled_weights(shape, seed=1)
    toks, offs = workloads.make_prompts(2, 6, 20, shape.vocab, seed=71)
    eng = make_engine(shape, w, max_live_samples=4, max_context=128, max_batch_tokens=128, seed=11)
    ids, tk, lps, fin = eng.rollout_prefill(toks, offs, 1, np.array([4, 3], np.int32), temperature=0.9, top_p=0.8)
    inv_t = sampler.inv_temperature(0.9)
    ids, tk, lps, fin = eng.rollout_decode_step()                          # position 1 of both
    obs = np.arange(40, dtype=np.int32) % shape.vocab
    tk, lps, fin = eng.rollout_extend(ids, np.concatenate([obs, obs[:3]]), np.array([0, 40, 43], np.int32))
    gpu = eng.rollout_debug_logits()
    for k, sid in enumerate(ids):
        want, lp = sampler.sample(gpu[k], inv_t, 0.8, philox.rollout_uniform(11, int(sid), 2))
        assert want == tk[k] and abs(lp - lps[k]) < 1e-4
    assert fin.tolist() == [False, True]                                   # sample 1 had 3 tokens
    assert eng.rollout_live_samples().tolist() == [0]
    ids, tk, lps, fin = eng.rollout_decode_step()                          # position 3: sample 0's last
    gpu = eng.rollout_debug_logits()
    want, lp = sampler.sample(gpu[0], inv_t, 0.8, philox.rollout_uniform(11, 0, 3))
    assert want == tk[0] and fin.tolist() == [True]
    st = eng.rollout_get_stats()
    assert st["live_samples"] == 0 and st["pages_in_use"] == 0
    eng.close()


def test_extend_rejects_without_side_effects():
    shape = workloads.C1_TINY
    w = scaled_weights(shape, seed=1)
    page_bytes = 32 * shape.n_layers * shape.n_kv_heads * shape.head_dim * 2 * 4
    eng = make_engine(shape, w, kv_pool_bytes=4 * page_bytes, max_live_samples=4, max_context=96,
                      max_batch_tokens=128, seed=1)
    toks, offs = workloads.make_prompts(1, 10, 10, shape.vocab, seed=81)
    ids, tk, lps, fin = eng.rollout_prefill(toks, offs, 2, np.array([8, 8], np.int32))
    before = eng.rollout_get_stats()
    one = np.array([0, 1], np.int32)
    with pytest.raises(R.RolloutError):                  # not live
        eng.rollout_extend([7], [1], one)
    with pytest.raises(R.RolloutError):                  # listed twice
        eng.rollout_extend([0, 0], [1, 2], np.array([0, 1, 2], np.int32))
    with pytest.raises(R.RolloutError):                  # nothing to append
        eng.rollout_extend([0], [], np.array([0, 0], np.int32))
    with pytest.raises(R.RolloutError):                  # 10 + 80 + 8 - 1 > max_context
        eng.rollout_extend([0], np.zeros(80, np.int32), np.array([0, 80], np.int32))
    with pytest.raises(R.RolloutError):                  # 2 x 71 rows beyond max_batch_tokens
        eng.rollout_extend([0, 1], np.zeros(140, np.int32), np.array([0, 70, 140], np.int32))
    # pages: each sample holds 1 page (17 positions); 50 more tokens need 2 more each, 2 are free
    assert before["pages_in_use"] == 2 and before["pages_total"] == 4
    with pytest.raises(R.RolloutError):
        eng.rollout_extend([0, 1], np.zeros(100, np.int32), np.array([0, 50, 100], np.int32))
    after = eng.rollout_get_stats()
    clocks = ("prefill_ms", "decode_ms", "extend_ms", "logprobs_ms")   # time was spent in the refused calls
    assert {k: v for k, v in after.items() if k not in clocks} == {k: v for k, v in before.items() if k not in clocks}
    assert after["extend_ms"] > before["extend_ms"]
    tk, lps, fin = eng.rollout_extend([1], np.zeros(20, np.int32), np.array([0, 20], np.int32))   # takes the free page
    assert eng.rollout_get_stats()["pages_in_use"] == before["pages_in_use"] + 1
    ids, tk, lps, fin = eng.rollout_decode_step()
    assert ids.tolist() == [0, 1]
    eng.close()
