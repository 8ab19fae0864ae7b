"""GPU parity of the decode attention that reads a prompt's shared pages once per group of
samples (runtime flag; more than 32 live rows, at least a fifth of the cached positions shared)."""
import numpy as np
import pytest

import workloads
from gpu_util import make_engine, oracle_model, scaled_weights
from oracle import sampler
from oracle import transformer as T
from paper_2506_06122_amd import binding as B

pytestmark = pytest.mark.gpu


def shape_with_heads(n_q, n_kv):
    return workloads.ModelShape(f"small-{n_q}q{n_kv}kv-bf16", 2, 512, n_q, n_kv, 128, 1024, 2048)


def grouped_launches(eng):
    return sum(k["launches"] for k in eng.rollout_kernel_stats() if k["name"].startswith("attn_decode_grouped"))


@pytest.mark.parametrize("n_q,n_kv,n", [(4, 2, 8), (8, 2, 8), (12, 2, 8), (16, 2, 8), (28, 4, 8), (8, 2, 16)],
                         ids=["G2", "G4", "G6", "G8", "G7-4kv", "G4-16-samples"])
def test_grouped_attention_matches_oracle(n_q, n_kv, n):
    """Prompts of 300, 70, 33, 150, 64, 200 and 129 tokens (shared pages: 288, 64, none worth a
    group, 128, 64, 192, 128 positions) with n samples each; after the prefill some samples are
    aborted so that prompts keep 8, 5, 2 and 1 samples (groups of 4, 4+1, 2; a lone sample attends alone).  Four
    teacher-forced decode steps: every logits row and log-prob against the oracle; the grouped
    kernel must have run.  n = 16: a prompt's samples form four groups of 4."""
    shape = shape_with_heads(n_q, n_kv)
    w = scaled_weights(shape, seed=1)
    model = oracle_model(shape, w)
    fwd = T.KVForward(model)
    lens = [300, 70, 33, 150, 64, 200, 129] if n == 8 else [300, 70, 150]
    P, steps = len(lens), 4
    rng = np.random.default_rng(7)
    toks = rng.integers(0, shape.vocab, sum(lens)).astype(np.int32)
    offs = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    forced = rng.integers(0, shape.vocab, (P * n, steps + 1)).astype(np.int32)
    eng = make_engine(shape, w, max_live_samples=64, max_context=512, max_batch_tokens=2048,
                      flags=B.RT_KERNEL_TIMING | B.RT_PROMPT_GROUPS, timing_stride=1)
    ids, tk, lps, fin = eng.rollout_prefill(toks, offs, n, np.full(P * n, steps + 1, np.int32), forced_first=forced[:, 0])
    caches = {}
    for p in range(P):
        c = fwd.new_cache()
        fwd.extend([c], [toks[offs[p]:offs[p + 1]]])
        for j in range(n):
            caches[p * n + j] = c.fork()
    if n == 8:   # prompt 0: 5 left; prompt 1: 2 left; prompt 3: 1 left
        gone = [1, 2, 3] + [8 + j for j in range(2, 8)] + [24 + j for j in range(1, 8)]
        assert eng.rollout_abort(gone) == len(gone)
        for i in gone:
            del caches[i]
    live = sorted(caches)
    assert len(live) > 32 and eng.rollout_live_samples().tolist() == live
    inv_t = np.float32(1.0)
    worst = worst_lp = 0.0
    last = {i: int(forced[i, 0]) for i in live}
    for t in range(1, steps + 1):
        ids2, tk, lps, fin = eng.rollout_decode_step(forced_tokens=forced[live, t])
        assert ids2.tolist() == live
        gpu = eng.rollout_debug_logits()
        ref = fwd.extend([caches[i] for i in live], [[last[i]] for i in live])
        for r, i in enumerate(live):
            worst = max(worst, float(np.max(np.abs(gpu[r] - ref[r][0]))))
            worst_lp = max(worst_lp, abs(sampler.log_prob(ref[r][0].astype(np.float32), inv_t, int(forced[i, t])) - float(lps[r])))
            last[i] = int(forced[i, t])
    launches = grouped_launches(eng)
    print(f"{shape.name} n={n}: max |dlogits| = {worst:.3e}, max |dlogp| = {worst_lp:.3e}; grouped launches {launches}")
    assert worst <= 2e-2 and worst_lp <= 2e-2
    assert launches == steps * shape.n_layers
    eng.close()


def test_grouping_follows_the_live_set():
    """Samples leave one by one: while more than 32 rows are live and enough positions are shared
    the grouped kernel runs, afterwards the plain one; results agree with the oracle throughout
    and a group that shrinks to one member keeps attending correctly."""
    shape = shape_with_heads(8, 2)
    w = scaled_weights(shape, seed=2)
    model = oracle_model(shape, w)
    fwd = T.KVForward(model)
    P, n, steps = 5, 8, 10
    toks, offs = workloads.make_prompts(P, 96, 200, shape.vocab, seed=9)
    rng = np.random.default_rng(10)
    forced = rng.integers(0, shape.vocab, (P * n, steps + 1)).astype(np.int32)
    max_new = rng.integers(2, steps + 2, P * n).astype(np.int32)      # ragged ends
    eng = make_engine(shape, w, max_live_samples=64, max_context=512, max_batch_tokens=2048,
                      flags=B.RT_KERNEL_TIMING | B.RT_PROMPT_GROUPS, timing_stride=1)
    ids, tk, lps, fin = eng.rollout_prefill(toks, offs, n, max_new, forced_first=forced[:, 0])
    caches = {}
    for p in range(P):
        c = fwd.new_cache()
        fwd.extend([c], [toks[offs[p]:offs[p + 1]]])
        for j in range(n):
            caches[p * n + j] = c.fork()
    last = {i: int(forced[i, 0]) for i in caches}
    worst, seen = 0.0, []
    for t in range(1, steps + 1):
        live = eng.rollout_live_samples().tolist()
        if not live:
            break
        before = grouped_launches(eng)
        ids2, tk, lps, fin = eng.rollout_decode_step(forced_tokens=forced[live, t])
        seen.append((len(live), grouped_launches(eng) > before))
        gpu = eng.rollout_debug_logits()
        ref = fwd.extend([caches[i] for i in live], [[last[i]] for i in live])
        for r, i in enumerate(live):
            worst = max(worst, float(np.max(np.abs(gpu[r] - ref[r][0]))))
            last[i] = int(forced[i, t])
    print("rows, grouped:", seen, f"max |dlogits| = {worst:.3e}")
    assert worst <= 2e-2
    assert seen[0] == (40, True) and all(g == (rows > 32) for rows, g in seen)
    assert any(not g for _, g in seen)
    eng.close()
