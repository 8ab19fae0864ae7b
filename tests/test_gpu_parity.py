"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs.  Tolerances: logits max-abs 1e-4 (fp32 models) / 2e-2 (bf16 models);
sampled token ids bit-exact given the same fp32 logits row and 32-bit word."""
import numpy as np
import pytest

import workloads
from gpu_util import make_engine, oracle_model, scaled_weights, teacher_forced_compare
from oracle import philox, rollout, sampler
from oracle import transformer as T

pytestmark = pytest.mark.gpu

TOL = {"fp32": 1e-4, "bf16": 2e-2}


def test_philox_words_match_oracle():
    import paper_2506_06122_amd as R
    rng = np.random.default_rng(0)
    ids = np.concatenate([np.arange(40), rng.integers(0, 2 ** 62, 60)]).astype(np.int64)
    steps = rng.integers(0, 20000, 100).astype(np.uint32)
    seed = (0xDEADBEEF << 32) | 0x12345678
    got = R.rollout_philox_words(seed, ids, steps)
    want = [philox.rollout_uniform(seed, int(i), int(s)) for i, s in zip(ids, steps)]
    assert got.tolist() == want


@pytest.mark.parametrize("vocab,rows", [(8, 64), (1024, 48), (1000, 16), (151936, 6)])
@pytest.mark.parametrize("top_p", [1.0, 0.9, 0.3, 0.0])
def test_sampler_tokens_bit_exact(vocab, rows, top_p):
    import torch
    import paper_2506_06122_amd as R
    logits = workloads.random_logits(rows, vocab, seed=vocab + int(top_p * 10), scale=2.0)
    if vocab <= 1024:                      # ties at the top, a dominant token, a flat row
        logits[0, :] = 0.0
        logits[1, : vocab // 2] = 1.5
        logits[2, vocab // 3] = 60.0
        logits[3, ::2] = np.float32(-1e30)
    x = workloads.uniform_words(rows, seed=5)
    x[:2] = (0, 2 ** 32 - 1)
    temperature = 0.7
    toks, lps, sums = R.rollout_sample(torch.from_numpy(logits).cuda(), temperature, top_p, x)
    inv_t = sampler.inv_temperature(temperature)
    for r in range(rows):
        w = sampler.fixexp_weights(logits[r], inv_t)
        assert int(sums[r]) == int(np.sum(w, dtype=np.uint64))
        tok, lp = sampler.sample(logits[r], inv_t, top_p, int(x[r]))
        assert int(toks[r]) == tok, f"row {r}"
        assert abs(float(lps[r]) - lp) < 2e-5
    forced = np.arange(rows, dtype=np.int32) % vocab
    toks2, lps2, _ = R.rollout_sample(torch.from_numpy(logits).cuda(), temperature, top_p, x, forced=forced)
    assert np.array_equal(toks2, forced)
    for r in range(0, rows, 5):
        assert abs(float(lps2[r]) - sampler.log_prob(logits[r], inv_t, int(forced[r]))) < 2e-5 \
            or not np.isfinite(sampler.log_prob(logits[r], inv_t, int(forced[r])))


CASES = {
    "c1": (workloads.C1_TINY, 1.0, dict()),
    "tiny-moe-fp32": (workloads.TINY_MOE_FP32, 6.0, dict()),
    "small-bf16": (workloads.SMALL_BF16, 1.0, dict()),
    "small-moe-bf16": (workloads.SMALL_MOE_BF16, 1.5, dict()),
}


@pytest.mark.parametrize("name", list(CASES))
@pytest.mark.parametrize("simple", [True, False], ids=["plain", "fast"])
def test_teacher_forced_logits_match_oracle(name, simple):
    shape, scale, kw = CASES[name]
    w = scaled_weights(shape, seed=1, scale=scale)
    model = oracle_model(shape, w)
    eng = make_engine(shape, w, flags=(1 if simple else 0) | (2 if shape.is_moe else 0), **kw)
    toks, offs = workloads.make_prompts(3, 5, 70, shape.vocab, seed=2)     # ragged, crosses pages
    steps, n = 6, 2
    forced = np.random.default_rng(4).integers(0, shape.vocab, (3 * n, steps)).astype(np.int32)
    worst, worst_lp = teacher_forced_compare(eng, model, toks, offs, n, forced, steps)
    print(f"{name}: max |dlogits| = {worst:.3e}, max |dlogp| = {worst_lp:.3e}")
    assert worst <= TOL[shape.dtype]
    assert worst_lp <= TOL[shape.dtype]
    if shape.is_moe:      # the GPU's expert sets are the top-k of the oracle's own router logits up to rounding
        below, outside = (max(g[i] for g in model.routing_regret) for i in (0, 1))
        print(f"{name}: worst routing gaps = {below:.3e} (k-th logit above the weakest pick), {outside:.3e} "
              f"(best expert left out above the weakest pick) over {len(model.routing_regret)} decisions")
        assert below <= TOL[shape.dtype] and outside <= TOL[shape.dtype]
    st = eng.rollout_get_stats()
    assert st["live_samples"] == 0 and st["pages_in_use"] == 0
    assert st["matrix_core_path"] == int(not simple and shape.dtype == "bf16")
    eng.close()


@pytest.mark.parametrize("n_prompts,n_samples,lo,hi", [(3, 8, 5, 40), (5, 8, 5, 40), (9, 8, 3, 20), (2, 1, 300, 700),
                                                      (1, 3, 1, 1)],
                         ids=["24rows", "40rows", "72rows", "long-context-splits", "one-token-prompt"])
def test_matrix_core_decode_shapes(n_prompts, n_samples, lo, hi):
    """Row-tile configurations of the streamed projections (<=16, <=32, <=64, several row
    blocks) and attention over several KV splits with the merge in the last workgroup."""
    shape = workloads.SMALL_BF16
    w = scaled_weights(shape, seed=1)
    model = oracle_model(shape, w)
    eng = make_engine(shape, w, max_live_samples=80, max_context=1024, max_batch_tokens=2048)
    toks, offs = workloads.make_prompts(n_prompts, lo, hi, shape.vocab, seed=11)
    steps = 4
    forced = np.random.default_rng(5).integers(0, shape.vocab, (n_prompts * n_samples, steps)).astype(np.int32)
    worst, worst_lp = teacher_forced_compare(eng, model, toks, offs, n_samples, forced, steps)
    print(f"max |dlogits| = {worst:.3e}, max |dlogp| = {worst_lp:.3e}")
    assert worst <= TOL["bf16"] and worst_lp <= TOL["bf16"]
    assert eng.rollout_get_stats()["matrix_core_path"] == 1
    eng.close()


@pytest.mark.parametrize("lens,n_samples", [([3000, 1536], 2), ([2900], 40)], ids=["4rows-12-splits", "40rows-4-splits"])
def test_long_contexts_over_many_pages_and_splits(lens, n_samples):
    """Contexts of thousands of positions, as the long tail of configs 3 and 4 has them: prefill
    attention over 94 pages of one sequence, then decode attention with every wavefront walking
    several groups per split and up to twelve splits to merge - on the streamed path (4 rows)
    and on the tile path (40 rows, the prompt's pages shared by all of them)."""
    shape = workloads.SMALL_BF16
    w = scaled_weights(shape, seed=1)
    model = oracle_model(shape, w)
    rng = np.random.default_rng(23)
    toks = rng.integers(0, shape.vocab, sum(lens)).astype(np.int32)
    offs = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    rows = len(lens) * n_samples
    eng = make_engine(shape, w, max_live_samples=rows, max_context=3072, max_batch_tokens=8192)
    steps = 3
    forced = rng.integers(0, shape.vocab, (rows, steps)).astype(np.int32)
    worst, worst_lp = teacher_forced_compare(eng, model, toks, offs, n_samples, forced, steps)
    print(f"contexts {lens} x {n_samples}: max |dlogits| = {worst:.3e}, max |dlogp| = {worst_lp:.3e}")
    assert worst <= TOL["bf16"] and worst_lp <= TOL["bf16"]


def test_decode_attention_of_a_long_tailed_large_batch():
    """128 live rows x 2 KV heads (a workgroup per row and head already fills the chip: no KV
    splits) with contexts of 6 to 700 positions, mean about 60, as a long-tailed rollout leaves
    them: a few workgroups walk hundreds of positions while most are done after one group.
    Every row against the oracle."""
    shape = workloads.SMALL_BF16
    w = scaled_weights(shape, seed=1)
    model = oracle_model(shape, w)
    eng = make_engine(shape, w, max_live_samples=128, max_context=1024, max_batch_tokens=4096)
    rng = np.random.default_rng(23)
    lens = rng.integers(6, 40, 16)
    lens[3], lens[11] = 700, 333
    offs = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    toks = rng.integers(0, shape.vocab, int(offs[-1])).astype(np.int32)
    steps, n = 3, 8
    forced = rng.integers(0, shape.vocab, (16 * n, steps)).astype(np.int32)
    worst, worst_lp = teacher_forced_compare(eng, model, toks, offs, n, forced, steps)
    print(f"long-tailed batch of 128 rows: max |dlogits| = {worst:.3e}, max |dlogp| = {worst_lp:.3e}")
    assert worst <= TOL["bf16"] and worst_lp <= TOL["bf16"]
    eng.close()


@pytest.mark.parametrize("simple", [False, True], ids=["fast", "plain"])
def test_c2_shape_slice_matches_oracle(simple):
    """The benchmark's model shape (28 layers, hidden 1536, 12/2 heads, FFN 8960, vocab 151936,
    bf16) on a slice the oracle can afford: 2 prompts x 2 samples, 4 teacher-forced steps."""
    shape = workloads.C2_1P5B
    w = workloads.make_weights(shape, seed=1)
    model = oracle_model(shape, w)
    eng = make_engine(shape, w, kv_pool_bytes=1 << 30, max_live_samples=8, max_context=512, max_batch_tokens=512,
                      flags=int(simple))
    toks, offs = workloads.make_prompts(2, 40, 90, shape.vocab, seed=12)
    forced = np.random.default_rng(6).integers(0, shape.vocab, (4, 4)).astype(np.int32)
    worst, worst_lp = teacher_forced_compare(eng, model, toks, offs, 2, forced, 4)
    print(f"c2 shape: max |dlogits| = {worst:.3e}, max |dlogp| = {worst_lp:.3e}")
    assert eng.rollout_get_stats()["matrix_core_path"] == int(not simple)
    assert worst <= TOL["bf16"] and worst_lp <= TOL["bf16"]
    eng.close()


def full_batch_case(shape, load, picks, max_batch_tokens=16384):
    """The whole batch of a benchmark configuration as bench.py launches it, teacher-forced for 3
    steps, checked two ways.  (1) Rows the oracle can afford, computed one by one: the prompts
    `picks` and one sample of each through the decode steps.  (2) A property that holds at any
    size, on all rows: a row's result does not depend on where it sits in the batch, so samples
    of one prompt that are fed the same tokens must produce bit-identical logits, and every
    returned log-prob must be the log-softmax of its own logits row.  Returns the largest
    logits error on the oracle's rows."""
    w = workloads.make_weights(shape, seed=1)
    P, n = load.n_prompts, load.n_samples
    toks, offs = load.prompt_tokens, load.prompt_offsets
    lens = np.diff(offs)
    steps = 3
    rng = np.random.default_rng(17)
    forced = rng.integers(0, shape.vocab, (P * n, steps)).astype(np.int32)
    for p in range(P):  # samples 0..3 of a prompt share their tokens
        forced[p * n + 1: p * n + 4] = forced[p * n]
    kv_per_token = 2 * shape.n_layers * shape.n_kv_heads * shape.head_dim * 2
    need = int(lens.sum()) + P * n * (steps + 64)
    eng = make_engine(shape, w, kv_pool_bytes=max(need * kv_per_token, 1 << 30), max_live_samples=P * n,
                      max_context=int(lens.max()) + steps + 1, max_batch_tokens=max_batch_tokens)
    ids, tk, lps, fin = eng.rollout_prefill(toks, offs, n, np.full(P * n, steps, np.int32), forced_first=forced[:, 0])
    assert len(ids) == P * n and np.array_equal(tk, forced[:, 0])
    model = oracle_model(shape, w)
    fwd = T.KVForward(model)
    gpu = eng.rollout_debug_logits()
    caches, worst = {}, 0.0
    for p in picks:
        c = fwd.new_cache()
        ref = fwd.extend([c], [toks[offs[p]:offs[p + 1]]])[0][-1]
        worst = max(worst, float(np.max(np.abs(gpu[p] - ref))))
        caches[p] = c
    inv_t = np.float32(1.0)
    for i in range(0, P * n, 7):
        assert abs(sampler.log_prob(gpu[i // n], inv_t, int(forced[i, 0])) - float(lps[i])) < 2e-5
    for t in range(1, steps):
        ids2, tk, lps, fin = eng.rollout_decode_step(forced_tokens=forced[:, t])
        assert np.array_equal(ids2, ids) and np.array_equal(tk, forced[:, t])
        gpu = eng.rollout_debug_logits()
        assert gpu.shape == (P * n, shape.vocab)
        for p in range(P):
            for j in range(1, 4):
                assert np.array_equal(gpu[p * n], gpu[p * n + j]), f"prompt {p}: row {j} differs from row 0"
        for i in range(0, P * n, 7):
            assert abs(sampler.log_prob(gpu[i], inv_t, int(forced[i, t])) - float(lps[i])) < 2e-5
        for p in picks:  # sample 5 of the prompt (its own tokens), oracle one row at a time
            i = p * n + 5
            if t == 1:
                caches[p] = caches[p].fork()
            ref = fwd.extend([caches[p]], [[int(forced[i, t - 1])]])[0][0]
            worst = max(worst, float(np.max(np.abs(gpu[i] - ref))))
    assert eng.rollout_get_stats()["matrix_core_path"] == 1
    eng.close()
    return worst


def test_c2_full_batch_sampled_rows_and_row_invariance():
    """The headline job as it is launched in the benchmark - the full 1.5B-shaped model, all 32
    prompts x 8 samples (256 live rows: packed prefill of about 9k prompt tokens, 64 x 128 tile
    projections, one-split attention); the oracle takes the shortest and the longest prompt."""
    load = workloads.load_c2()
    lens = np.diff(load.prompt_offsets)
    worst = full_batch_case(workloads.C2_1P5B, load, [int(np.argmin(lens)), int(np.argmax(lens))])
    print(f"c2 full batch: max |dlogits| on the oracle's rows = {worst:.3e}")
    assert worst <= TOL["bf16"]


def test_c3_full_batch_sampled_rows_and_row_invariance():
    """Config 3 as it is launched in the benchmark - the 7B-shaped model at its full depth, all
    64 prompts x 8 samples (512 live rows, about 37k prompt tokens prefilled in chunks of at most
    16384 rows); the oracle (57 GB of widened weights) takes the shortest prompt."""
    load = workloads.load_c3()
    lens = np.diff(load.prompt_offsets)
    worst = full_batch_case(workloads.C3_7B, load, [int(np.argmin(lens))])
    print(f"c3 full batch: max |dlogits| on the oracle's rows = {worst:.3e}")
    assert worst <= TOL["bf16"]


@pytest.mark.parametrize("which", ["c3-dense", "c4-moe"])
def test_large_config_shapes_reduced_depth(which):
    """Every matrix shape of configs 3/5 (hidden 3584, 28/4 heads, FFN 18944, vocab 152064) and
    of config 4 (hidden 2048, 32/4 heads, 128 experts, top-8, expert FFN 768), with the layer
    count cut (4 and 2 layers) so that the fp64 oracle fits in host memory: 2 prompts x 2
    samples, 3 teacher-forced steps."""
    import dataclasses
    if which == "c3-dense":
        shape = dataclasses.replace(workloads.C3_7B, n_layers=4, name="qwen2.5-7b-shape-4-layers")
    else:
        shape = dataclasses.replace(workloads.C4_30B_A3B, n_layers=2, name="qwen3-30b-a3b-shape-2-layers")
    w = workloads.make_weights(shape, seed=1)
    model = oracle_model(shape, w)
    eng = make_engine(shape, w, kv_pool_bytes=1 << 30, max_live_samples=8, max_context=512, max_batch_tokens=512,
                      flags=2 if shape.is_moe else 0)
    toks, offs = workloads.make_prompts(2, 40, 90, shape.vocab, seed=14)
    forced = np.random.default_rng(8).integers(0, shape.vocab, (4, 3)).astype(np.int32)
    worst, worst_lp = teacher_forced_compare(eng, model, toks, offs, 2, forced, 3)
    print(f"{shape.name}: max |dlogits| = {worst:.3e}, max |dlogp| = {worst_lp:.3e}")
    assert eng.rollout_get_stats()["matrix_core_path"] == 1
    assert worst <= TOL["bf16"] and worst_lp <= TOL["bf16"]
    eng.close()


def test_c3_full_depth_slice_matches_oracle():
    """Configs 3 and 5's model at its full depth - 28 layers, hidden 3584, 28/4 heads, FFN 18944,
    vocab 152064 - on a slice the fp64 oracle can afford on the GPU host (57 GB of widened
    weights, about 2 x 10^12 flop): 2 prompts x 2 samples, 3 teacher-forced steps.  This is the
    depth at which rounding has accumulated most: the 16-bit KV cache alone leaves 1.3e-2 here
    (4 layers of the same shape: 5e-3)."""
    shape = workloads.C3_7B
    w = workloads.make_weights(shape, seed=1)
    model = oracle_model(shape, w)
    eng = make_engine(shape, w, kv_pool_bytes=1 << 30, max_live_samples=8, max_context=512, max_batch_tokens=512)
    toks, offs = workloads.make_prompts(2, 40, 90, shape.vocab, seed=14)
    forced = np.random.default_rng(8).integers(0, shape.vocab, (4, 3)).astype(np.int32)
    worst, worst_lp = teacher_forced_compare(eng, model, toks, offs, 2, forced, 3)
    print(f"{shape.name}, all {shape.n_layers} layers: max |dlogits| = {worst:.3e}, max |dlogp| = {worst_lp:.3e}")
    assert eng.rollout_get_stats()["matrix_core_path"] == 1
    assert worst <= TOL["bf16"] and worst_lp <= TOL["bf16"]
    eng.close()


def test_c4_shape_many_rows_four_layers():
    """Config 4's mixture-of-experts shape - hidden 2048, 32/4 heads, 128 experts, top-8, expert FFN
    768, vocab 151936 - with 4 of its 48 layers (the fp64 oracle of more does not fit a test), at
    a batch the grouped expert projections see in the benchmark: 9 prompts x 8 samples = 72 live
    rows (about 4.5 picks per expert and step, most experts touched), 3 teacher-forced steps;
    the oracle computes with the GPU's recorded expert sets, which must be the top-8 of its own
    router logits up to the tolerance."""
    import dataclasses
    shape = dataclasses.replace(workloads.C4_30B_A3B, n_layers=4, name="qwen3-30b-a3b-shape-4-layers")
    w = workloads.make_weights(shape, seed=1)
    model = oracle_model(shape, w)
    eng = make_engine(shape, w, kv_pool_bytes=1 << 30, max_live_samples=80, max_context=256, max_batch_tokens=1024,
                      flags=2)
    P, n, steps = 9, 8, 3
    toks, offs = workloads.make_prompts(P, 20, 60, shape.vocab, seed=15)
    forced = np.random.default_rng(9).integers(0, shape.vocab, (P * n, steps)).astype(np.int32)
    worst, worst_lp = teacher_forced_compare(eng, model, toks, offs, n, forced, steps)
    below, outside = (max(g[i] for g in model.routing_regret) for i in (0, 1))
    print(f"{shape.name}, {P * n} rows: max |dlogits| = {worst:.3e}, max |dlogp| = {worst_lp:.3e}, routing gaps "
          f"{below:.3e} / {outside:.3e} over {len(model.routing_regret)} decisions")
    assert eng.rollout_get_stats()["matrix_core_path"] == 1
    assert worst <= TOL["bf16"] and worst_lp <= TOL["bf16"] and below <= TOL["bf16"] and outside <= TOL["bf16"]
    eng.close()


def test_c4_shape_512_live_rows_sampled():
    """Config 4's batch size on its matrix shapes (128 experts, top-8; 4 of the 48 layers): 64
    prompts x 8 samples = 512 live rows, 32 picks per expert and step on average, every expert's
    row blocks in use.  The oracle follows three prompts and one sample of each through the
    decode steps, computing with the expert sets the GPU recorded for exactly those rows - which
    must be valid top-8 sets of its own router logits."""
    import dataclasses
    shape = dataclasses.replace(workloads.C4_30B_A3B, n_layers=4, name="qwen3-30b-a3b-shape-4-layers")
    w = workloads.make_weights(shape, seed=1)
    model = oracle_model(shape, w)
    P, n, steps = 64, 8, 3
    eng = make_engine(shape, w, kv_pool_bytes=2 << 30, max_live_samples=P * n, max_context=128, max_batch_tokens=4096,
                      flags=2)
    toks, offs = workloads.make_prompts(P, 20, 60, shape.vocab, seed=16)
    forced = np.random.default_rng(10).integers(0, shape.vocab, (P * n, steps)).astype(np.int32)
    ids, tk, lps, fin = eng.rollout_prefill(toks, offs, n, np.full(P * n, steps, np.int32), forced_first=forced[:, 0])
    assert len(ids) == P * n and np.array_equal(tk, forced[:, 0])
    gpu = eng.rollout_debug_logits()
    routing = eng.rollout_debug_routing(int(offs[-1]))
    fwd = T.KVForward(model)
    picks, caches, worst = [0, 31, 63], {}, 0.0
    for p in picks:
        model.routing_override = {l: routing[l][offs[p]:offs[p + 1]] for l in range(shape.n_layers)}
        c = fwd.new_cache()
        ref = fwd.extend([c], [toks[offs[p]:offs[p + 1]]])[0][-1]
        worst = max(worst, float(np.max(np.abs(gpu[p] - ref))))
        caches[p] = c.fork()
    for t in range(1, steps):
        ids2, tk, lps, fin = eng.rollout_decode_step(forced_tokens=forced[:, t])
        assert np.array_equal(ids2, ids)
        gpu = eng.rollout_debug_logits()
        routing = eng.rollout_debug_routing(P * n)
        assert routing.shape == (shape.n_layers, P * n, shape.top_k)
        for layer in range(shape.n_layers):   # every row picked 8 different experts
            assert all(len(set(row)) == shape.top_k for row in routing[layer][::37].tolist())
        for p in picks:
            i = p * n + 3
            model.routing_override = {l: routing[l][[i]] for l in range(shape.n_layers)}
            ref = fwd.extend([caches[p]], [[int(forced[i, t - 1])]])[0][0]
            worst = max(worst, float(np.max(np.abs(gpu[i] - ref))))
    below, outside = (max(g[i] for g in model.routing_regret) for i in (0, 1))
    print(f"{shape.name}, {P * n} live rows: max |dlogits| on the oracle's rows = {worst:.3e}, routing gaps "
          f"{below:.3e} / {outside:.3e} over {len(model.routing_regret)} decisions")
    assert eng.rollout_get_stats()["matrix_core_path"] == 1
    assert worst <= TOL["bf16"] and below <= TOL["bf16"] and outside <= TOL["bf16"]
    eng.close()


@pytest.mark.parametrize("n_prompts,n_samples,lo,hi", [(1, 2, 3, 9), (6, 8, 30, 200)], ids=["few-rows", "many-rows"])
def test_matrix_core_moe_row_blocks(n_prompts, n_samples, lo, hi):
    """Grouped expert projections: a handful of rows (most experts untouched, one row each) and
    hundreds of prompt rows / 48 decode rows (several 64-row blocks per expert)."""
    shape = workloads.SMALL_MOE_BF16
    w = scaled_weights(shape, seed=1, scale=1.5)
    model = oracle_model(shape, w)
    eng = make_engine(shape, w, max_live_samples=64, max_context=512, max_batch_tokens=2048, flags=2)
    toks, offs = workloads.make_prompts(n_prompts, lo, hi, shape.vocab, seed=21)
    steps = 3
    forced = np.random.default_rng(9).integers(0, shape.vocab, (n_prompts * n_samples, steps)).astype(np.int32)
    worst, worst_lp = teacher_forced_compare(eng, model, toks, offs, n_samples, forced, steps)
    below, outside = (max(g[i] for g in model.routing_regret) for i in (0, 1))
    print(f"max |dlogits| = {worst:.3e}, max |dlogp| = {worst_lp:.3e}, routing gaps {below:.3e} / {outside:.3e}")
    assert worst <= TOL["bf16"] and worst_lp <= TOL["bf16"] and below <= TOL["bf16"] and outside <= TOL["bf16"]
    assert eng.rollout_get_stats()["matrix_core_path"] == 1
    eng.close()


@pytest.mark.parametrize("name,simple", [("tiny-moe-fp32", True), ("tiny-moe-fp32", False), ("small-moe-bf16", False)],
                         ids=["fp32-plain", "fp32-default", "bf16-fast"])
def test_moe_routing_decided_independently(name, simple):
    """The GPU and the oracle route on their own: no expert set is handed from one to the
    other.  The GPU's recorded sets must be the oracle's `route()` result wherever the oracle's
    own gap between the k-th and the (k+1)-th router logit exceeds what rounding can move
    (1e-5 for the fp32 model, the logits tolerance for the bf16 model); for the fp32 model the
    logits of the two independent runs must agree as well (a routing difference on a near-tie
    of that size moves them by less than the tolerance).  For the bf16 model only the first
    layer is compared: a near-tie there that the two sides resolve differently (legitimately, at
    that margin) gives every later layer different inputs, so later decisions no longer refer to
    the same logits."""
    shape, scale, kw = CASES[name]
    w = scaled_weights(shape, seed=1, scale=scale)
    model = oracle_model(shape, w)
    model.routing_trace = []
    eng = make_engine(shape, w, flags=(1 if simple else 0) | 2, **kw)
    P, n, steps, k = 3, 2, 5, shape.top_k
    toks, offs = workloads.make_prompts(P, 5, 70, shape.vocab, seed=2)
    forced = np.random.default_rng(4).integers(0, shape.vocab, (P * n, steps)).astype(np.int32)
    margin = 1e-5 if shape.dtype == "fp32" else TOL["bf16"]
    fwd = T.KVForward(model)

    def compare_routing(gpu_sets, n_rows):
        """gpu_sets [layers][rows][k] against the oracle's trace of the forward it just ran."""
        trace, decided, near = model.routing_trace, 0, 0
        assert len(trace) == shape.n_layers * n_rows
        for i, (layer, r, experts) in enumerate(trace):
            row = i % n_rows
            assert layer == i // n_rows
            srt = np.sort(r)[::-1]
            got = set(int(e) for e in gpu_sets[layer][row])
            assert len(got) == k
            if shape.dtype != "fp32" and layer > 0:
                continue
            if srt[k - 1] - srt[k] > margin:
                assert got == set(int(e) for e in experts), f"layer {layer} row {row}"
                decided += 1
            else:
                near += 1
        model.routing_trace = []
        return decided, near

    ids, tk, lps, fin = eng.rollout_prefill(toks, offs, n, np.full(P * n, steps, np.int32), forced_first=forced[:, 0])
    gpu_logits = eng.rollout_debug_logits()
    routing = eng.rollout_debug_routing(int(offs[-1]))
    caches, worst, decided, near = [], 0.0, 0, 0
    for p in range(P):
        prefix = fwd.new_cache()
        ref = fwd.extend([prefix], [toks[offs[p]:offs[p + 1]]])[0][-1]
        d, m = compare_routing([routing[l][offs[p]:offs[p + 1]] for l in range(shape.n_layers)], int(offs[p + 1] - offs[p]))
        decided, near = decided + d, near + m
        worst = max(worst, float(np.max(np.abs(gpu_logits[p] - ref))))
        caches += [prefix.fork() for _ in range(n)]
    for t in range(1, steps):
        eng.rollout_decode_step(forced_tokens=forced[:, t])
        gpu_logits = eng.rollout_debug_logits()
        routing = eng.rollout_debug_routing(P * n)
        ref = fwd.extend(caches, [[int(x)] for x in forced[:, t - 1]])
        d, m = compare_routing(routing, P * n)
        decided, near = decided + d, near + m
        worst = max([worst] + [float(np.max(np.abs(gpu_logits[i] - ref[i][0]))) for i in range(P * n)])
    print(f"{name}: {decided} routing decisions identical, {near} within the margin and not compared; "
          f"max |dlogits| without any override = {worst:.3e}")
    assert decided > (10 if shape.dtype == "fp32" else 4) * max(near, 1)   # most decisions are clear of the margin
    if shape.dtype == "fp32":
        assert worst <= TOL["fp32"]
    eng.close()


def test_c1_full_config_rollout():
    """Config 1 as stated: 4 prompts x 2 samples, prompt length 32, exactly 32 new tokens,
    temperature 1.0, top-p 0.9, Philox uniforms.  Free-running on the GPU; every emitted
    token must be the oracle sampler's choice on the GPU's own logits row."""
    shape = workloads.C1_TINY
    w = scaled_weights(shape, seed=1)
    load = workloads.load_c1()
    eng = make_engine(shape, w, seed=load.sampler_seed)
    inv_t = sampler.inv_temperature(load.temperature)
    ids, toks, lps, fin = eng.rollout_prefill(load.prompt_tokens, load.prompt_offsets, load.n_samples,
                                              load.max_new_tokens, temperature=load.temperature, top_p=load.top_p)
    assert ids.tolist() == list(range(8)) and not fin.any()
    logits = eng.rollout_debug_logits()
    seqs = {int(i): [int(t)] for i, t in zip(ids, toks)}
    for k, sid in enumerate(ids):
        tok, lp = sampler.sample(logits[k // 2], inv_t, load.top_p, philox.rollout_uniform(3, int(sid), 0))
        assert tok == toks[k] and abs(lp - lps[k]) < 1e-4
    for t in range(1, 32):
        ids, toks, lps, fin = eng.rollout_decode_step()
        assert len(ids) == 8 and fin.all() == (t == 31)
        logits = eng.rollout_debug_logits()
        for k, sid in enumerate(ids):
            tok, lp = sampler.sample(logits[k], inv_t, load.top_p, philox.rollout_uniform(3, int(sid), t))
            assert tok == toks[k] and abs(lp - lps[k]) < 1e-4
            seqs[int(sid)].append(int(toks[k]))
    assert len(eng.rollout_decode_step()[0]) == 0
    # the oracle, teacher-forced on the GPU's tokens, sees the same logits within 1e-4 ...
    model = oracle_model(shape, w)
    ref = rollout.generate(model, load.prompt_tokens, load.prompt_offsets, 2, load.max_new_tokens, -1,
                           load.temperature, load.top_p, 3, keep_logits=True, forced_tokens=seqs)
    # ... and running free it draws the very same tokens (fp32 logits differ by ~1e-6)
    free = rollout.generate(model, load.prompt_tokens, load.prompt_offsets, 2, load.max_new_tokens, -1,
                            load.temperature, load.top_p, 3)
    same = sum(f.tokens == seqs[f.sample_id] for f in free)
    print(f"free-running oracle reproduced {same}/8 GPU trajectories")
    assert same >= 7
    eng.close()


def test_teacher_forced_logprob_pass_matches_oracle():
    cases = ((workloads.C1_TINY, 1.0, 96, (7, 1, 90)), (workloads.SMALL_BF16, 1.0, 96, (7, 1, 90)),
             (workloads.TINY_MOE_FP32, 6.0, 96, (7, 1, 90)), (workloads.SMALL_MOE_BF16, 1.5, 96, (7, 1, 90)),
             # one chunk of about 2000 rows: the widest tile configuration of the fused log-sum-exp
             (workloads.SMALL_BF16, 1.0, 2048, (12, 40, 300)))
    for shape, scale, chunk, (n_seqs, lo, hi) in cases:
        w = scaled_weights(shape, seed=1, scale=scale)
        model = oracle_model(shape, w)
        eng = make_engine(shape, w, max_batch_tokens=chunk)                   # 96 forces several chunks
        toks, cu = workloads.packed_sequences(n_seqs, lo, hi, shape.vocab, seed=6)
        got = eng.rollout_logprobs(toks, cu, temperature=0.8)
        want = T.packed_log_probs(model, toks, cu, temperature=float(np.float32(1) / sampler.inv_temperature(0.8)))
        err = float(np.max(np.abs(got - want)))
        print(f"{shape.name}: max |dlogp| = {err:.3e}")
        assert err <= TOL[shape.dtype]
        assert all(got[a] == 0.0 for a in cu[:-1])
        assert eng.rollout_get_stats()["pages_in_use"] == 0
        eng.close()


def test_logprob_pass_at_config5_logits_shape():
    """The teacher-forced pass as config 5 runs it - the 7B matrix shapes, hidden 3584, the full
    152064-entry vocabulary (1188 column parts per row in the fused log-sum-exp), chunks of more
    than 512 packed rows (the 64 x 256 tile plan) - with the layer count cut to 2 so that the
    fp64 oracle fits: 8 sequences of 1 to 320 tokens in three chunks of up to 640 rows."""
    import dataclasses
    shape = dataclasses.replace(workloads.C3_7B, n_layers=2, name="qwen2.5-7b-shape-2-layers")
    w = workloads.make_weights(shape, seed=1)
    model = oracle_model(shape, w)
    eng = make_engine(shape, w, kv_pool_bytes=64 << 20, max_live_samples=8, max_context=512, max_batch_tokens=640)
    lens = [200, 150, 260, 300, 320, 17, 1, 280]          # chunks: 610 rows, 620 rows, 298 rows
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    toks = np.random.Generator(np.random.Philox(key=[31, 5])).integers(0, shape.vocab, int(cu[-1])).astype(np.int32)
    got = eng.rollout_logprobs(toks, cu, temperature=1.0)
    assert eng.rollout_get_stats()["matrix_core_path"] == 1 and eng.rollout_get_stats()["pages_in_use"] == 0
    eng.close()
    want = T.packed_log_probs(model, toks, cu, temperature=1.0)
    err = float(np.max(np.abs(got - want)))
    print(f"{shape.name}, vocab {shape.vocab}, {int(cu[-1])} rows in 3 chunks: max |dlogp| = {err:.3e}; "
          f"mean log-prob {want[want != 0].mean():.3f}")
    assert err <= TOL["bf16"]
    assert all(got[a] == 0.0 for a in cu[:-1])
    # the same sequence alone (300 rows: the 64 x 128 tile plan and other split-K counts) agrees with
    # its rows inside the 620-row chunk far inside the tolerance: what differs is summation order
    eng = make_engine(shape, w, kv_pool_bytes=64 << 20, max_live_samples=8, max_context=512, max_batch_tokens=640)
    alone = eng.rollout_logprobs(toks[cu[3]:cu[4]], [0, lens[3]], temperature=1.0)
    eng.close()
    diff = float(np.max(np.abs(alone - got[cu[3]:cu[4]])))
    print(f"alone vs inside a chunk: max |dlogp| = {diff:.3e}")
    assert diff <= 2e-3


def test_logprob_pass_at_config5_full_size():
    """The teacher-forced pass in the launch configuration the benchmark times: the 7B-shaped
    model at its full depth, 16384-row chunks, sequences of config 5's lengths (up to 8192
    tokens) packed with two short ones the fp64 oracle can afford at this depth.  The oracle
    checks the short sequences; for the rest, properties that hold at any size: every log-prob is
    finite and not positive, a sequence's first position reads 0, and a long sequence run alone
    (another chunk composition, another tile plan for its last rows) agrees with its rows inside
    the batch far inside the tolerance."""
    shape = workloads.C3_7B
    w = workloads.make_weights(shape, seed=1)
    kv_per_token = 2 * shape.n_layers * shape.n_kv_heads * shape.head_dim * 2
    kw = dict(kv_pool_bytes=(16384 + 8192 + 64 * 32) * kv_per_token, max_live_samples=8, max_context=8192,
              max_batch_tokens=16384)
    lens = [8192, 6000, 4500, 150, 3000, 120]          # chunks: 14192 rows, 7770 rows
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    toks = np.random.Generator(np.random.Philox(key=[33, 5])).integers(0, shape.vocab, int(cu[-1])).astype(np.int32)
    eng = make_engine(shape, w, **kw)
    got = eng.rollout_logprobs(toks, cu, temperature=1.0)
    assert eng.rollout_get_stats()["matrix_core_path"] == 1 and eng.rollout_get_stats()["pages_in_use"] == 0
    alone = eng.rollout_logprobs(toks[cu[2]:cu[3]], [0, lens[2]], temperature=1.0)
    eng.close()
    assert np.all(np.isfinite(got)) and np.all(got <= 0.0) and all(got[a] == 0.0 for a in cu[:-1])
    diff = float(np.max(np.abs(alone - got[cu[2]:cu[3]])))
    model = oracle_model(shape, w)
    err = 0.0
    for s in (3, 5):
        want = T.packed_log_probs(model, toks[cu[s]:cu[s + 1]], [0, lens[s]], temperature=1.0)
        err = max(err, float(np.max(np.abs(got[cu[s]:cu[s + 1]] - want))))
    print(f"{shape.name}, all {shape.n_layers} layers, {int(cu[-1])} rows in 2 chunks: max |dlogp| = {err:.3e} on the "
          f"oracle's sequences; 4500 tokens alone vs inside the batch: {diff:.3e}")
    assert err <= TOL["bf16"]
    assert diff <= 5e-3


def test_lifecycle_add_abort_eos_and_batch_invariance():
    shape = workloads.C1_TINY
    w = scaled_weights(shape, seed=1)
    toks, offs = workloads.make_prompts(3, 20, 80, shape.vocab, seed=8)
    limits = np.array([9, 1, 5, 12, 7, 3], np.int32)

    def run_together():
        eng = make_engine(shape, w)
        out = {}
        ids, t, lp, fin = eng.rollout_prefill(toks, offs, 2, limits, top_p=0.95)
        assert fin.tolist() == [False, True, False, False, False, False]
        for i, tk in zip(ids, t):
            out[int(i)] = [int(tk)]
        while True:
            ids, t, lp, fin = eng.rollout_decode_step()
            if not len(ids):
                break
            for i, tk in zip(ids, t):
                out[int(i)].append(int(tk))
        st = eng.rollout_get_stats()
        assert st["pages_in_use"] == 0 and st["samples_finished"] == 6 and st["tokens_emitted"] == limits.sum()
        eng.close()
        return out

    def run_staggered():
        """Same prompts admitted one at a time, in reverse order of arrival on the device
        (different physical pages, different batch composition at every step)."""
        eng = make_engine(shape, w)
        out = {}
        pending = [0, 1, 2]
        # prompt counters are assigned in call order, so admit 0, 1, 2 but interleave decode steps
        step = 0
        while pending or len(eng.rollout_live_samples()):
            if pending and step % 3 == 0:
                p = pending.pop(0)
                ids, t, lp, fin = eng.rollout_prefill(toks[offs[p]:offs[p + 1]], [0, offs[p + 1] - offs[p]], 2,
                                                      limits[2 * p:2 * p + 2], top_p=0.95)
                for i, tk in zip(ids, t):
                    out[int(i)] = [int(tk)]
            ids, t, lp, fin = eng.rollout_decode_step()
            for i, tk in zip(ids, t):
                out[int(i)].append(int(tk))
            step += 1
        assert eng.rollout_get_stats()["pages_in_use"] == 0
        eng.close()
        return out

    a, b = run_together(), run_staggered()
    assert [len(a[i]) for i in range(6)] == limits.tolist()
    assert a == b                                            # schedule-independent samples

    # abort frees exactly that sample's pages; the survivors are unaffected
    eng = make_engine(shape, w)
    ids, t, lp, fin = eng.rollout_prefill(toks, offs, 2, limits, top_p=0.95)
    before = eng.rollout_get_stats()["pages_in_use"]
    assert eng.rollout_abort([3, 1, 999]) == 1               # 1 already finished, 999 unknown
    after = eng.rollout_get_stats()
    assert after["pages_in_use"] < before and after["samples_aborted"] == 1
    out = {int(i): [int(tk)] for i, tk in zip(ids, t)}
    while len(eng.rollout_live_samples()):
        ids, t, lp, fin = eng.rollout_decode_step()
        assert 3 not in ids
        for i, tk in zip(ids, t):
            out[int(i)].append(int(tk))
    for i in (0, 2, 4, 5):
        assert out[i] == a[i]
    assert eng.rollout_get_stats()["pages_in_use"] == 0

    # EOS: the token is reported, the sample ends, the others go on
    eos = a[0][3]
    ids, t, lp, fin = eng.rollout_prefill(toks, offs, 2, limits, eos_id=eos, top_p=0.95)
    got = {int(i): [int(tk)] for i, tk in zip(ids, t)}
    while len(eng.rollout_live_samples()):
        ids, t, lp, fin = eng.rollout_decode_step()
        for i, tk, f in zip(ids, t, fin):
            got[int(i)].append(int(tk))
            assert bool(f) == (int(tk) == eos or len(got[int(i)]) == limits[int(i) - 6])
    # these are prompts 3..5 for the context (ids 6..11) and draw from their own streams
    assert sorted(got) == list(range(6, 12))
    assert eng.rollout_get_stats()["pages_in_use"] == 0
    eng.close()


def test_admission_control_rejects_without_side_effects():
    import paper_2506_06122_amd as R
    shape = workloads.C1_TINY
    w = scaled_weights(shape, seed=1)
    page_bytes = shape.n_layers * shape.n_kv_heads * 2 * 32 * shape.head_dim * 4
    eng = make_engine(shape, w, kv_pool_bytes=6 * page_bytes, max_live_samples=4, max_context=256)
    toks, offs = workloads.make_prompts(1, 40, 40, shape.vocab, seed=9)
    with pytest.raises(R.RolloutError) as e:                 # 1 shared + 1 tail + 2 x 3 private = 8 > 6
        eng.rollout_prefill(toks, offs, 2, [80, 80])
    assert e.value.code == -2
    with pytest.raises(R.RolloutError) as e:                 # 5 samples > 4 slots
        eng.rollout_prefill(toks, offs, 5, [2] * 5)
    assert e.value.code == -2
    with pytest.raises(R.RolloutError) as e:
        eng.rollout_prefill(toks, offs, 1, [300])            # exceeds max_context
    assert e.value.code == -2
    with pytest.raises(R.RolloutError) as e:
        eng.rollout_prefill(np.array([5, shape.vocab], np.int32), [0, 2], 1, [2])
    assert e.value.code == -1
    st = eng.rollout_get_stats()
    assert st["pages_in_use"] == 0 and st["live_samples"] == 0 and st["samples_admitted"] == 0
    ids, t, lp, fin = eng.rollout_prefill(toks, offs, 2, [20, 20])   # 1 + 1 + 2 x 1 = 4 pages: fits
    assert ids.tolist() == [0, 1]
    eng.close()


@pytest.mark.parametrize("name", ["c1", "small-bf16"])
def test_empty_ragged_and_boundary_inputs(name):
    """Degenerate cases of the path: nothing live, empty prompt lists, one-token prompts and
    sequences, prompts that end exactly on a page boundary, a response that ends at the
    prefill, and a context that reaches max_context exactly."""
    import paper_2506_06122_amd as R
    shape, scale, _ = CASES[name]
    w = scaled_weights(shape, seed=1, scale=scale)
    model = oracle_model(shape, w)
    eng = make_engine(shape, w, max_live_samples=16, max_context=96, max_batch_tokens=256)
    assert len(eng.rollout_decode_step()[0]) == 0                       # nothing live: an empty step
    with pytest.raises(R.RolloutError) as e:                             # no prompts
        eng.rollout_prefill(np.zeros(0, np.int32), [0], 1, np.zeros(0, np.int32))
    assert e.value.code == -1
    with pytest.raises(R.RolloutError) as e:                             # an empty prompt among others
        eng.rollout_prefill([1, 2], [0, 2, 2], 1, [2, 2])
    assert e.value.code == -1
    assert eng.rollout_get_stats()["pages_in_use"] == 0
    assert len(eng.rollout_logprobs(np.zeros(0, np.int32), [0])) == 0    # no sequences
    assert eng.rollout_logprobs([7], [0, 1]).tolist() == [0.0]           # a one-token sequence has no target

    # prompt lengths 1, 31, 32, 33, 64 (page size 32); limits 1 (ends at the prefill), 2, and up to max_context
    lens = [1, 31, 32, 33, 64]
    rng = np.random.default_rng(17)
    toks = rng.integers(0, shape.vocab, sum(lens)).astype(np.int32)
    offs = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    limits = np.array([1, 2, 4, 3, 96 - 64 + 1], np.int32)               # the last one reaches position 95
    steps = int(limits.max())
    forced = rng.integers(0, shape.vocab, (5, steps)).astype(np.int32)
    ids, t, lp, fin = eng.rollout_prefill(toks, offs, 1, limits, forced_first=forced[:, 0])
    assert fin.tolist() == [True, False, False, False, False]
    fwd = T.KVForward(model)
    caches = [fwd.new_cache() for _ in lens]
    ref = fwd.extend(caches, [toks[offs[i]:offs[i + 1]] for i in range(5)])
    got = eng.rollout_debug_logits()
    worst = max(float(np.max(np.abs(got[i] - ref[i][-1]))) for i in range(5))
    live = [1, 2, 3, 4]
    for s in range(1, steps):
        ids, t, lp, fin = eng.rollout_decode_step(forced_tokens=forced[live, s])
        assert ids.tolist() == live
        ref = fwd.extend([caches[i] for i in live], [[int(forced[i, s - 1])] for i in live])
        got = eng.rollout_debug_logits()
        worst = max([worst] + [float(np.max(np.abs(got[k] - ref[k][0]))) for k in range(len(live))])
        assert fin.tolist() == [s + 1 == limits[i] for i in live]
        live = [i for i in live if s + 1 < limits[i]]
    assert not live and len(eng.rollout_decode_step()[0]) == 0
    print(f"{name}: max |dlogits| = {worst:.3e}")
    assert worst <= TOL[shape.dtype]
    with pytest.raises(R.RolloutError) as e:                             # one position too many
        eng.rollout_prefill(toks[:64], [0, 64], 1, [96 - 64 + 2])
    assert e.value.code == -2
    st = eng.rollout_get_stats()
    assert st["pages_in_use"] == 0 and st["live_samples"] == 0
    eng.close()


@pytest.mark.parametrize("name", ["c1", "small-bf16"])
def test_page_size_and_prefix_sharing_do_not_change_results(name):
    """The same prompts with 32- and 64-token pages, and n samples forked from one prefill
    against the same sample prefilled alone: paging and prefix sharing are bookkeeping, so
    logits agree to the last bit when the batch composition is the same, and within the
    tolerance when it is not."""
    shape, scale, _ = CASES[name]
    w = scaled_weights(shape, seed=1, scale=scale)
    toks, offs = workloads.make_prompts(2, 20, 75, shape.vocab, seed=23)
    forced = np.random.default_rng(3).integers(0, shape.vocab, (6, 5)).astype(np.int32)

    def run(page_tokens, prompts, n, rows):
        eng = make_engine(shape, w, page_tokens=page_tokens, max_context=128)
        t = np.concatenate([toks[offs[p]:offs[p + 1]] for p in prompts])
        o = np.concatenate([[0], np.cumsum([offs[p + 1] - offs[p] for p in prompts])]).astype(np.int32)
        f = forced[rows]
        out = []
        eng.rollout_prefill(t, o, n, np.full(len(prompts) * n, 5, np.int32), forced_first=f[:, 0])
        out.append(eng.rollout_debug_logits())
        for s in range(1, 5):
            eng.rollout_decode_step(forced_tokens=f[:, s])
            out.append(eng.rollout_debug_logits())
        eng.close()
        return out

    a = run(32, [0, 1], 3, list(range(6)))
    b = run(64, [0, 1], 3, list(range(6)))
    for x, y in zip(a, b):
        assert np.array_equal(x, y)
    alone = run(32, [1], 1, [4])                 # sample 1 of prompt 1, prefilled alone
    for s in range(1, 5):
        err = float(np.max(np.abs(alone[s][0] - a[s][4])))
        assert err <= TOL[shape.dtype]
        if shape.dtype == "fp32":
            assert err <= 1e-5


@pytest.mark.parametrize("name", ["c1", "small-bf16", "small-moe-bf16"])
def test_results_are_repeatable_and_independent_of_physical_pages_and_slots(name):
    """A race or a read of memory that nobody wrote shows as run-to-run noise, so: the same
    prompts and forced tokens (a) in a fresh context, (b) in a context whose pages and slots were
    used before by other, longer samples that were aborted in a shuffled order - the free lists
    hand everything out in another order and every page holds stale keys and values - and (c)
    once more in that context.  The logits of every step must agree to the last bit in all three."""
    shape, scale, _ = CASES[name]
    w = scaled_weights(shape, seed=1, scale=scale)
    toks, offs = workloads.make_prompts(3, 10, 90, shape.vocab, seed=29)
    P, n, steps = 3, 2, 6
    forced = np.random.default_rng(5).integers(0, shape.vocab, (P * n, steps)).astype(np.int32)
    # a pool just large enough that the second use must take over pages of the first
    eng_kw = dict(max_live_samples=16, max_context=160, max_batch_tokens=512)

    def job(eng):
        out = []
        ids = eng.rollout_prefill(toks, offs, n, np.full(P * n, steps + 1, np.int32), forced_first=forced[:, 0])[0]
        out.append(eng.rollout_debug_logits())
        for s in range(1, steps):
            eng.rollout_decode_step(forced_tokens=forced[:, s])
            out.append(eng.rollout_debug_logits())
        assert eng.rollout_abort(ids) == P * n and eng.rollout_get_stats()["pages_in_use"] == 0
        return out

    fresh = make_engine(shape, w, **eng_kw)
    a = job(fresh)
    fresh.close()
    used = make_engine(shape, w, **eng_kw)
    d_toks, d_offs = workloads.make_prompts(4, 40, 120, shape.vocab, seed=30)
    d_ids = used.rollout_prefill(d_toks, d_offs, 3, np.full(12, 20, np.int32))[0]
    for _ in range(5):
        used.rollout_decode_step()
    np.random.default_rng(6).shuffle(d_ids)
    for i in d_ids:                                    # one by one: pages and slots return in this order
        assert used.rollout_abort([i]) == 1
    assert used.rollout_get_stats()["pages_in_use"] == 0
    b = job(used)
    c = job(used)
    st = used.rollout_get_stats()                      # the phase clocks: host time inside the calls
    assert st["prefill_ms"] > 0 and st["decode_ms"] > 0 and st["extend_ms"] == 0 and st["logprobs_ms"] == 0
    used.close()
    for s in range(steps):
        assert np.array_equal(a[s], b[s]), f"step {s}: a used context gives other logits than a fresh one"
        assert np.array_equal(b[s], c[s]), f"step {s}: a second run in the same context gives other logits"
