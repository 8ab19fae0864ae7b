"""GPU parity for the options that tell the named model families apart: QKV bias (Qwen2.5),
per-head QK RMSNorm before the rotary embedding (Qwen3), tied lm_head (small Qwen2.5)."""
import dataclasses

import numpy as np
import pytest

import paper_2506_06122_amd as R
import workloads
from gpu_util import make_engine, oracle_model, scaled_weights, teacher_forced_compare

pytestmark = pytest.mark.gpu

QWEN25 = dict(qkv_bias=True)
QWEN25_SMALL = dict(qkv_bias=True, tied_lm_head=True)
QWEN3 = dict(qk_norm=True)
ALL = dict(qkv_bias=True, qk_norm=True, tied_lm_head=True)

CASES = {
    "c1-fp32-all": (workloads.C1_TINY, ALL, 1.0, 0, 1e-4),
    "small-bf16-qwen2.5": (workloads.SMALL_BF16, QWEN25, 1.0, 0, 2e-2),
    "small-bf16-qwen2.5-tied": (workloads.SMALL_BF16, QWEN25_SMALL, 1.0, 0, 2e-2),
    "small-bf16-qwen3": (workloads.SMALL_BF16, QWEN3, 1.0, 0, 2e-2),
    "small-bf16-all-plain": (workloads.SMALL_BF16, ALL, 1.0, 1, 2e-2),
    "small-moe-bf16-qwen3": (workloads.SMALL_MOE_BF16, QWEN3, 1.5, 2, 2e-2),
}


@pytest.mark.parametrize("rows", ["6rows", "40rows"])
@pytest.mark.parametrize("name", list(CASES))
def test_family_options_match_oracle(name, rows):
    """Prefill and teacher-forced decode steps against the oracle with the option on: 6 live rows
    (streamed projections, fused attention prologue) and 40 (tile projections, split planes)."""
    base, opts, scale, flags, tol = CASES[name]
    shape = dataclasses.replace(base, name=base.name + "+" + "+".join(opts), **opts)
    w = scaled_weights(shape, seed=1, scale=scale)
    assert ("lm_head" in w) == (not shape.tied_lm_head) and ("layers.0.bq" in w) == shape.qkv_bias
    model = oracle_model(shape, w)
    P, n = (3, 2) if rows == "6rows" else (5, 8)
    eng = make_engine(shape, w, max_live_samples=48, max_context=128, max_batch_tokens=512, flags=flags)
    toks, offs = workloads.make_prompts(P, 5, 60, shape.vocab, seed=101)
    forced = np.random.default_rng(102).integers(0, shape.vocab, (P * n, 3)).astype(np.int32)
    worst, worst_lp = teacher_forced_compare(eng, model, toks, offs, n, forced, 3)
    # the option is live on the GPU too: the oracle without it is far away
    plain = oracle_model(dataclasses.replace(shape, qkv_bias=False, qk_norm=False), w)
    far, _ = teacher_forced_compare(make_engine(shape, w, max_live_samples=48, max_context=128, max_batch_tokens=512,
                                                flags=flags), plain, toks[:offs[1]], offs[:2], 1, forced[:1], 2) \
        if (shape.qkv_bias or shape.qk_norm) and not shape.n_experts else (1.0, 0)
    print(f"{shape.name} {rows}: max |dlogits| = {worst:.3e}, max |dlogp| = {worst_lp:.3e}; without the option {far:.2e}")
    assert worst <= tol and worst_lp <= tol and far > 10 * tol
    assert eng.rollout_get_stats()["matrix_core_path"] == int(flags != 1 and shape.dtype == "bf16")
    eng.close()


def test_family_tensors_refresh_and_are_checked():
    shape = dataclasses.replace(workloads.SMALL_BF16, **ALL)
    wa, wb = scaled_weights(shape, seed=1), scaled_weights(shape, seed=2)
    eng = make_engine(shape, wa, max_live_samples=8, max_context=128, max_batch_tokens=256)
    eng.rollout_update_weights(wb)                       # every tensor, embed doubling as lm_head
    toks, offs = workloads.make_prompts(2, 5, 40, shape.vocab, seed=111)
    forced = np.random.default_rng(112).integers(0, shape.vocab, (4, 3)).astype(np.int32)
    worst, worst_lp = teacher_forced_compare(eng, oracle_model(shape, wb), toks, offs, 2, forced, 3)
    assert worst <= 2e-2 and worst_lp <= 2e-2
    with pytest.raises(R.RolloutError):                  # tied: there is no separate lm_head to refresh
        eng.rollout_update_weights({"lm_head": wb["embed"]})
    eng.close()
    plain = make_engine(workloads.SMALL_BF16, scaled_weights(workloads.SMALL_BF16, seed=1), max_live_samples=8,
                        max_context=128, max_batch_tokens=256)
    with pytest.raises(R.RolloutError):                  # a model without the option has no such tensor
        plain.rollout_update_weights({"layers.0.bq": wb["layers.0.bq"]})
    with pytest.raises(R.RolloutError):
        plain.rollout_update_weights({"layers.0.q_norm": wb["layers.0.q_norm"]})
    plain.close()


@pytest.mark.parametrize("n_q,n_kv,fast", [(32, 2, 1), (32, 1, 0)], ids=["G16", "G32-plain-path"])
def test_many_query_heads_per_kv_head(n_q, n_kv, fast):
    """16 query heads per KV head fill the attention tile's 16 columns (and the merge of the KV
    splits walks 2048 outputs per KV head); 32 do not fit and must take the plain path.  Contexts
    of 200-330 positions: the decode attention runs split, with 6 rows (streamed projections)
    and with 40 (tile projections)."""
    shape = workloads.ModelShape(f"small-{n_q}q{n_kv}kv-bf16", 2, 512, n_q, n_kv, 128, 1024, 2048)
    w = scaled_weights(shape, seed=1)
    model = oracle_model(shape, w)
    for prompts, samples in ((3, 2), (5, 8)):
        eng = make_engine(shape, w, max_live_samples=64, max_context=512, max_batch_tokens=2048)
        assert eng.rollout_get_stats()["matrix_core_path"] == fast
        toks, offs = workloads.make_prompts(prompts, 200, 330, shape.vocab, seed=17)
        forced = np.random.default_rng(18).integers(0, shape.vocab, (prompts * samples, 4)).astype(np.int32)
        worst = teacher_forced_compare(eng, model, toks, offs, samples, forced, 4)
        print(f"{n_q} query heads, {n_kv} KV heads, {prompts * samples} rows: max |dlogits|, |dlogp| = {worst[0]:.3e}, {worst[1]:.3e}")
        assert max(worst) <= 2e-2
        eng.close()
