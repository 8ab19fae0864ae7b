"""GPU tests of rollout_update_weights: after a refresh the context must behave exactly as a
context created with the new weights - checked against the oracle on the new weights."""
import numpy as np
import pytest

import paper_2506_06122_amd as R
import workloads
from gpu_util import make_engine, oracle_model, scaled_weights, teacher_forced_compare

pytestmark = pytest.mark.gpu

CASES = {
    "c1-fp32": (workloads.C1_TINY, 1.0, 0, 1e-4),
    "tiny-moe-fp32": (workloads.TINY_MOE_FP32, 6.0, 2, 1e-4),
    "small-bf16": (workloads.SMALL_BF16, 1.0, 0, 2e-2),
    "small-moe-bf16": (workloads.SMALL_MOE_BF16, 1.5, 2, 2e-2),
    # hidden = 17 and FFN = 45 fragments deep: the re-ordering kernel's odd last k-tile
    "odd-k-tiles-bf16": (workloads.ModelShape("odd-k-bf16", 2, 544, 8, 2, 128, 1440, 2048), 1.0, 0, 2e-2),
}


def run(eng, shape, w, seed):
    model = oracle_model(shape, w)
    toks, offs = workloads.make_prompts(3, 5, 50, shape.vocab, seed=seed)
    forced = np.random.default_rng(seed).integers(0, shape.vocab, (6, 3)).astype(np.int32)
    return teacher_forced_compare(eng, model, toks, offs, 2, forced, 3)


@pytest.mark.parametrize("name", list(CASES))
def test_refresh_equals_a_fresh_context(name):
    """Weights A -> run; refresh every tensor to weights B, one bucket per layer plus one for the
    model-level tensors -> run against the oracle on B; then refresh only the lm_head and layer
    0's attention back to A -> run against the oracle on that mixture.  The KV pool is kept:
    pages of the earlier runs are reused under the new weights."""
    shape, scale, flags, tol = CASES[name]
    wa = scaled_weights(shape, seed=1, scale=scale)
    wb = scaled_weights(shape, seed=2, scale=scale)
    eng = make_engine(shape, wa, max_live_samples=8, max_context=128, max_batch_tokens=256, flags=flags)
    worst = [max(run(eng, shape, wa, 91))]
    eng.rollout_update_weights({k: wb[k] for k in ("embed", "final_norm", "lm_head")})
    for i in range(shape.n_layers):
        eng.rollout_update_weights({k: v for k, v in wb.items() if k.startswith(f"layers.{i}.")})
    worst.append(max(run(eng, shape, wb, 92)))
    back = ["lm_head", "layers.0.wq", "layers.0.wk", "layers.0.wv", "layers.0.wo", "layers.0.norm1"]
    eng.rollout_update_weights({k: wa[k] for k in back})
    wmix = dict(wb)
    wmix.update({k: wa[k] for k in back})
    worst.append(max(run(eng, shape, wmix, 93)))
    print(f"{name}: max error before / after full refresh / after partial refresh = "
          + " / ".join(f"{x:.3e}" for x in worst))
    assert max(worst) <= tol
    assert eng.rollout_get_stats()["pages_in_use"] == 0
    eng.close()


def test_refresh_is_refused_while_samples_run():
    shape = workloads.C1_TINY
    w = scaled_weights(shape, seed=1)
    eng = make_engine(shape, w, max_live_samples=4, max_context=64, max_batch_tokens=64)
    toks, offs = workloads.make_prompts(1, 8, 8, shape.vocab, seed=1)
    ids, tk, lps, fin = eng.rollout_prefill(toks, offs, 1, np.array([3], np.int32))
    with pytest.raises(R.RolloutError) as e:
        eng.rollout_update_weights({"lm_head": w["lm_head"]})
    assert e.value.code == R.binding.E_STATE
    eng.rollout_abort(ids)
    eng.rollout_queue_push(toks, offs, 1, np.array([3], np.int32))
    with pytest.raises(R.RolloutError):
        eng.rollout_update_weights({"lm_head": w["lm_head"]})
    while len(eng.rollout_queue_step()[0]):
        pass
    eng.rollout_update_weights({"lm_head": w["lm_head"]})
    arr = (R.binding.rollout_tensor_update * 1)(R.binding.rollout_tensor_update(5, 4, 1))   # layer 5 of 2
    assert eng.lib.rollout_update_weights(eng.ctx, 1, arr) == R.binding.E_INVAL
    arr = (R.binding.rollout_tensor_update * 1)(R.binding.rollout_tensor_update(0, 12, 1))  # router, dense model
    assert eng.lib.rollout_update_weights(eng.ctx, 1, arr) == R.binding.E_INVAL
    eng.close()
