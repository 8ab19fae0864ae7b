"""Helpers shared by the GPU parity tests."""
import numpy as np

import paper_2506_06122_amd as R
import workloads
from oracle import transformer as T


def scaled_weights(shape, seed, scale=1.0):
    """Random-init weights; matrices optionally scaled up (then re-rounded to the storage
    type) so that small test shapes have logits of order one rather than of order 0.01."""
    w = workloads.make_weights(shape, seed)
    if scale != 1.0:
        for k in w:
            if w[k].ndim > 1:
                w[k] = (w[k] * np.float32(scale)).astype(np.float32)
                if shape.dtype == "bf16":
                    w[k] = workloads.round_to_bf16(w[k])
    return w


def make_engine(shape, weights, **kw):
    args = dict(kv_pool_bytes=256 << 20, page_tokens=32, max_live_samples=32, max_context=512,
                max_batch_tokens=1024, seed=3)
    args.update(kw)
    return R.Rollout(shape, weights, **args)


def oracle_model(shape, weights):
    return T.Model(shape, weights)


def teacher_forced_compare(eng, model, prompt_tokens, offsets, n_samples, forced, steps):
    """Prefill + `steps - 1` decode steps with forced tokens on the GPU; the oracle runs the
    same token sequences.  forced: int array [P * n][steps].  Returns (max abs logits
    error, max abs log-prob error) over all steps and samples."""
    P = len(offsets) - 1
    fwd = T.KVForward(model)
    inv_t = np.float32(1.0)
    ids, toks, lps, fin = eng.rollout_prefill(prompt_tokens, offsets, n_samples,
                                              np.full(P * n_samples, steps, np.int32),
                                              forced_first=forced[:, 0])
    assert np.array_equal(toks, forced[:, 0]) and not fin.any()
    gpu_logits = eng.rollout_debug_logits()
    assert gpu_logits.shape[0] == P
    caches, worst, worst_lp = [], 0.0, 0.0
    from oracle import sampler
    moe = bool(model.shape.n_experts)
    # MoE: the oracle takes the GPU's expert choices (an integer decision made from floats in
    # another precision) and records how far from optimal they are in its own router logits.
    routing = eng.rollout_debug_routing(int(offsets[-1])) if moe else None
    for p in range(P):
        if moe:
            model.routing_override = {l: routing[l][offsets[p]:offsets[p + 1]]
                                      for l in range(model.shape.n_layers)}
        prefix = fwd.new_cache()
        ref = fwd.extend([prefix], [prompt_tokens[offsets[p]:offsets[p + 1]]])[0][-1]
        worst = max(worst, float(np.max(np.abs(gpu_logits[p] - ref))))
        for j in range(n_samples):
            caches.append(prefix.fork())
            want = sampler.log_prob(ref.astype(np.float32), inv_t, int(forced[p * n_samples + j, 0]))
            worst_lp = max(worst_lp, abs(want - float(lps[p * n_samples + j])))
    for t in range(1, steps):
        ids2, toks, lps, fin = eng.rollout_decode_step(forced_tokens=forced[:, t])
        assert np.array_equal(ids2, ids) and np.array_equal(toks, forced[:, t])
        assert fin.all() == (t == steps - 1)
        gpu_logits = eng.rollout_debug_logits()
        if moe:
            routing = eng.rollout_debug_routing(len(caches))
            model.routing_override = {l: routing[l] for l in range(model.shape.n_layers)}
        ref = fwd.extend(caches, [[int(x)] for x in forced[:, t - 1]])
        for i in range(len(caches)):
            worst = max(worst, float(np.max(np.abs(gpu_logits[i] - ref[i][0]))))
            want = sampler.log_prob(ref[i][0].astype(np.float32), inv_t, int(forced[i, t]))
            worst_lp = max(worst_lp, abs(want - float(lps[i])))
    model.routing_override = {}
    return worst, worst_lp
