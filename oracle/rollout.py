"""Generation stage on the CPU: prefill each prompt, then decode n samples per prompt.

Test infrastructure.  Follows the paper's statement of the stage (section 2.1,
"Optimization Workflow": the prefill phase processes the prompt to compute its key-value
cache, the decoding phase generates tokens autoregressively until the termination
criterion) and its sample-granular view of a batch (section 4.1, "Rollout Scheduler": each
request's lifecycle is its own).  A sample's tokens depend only on the weights, its
prompt, the seed and its sample id.

Sample id = (global prompt index) * n_samples + j.  Response position 0 is drawn from the
prompt's last-position logits; position t from the logits after feeding token t - 1.  A
sample finishes when it emits `eos_id` (if eos_id >= 0; the token is kept) or when it has
emitted max_new_tokens[i] tokens.
"""
from __future__ import annotations

import dataclasses

import numpy as np

from . import philox, sampler
from .transformer import KVForward, Model


@dataclasses.dataclass
class SampleTrace:
    sample_id: int
    tokens: list            # emitted token ids
    logprobs: list          # log-prob of each emitted token
    logits: list            # fp32 logits row each token was drawn from (kept when asked)


def generate(model: Model, prompt_tokens, prompt_offsets, n_samples: int, max_new_tokens,
             eos_id: int, temperature: float, top_p: float, seed: int,
             first_prompt_index: int = 0, keep_logits: bool = False,
             forced_tokens: dict | None = None) -> list[SampleTrace]:
    """Roll out every sample to completion, one sample at a time.

    forced_tokens, when given, maps sample_id -> list of token ids to emit instead of the
    drawn ones (teacher forcing); log-probs are then those of the forced tokens.
    """
    fwd = KVForward(model)
    inv_t = sampler.inv_temperature(temperature)
    traces = []
    n_prompts = len(prompt_offsets) - 1
    for p in range(n_prompts):
        prompt = prompt_tokens[prompt_offsets[p]:prompt_offsets[p + 1]]
        prefix = fwd.new_cache()
        last_logits = fwd.extend([prefix], [prompt])[0][-1]
        for j in range(n_samples):
            sid = (first_prompt_index + p) * n_samples + j
            limit = int(max_new_tokens[p * n_samples + j])
            forced = None if forced_tokens is None else forced_tokens.get(sid)
            cache = prefix.fork()
            trace = SampleTrace(sid, [], [], [])
            row = last_logits
            for t in range(limit):
                row32 = row.astype(np.float32)
                if forced is not None:
                    tok = int(forced[t])
                    lp = sampler.log_prob(row32, inv_t, tok)
                else:
                    tok, lp = sampler.sample(row32, inv_t, top_p,
                                             philox.rollout_uniform(seed, sid, t))
                trace.tokens.append(tok)
                trace.logprobs.append(lp)
                if keep_logits:
                    trace.logits.append(row32)
                if (eos_id >= 0 and tok == eos_id) or t + 1 == limit:
                    break
                row = fwd.extend([cache], [[tok]])[0][0]
            traces.append(trace)
    return traces


def decode_slice_batched(model: Model, prompt, n_samples: int, n_new: int,
                         temperature: float, top_p: float, seed: int,
                         out_tokens: list | None = None) -> int:
    """Prefill one prompt, then decode n_samples samples together for n_new tokens each.

    Same arithmetic as `generate` with the samples' rows stacked into one matrix per step
    (the projections see [n_samples][hidden] instead of one row at a time); sample j has id j
    and runs without an end-of-sequence token.  Returns the number of tokens emitted; used to
    time the oracle on a bounded slice.  out_tokens, when given, receives one list of emitted
    token ids per sample (a test compares them with `generate`).
    """
    fwd = KVForward(model)
    inv_t = sampler.inv_temperature(temperature)
    prefix = fwd.new_cache()
    last = fwd.extend([prefix], [prompt])[0][-1]
    caches = [prefix.fork() for _ in range(n_samples)]
    rows = [last] * n_samples
    emitted = 0
    if out_tokens is not None:
        out_tokens[:] = [[] for _ in range(n_samples)]
    for t in range(n_new):
        toks = []
        for j in range(n_samples):
            tok, _ = sampler.sample(rows[j].astype(np.float32), inv_t, top_p,
                                    philox.rollout_uniform(seed, j, t))
            toks.append([tok])
            emitted += 1
            if out_tokens is not None:
                out_tokens[j].append(tok)
        if t + 1 < n_new:
            rows = [r[0] for r in fwd.extend(caches, toks)]
    return emitted
