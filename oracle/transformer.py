"""Decoder-only transformer forward in fp64: the function the rollout path evaluates.

Test infrastructure.  The paper names the phases (prefill builds the key-value cache,
decoding extends it one token at a time, the inference stage is a single forward pass:
section 2.1, "Optimization Workflow") and the model families (Qwen2.5 dense and Qwen3
mixture-of-experts: section 5.1) but not the operators, which are the standard public
ones:

  RMSNorm      h = x * g / sqrt(mean(x^2) + eps)
  projections  y = W x, no bias; W is [out][in]
  RoPE         half-split pairing: (u_i, u_{i+dh/2}) rotated by pos * theta^(-2i/dh)
  attention    grouped-query: query head j uses KV head j // (Hq / Hkv); causal softmax of
               q.k / sqrt(dh)
  FFN          W_down( silu(W_gate h) * (W_up h) ), silu(a) = a / (1 + exp(-a))
  MoE FFN      router logits r = W_r h; top-k experts by (r descending, index ascending);
               weights = softmax of the selected r; output = sum of weight * expert FFN
  logits       W_lm RMSNorm(x)

and, where the shape says so, what tells the named families apart in their public
definitions: a bias on the q, k and v projections (Qwen2.5), an RMSNorm over head_dim on
every q and k head before RoPE with gains q_norm, k_norm (Qwen3), logits through the
embedding matrix instead of a separate W_lm (the small Qwen2.5 models).

Two independent evaluations are kept: `forward_full` recomputes a whole sequence from
scratch with an explicit causal mask (the brute-force definition), and `KVForward`
processes rows incrementally against per-sequence key/value caches (what prefill followed
by decoding does).  They must agree; a test holds them to it.

Weights arrive as fp32 arrays that already hold the storage-rounded values (bf16-exact
for bf16 models) under the names used by the checkpoint layout: embed, layers.i.norm1,
wq, wk, wv, wo, norm2, w_gate, w_up, w_down (or router, experts.w_gate/w_up/w_down),
final_norm, lm_head.  Activations are never rounded.
"""
from __future__ import annotations

import numpy as np


# ----------------------------------------------------------------------------------------
# operators
# ----------------------------------------------------------------------------------------
def rmsnorm(x: np.ndarray, g: np.ndarray, eps: float) -> np.ndarray:
    return x * g / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps)


def rope(u: np.ndarray, pos, theta: float) -> np.ndarray:
    """Rotate the last axis of u ([..., heads, dh]) for positions pos ([...])."""
    dh = u.shape[-1]
    half = dh // 2
    inv_freq = theta ** (-2.0 * np.arange(half, dtype=np.float64) / dh)
    phi = np.asarray(pos, dtype=np.float64)[..., None, None] * inv_freq      # [..., 1, half]
    a, b = u[..., :half], u[..., half:]
    return np.concatenate([a * np.cos(phi) - b * np.sin(phi),
                           b * np.cos(phi) + a * np.sin(phi)], axis=-1)


def silu(a: np.ndarray) -> np.ndarray:
    return a / (1.0 + np.exp(-a))


def softmax(s: np.ndarray, axis: int = -1) -> np.ndarray:
    e = np.exp(s - np.max(s, axis=axis, keepdims=True))
    return e / np.sum(e, axis=axis, keepdims=True)


def route(r: np.ndarray, top_k: int):
    """Top-k experts of one router-logit vector and their mixing weights."""
    order = np.lexsort((np.arange(len(r)), -r))[:top_k]       # r descending, index ascending
    return order, softmax(r[order])


def routing_gaps(r: np.ndarray, chosen, top_k: int):
    """How far an expert set is from the top-k of the logits r, as two differences:

      below   = (k-th largest logit) - (smallest chosen logit): the weakest member is that much
                worse than the weakest member of the true top-k;
      outside = (largest logit not chosen) - (smallest chosen logit): an expert left out beats
                a member by that much.

    A set of k distinct experts is a valid top-k (up to ties) iff both are <= 0; a set that is
    the top-k up to a logit tolerance tol has both <= tol.  The second difference is the
    complete condition (every member >= every non-member); the first is kept because it is
    what a wrong weakest member alone shows.
    """
    chosen = np.asarray(chosen, dtype=np.int64)
    kth = np.sort(r)[::-1][top_k - 1]
    low = np.min(r[chosen])
    rest = np.ones(len(r), dtype=bool)
    rest[chosen] = False
    outside = (np.max(r[rest]) - low) if rest.any() else -np.inf
    return float(kth - low), float(outside)


class Model:
    """Shape + weights, widened to fp64 on access (cached when `cache` is true)."""

    def __init__(self, shape, weights: dict, cache: bool = True):
        self.shape = shape
        self._w = weights
        self._cache = {} if cache else None
        # Test hook for MoE parity: routing is an integer decision taken from floats, so a
        # lower-precision implementation may legitimately pick another expert on a near-tie.
        # When routing_override[layer] holds an int array [rows][top_k], `ffn` uses those
        # expert sets (mixing weights still come from this model's own router logits) and
        # appends to routing_regret, per row, how far the set is from the top-k of those
        # logits (`routing_gaps`): both numbers are <= 0 exactly when the set is the top-k.
        self.routing_override = {}
        self.routing_regret = []
        # Second test hook: when routing_trace is a list, `ffn` appends (layer, router logits of
        # the row, experts used) for every row it routes, in call order.
        self.routing_trace = None

    def w(self, name: str) -> np.ndarray:
        if self._cache is None:
            return self._w[name].astype(np.float64)
        if name not in self._cache:
            self._cache[name] = self._w[name].astype(np.float64)
        return self._cache[name]

    # ---- blocks shared by both evaluations (pure per-row math, no sequence structure) ----
    def qkv(self, layer: int, x: np.ndarray, pos: np.ndarray):
        s, p = self.shape, f"layers.{layer}."
        h = rmsnorm(x, self.w(p + "norm1"), s.rms_eps)
        q, k, v = h @ self.w(p + "wq").T, h @ self.w(p + "wk").T, h @ self.w(p + "wv").T
        if getattr(s, "qkv_bias", False):
            q, k, v = q + self.w(p + "bq"), k + self.w(p + "bk"), v + self.w(p + "bv")
        q = q.reshape(len(x), s.n_q_heads, s.head_dim)
        k = k.reshape(len(x), s.n_kv_heads, s.head_dim)
        v = v.reshape(len(x), s.n_kv_heads, s.head_dim)
        if getattr(s, "qk_norm", False):  # per head, over head_dim
            q, k = rmsnorm(q, self.w(p + "q_norm"), s.rms_eps), rmsnorm(k, self.w(p + "k_norm"), s.rms_eps)
        return rope(q, pos, s.rope_theta), rope(k, pos, s.rope_theta), v

    def ffn(self, layer: int, h: np.ndarray) -> np.ndarray:
        s, p = self.shape, f"layers.{layer}."
        if not s.n_experts:
            act = silu(h @ self.w(p + "w_gate").T) * (h @ self.w(p + "w_up").T)
            return act @ self.w(p + "w_down").T
        r = h @ self.w(p + "router").T                                   # [rows][E]
        wg, wu, wd = (self.w(p + "experts." + n) for n in ("w_gate", "w_up", "w_down"))
        out = np.zeros_like(h)
        forced = self.routing_override.get(layer)
        for i in range(len(h)):
            experts, mix = route(r[i], s.top_k)
            if forced is not None:
                chosen = np.asarray(forced[i], dtype=np.int64)
                assert len(set(chosen.tolist())) == s.top_k
                self.routing_regret.append(routing_gaps(r[i], chosen, s.top_k))
                experts, mix = chosen, softmax(r[i][chosen])
            if self.routing_trace is not None:
                self.routing_trace.append((layer, r[i].copy(), np.asarray(experts).copy()))
            for e, m in zip(experts, mix):
                act = silu(wg[e] @ h[i]) * (wu[e] @ h[i])
                out[i] += m * (wd[e] @ act)
        return out

    def post_attention(self, layer: int, x: np.ndarray, o: np.ndarray) -> np.ndarray:
        s, p = self.shape, f"layers.{layer}."
        x = x + o.reshape(len(x), s.n_q_heads * s.head_dim) @ self.w(p + "wo").T
        return x + self.ffn(layer, rmsnorm(x, self.w(p + "norm2"), s.rms_eps))

    def logits(self, x: np.ndarray) -> np.ndarray:
        head = "embed" if getattr(self.shape, "tied_lm_head", False) else "lm_head"
        return rmsnorm(x, self.w("final_norm"), self.shape.rms_eps) @ self.w(head).T


# ----------------------------------------------------------------------------------------
# evaluation 1: full recompute of one sequence (brute-force definition)
# ----------------------------------------------------------------------------------------
def forward_full(model: Model, tokens) -> np.ndarray:
    """Logits [T][V] of one sequence, every position recomputed from the tokens alone."""
    s = model.shape
    tokens = np.asarray(tokens)
    n_tok = len(tokens)
    pos = np.arange(n_tok)
    group = s.n_q_heads // s.n_kv_heads
    allowed = pos[None, :] <= pos[:, None]                     # key u visible to query t
    x = model.w("embed")[tokens]
    for layer in range(s.n_layers):
        q, k, v = model.qkv(layer, x, pos)
        o = np.empty_like(q)
        for j in range(s.n_q_heads):
            scores = q[:, j, :] @ k[:, j // group, :].T / np.sqrt(s.head_dim)
            probs = softmax(np.where(allowed, scores, -np.inf), axis=-1)
            o[:, j, :] = probs @ v[:, j // group, :]
        x = model.post_attention(layer, x, o)
    return model.logits(x)


# ----------------------------------------------------------------------------------------
# evaluation 2: incremental, against per-sequence key/value caches
# ----------------------------------------------------------------------------------------
class KVCache:
    """Keys and values of one sequence: per layer, arrays [ctx][Hkv][dh]."""

    def __init__(self, n_layers: int):
        self.k = [None] * n_layers
        self.v = [None] * n_layers
        self.length = 0

    def fork(self) -> "KVCache":
        c = KVCache(len(self.k))
        c.k = [None if a is None else a.copy() for a in self.k]
        c.v = [None if a is None else a.copy() for a in self.v]
        c.length = self.length
        return c

    def append(self, layer: int, k_rows: np.ndarray, v_rows: np.ndarray) -> None:
        if self.k[layer] is None:
            self.k[layer], self.v[layer] = k_rows.copy(), v_rows.copy()
        else:
            self.k[layer] = np.concatenate([self.k[layer], k_rows])
            self.v[layer] = np.concatenate([self.v[layer], v_rows])


class KVForward:
    """Extend cached sequences by new tokens and return the logits of the new rows."""

    def __init__(self, model: Model):
        self.model = model

    def new_cache(self) -> KVCache:
        return KVCache(self.model.shape.n_layers)

    def extend(self, caches: list[KVCache], new_tokens: list) -> list[np.ndarray]:
        """caches[i] grows by new_tokens[i] (one or more ids); returns logits [len][V] each."""
        model, s = self.model, self.model.shape
        group = s.n_q_heads // s.n_kv_heads
        counts = [len(t) for t in new_tokens]
        starts = np.concatenate([[0], np.cumsum(counts)])
        tokens = np.concatenate([np.asarray(t, dtype=np.int64) for t in new_tokens])
        pos = np.concatenate([c.length + np.arange(n) for c, n in zip(caches, counts)])
        x = model.w("embed")[tokens]
        for layer in range(s.n_layers):
            q, k, v = model.qkv(layer, x, pos)
            o = np.empty_like(q)
            for i, cache in enumerate(caches):
                lo, hi = starts[i], starts[i + 1]
                cache.append(layer, k[lo:hi], v[lo:hi])
                keys, vals = cache.k[layer], cache.v[layer]
                for row in range(lo, hi):
                    ctx = pos[row] + 1                           # keys 0 .. pos visible
                    for j in range(s.n_q_heads):
                        scores = keys[:ctx, j // group, :] @ q[row, j, :] / np.sqrt(s.head_dim)
                        o[row, j, :] = softmax(scores) @ vals[:ctx, j // group, :]
            x = model.post_attention(layer, x, o)
        for cache, n in zip(caches, counts):
            cache.length += n
        logits = model.logits(x)
        return [logits[starts[i]:starts[i + 1]] for i in range(len(caches))]


# ----------------------------------------------------------------------------------------
# inference-stage forward: per-token log-probs of packed sequences
# ----------------------------------------------------------------------------------------
def packed_log_probs(model: Model, tokens, cu_seqlens, temperature: float = 1.0) -> np.ndarray:
    """log p(token_t | tokens_<t) for packed sequences; 0 at each sequence's first token.

    Sequences are independent (block-diagonal causal mask, positions restart at 0), so
    each is evaluated alone by the brute-force forward.
    """
    tokens = np.asarray(tokens)
    out = np.zeros(len(tokens), dtype=np.float64)
    for a, b in zip(cu_seqlens[:-1], cu_seqlens[1:]):
        if b - a < 2:
            continue
        z = forward_full(model, tokens[a:b])[:-1] / temperature
        m = np.max(z, axis=-1, keepdims=True)
        lse = m[:, 0] + np.log(np.sum(np.exp(z - m), axis=-1))
        out[a + 1:b] = z[np.arange(b - a - 1), tokens[a + 1:b]] - lse
    return out
