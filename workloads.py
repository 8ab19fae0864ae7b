"""Seeded synthetic inputs for the rollout path: model shapes, random-init weights,
prompts, response-length draws and raw uniform words.

This module is the only code shared by the CPU oracle's tests and the HIP path's tests
and benchmark.  It holds no transformer, sampler or generator arithmetic of the method
itself: it only draws numbers, rounds weights to their storage type, and names shapes.

The paper trains Qwen2.5-7B and Qwen3-30B-A3B models on sequences of up to 8192 tokens
with long-tailed response lengths (paper section 5, "Experiments", and section 4.3,
"Sample-level Rollout Lifecycle Control").  Its datasets and pretrained weights are not
available, so every input here is a synthetic stand-in with the same shapes: token ids
uniform over the vocabulary, weights N(0, 0.02), response lengths drawn from capped
geometric / log-normal laws.
"""
from __future__ import annotations

import dataclasses
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np


@dataclasses.dataclass(frozen=True)
class ModelShape:
    name: str
    n_layers: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn_dim: int          # dense SwiGLU width (0 when every layer is MoE)
    vocab: int
    dtype: str = "bf16"   # storage type of weights and KV cache: "fp32" | "bf16"
    n_experts: int = 0
    top_k: int = 0
    expert_ffn_dim: int = 0
    rms_eps: float = 1e-6
    rope_theta: float = 1e6
    # what distinguishes the named model families (all off in the benchmark configurations)
    qkv_bias: bool = False      # q, k, v projections add a bias
    qk_norm: bool = False       # RMSNorm over head_dim on every q and k head, before the rotary embedding
    tied_lm_head: bool = False  # logits = h . embed^T, no separate lm_head

    @property
    def is_moe(self) -> bool:
        return self.n_experts > 0

    def with_layers(self, n_layers: int, name: str | None = None) -> "ModelShape":
        return dataclasses.replace(self, n_layers=n_layers,
                                   name=name or f"{self.name}-L{n_layers}")

    def param_count(self) -> int:
        d, qd, kd = self.hidden, self.n_q_heads * self.head_dim, self.n_kv_heads * self.head_dim
        per_layer = 2 * d + d * (qd + 2 * kd) + qd * d
        if self.is_moe:
            per_layer += self.n_experts * d + self.n_experts * 3 * self.expert_ffn_dim * d
        else:
            per_layer += 3 * self.ffn_dim * d
        return self.n_layers * per_layer + 2 * self.vocab * d + d


# The five configurations of the benchmark description, as shapes.
C1_TINY = ModelShape("tiny-fp32", 2, 256, 4, 2, 64, 688, 1024, dtype="fp32", rope_theta=10000.0)
C2_1P5B = ModelShape("qwen2.5-1.5b-shape", 28, 1536, 12, 2, 128, 8960, 151936)
C3_7B = ModelShape("qwen2.5-7b-shape", 28, 3584, 28, 4, 128, 18944, 152064)
C4_30B_A3B = ModelShape("qwen3-30b-a3b-shape", 48, 2048, 32, 4, 128, 0, 151936,
                        n_experts=128, top_k=8, expert_ffn_dim=768)
# Small shapes for fast parity cases (same operators, fewer/lesser dimensions).
SMALL_BF16 = ModelShape("small-bf16", 3, 512, 8, 2, 128, 1408, 4096)
SMALL_MOE_BF16 = ModelShape("small-moe-bf16", 2, 512, 8, 2, 128, 0, 2048,
                            n_experts=16, top_k=4, expert_ffn_dim=256)
TINY_MOE_FP32 = ModelShape("tiny-moe-fp32", 2, 128, 4, 2, 32, 0, 512, dtype="fp32",
                           n_experts=8, top_k=2, expert_ffn_dim=96, rope_theta=10000.0)


# ----------------------------------------------------------------------------------------
# storage rounding
# ----------------------------------------------------------------------------------------
def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16 (ties to even); result stays fp32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    bits = a.view(np.uint32)
    lsb = (bits >> np.uint32(16)) & np.uint32(1)
    rounded = (bits + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    return rounded.view(np.float32)


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """Upper 16 bits of bf16-exact fp32 values, as uint16 (the device storage format)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    bits = a.view(np.uint32)
    assert not np.any(bits & np.uint32(0xFFFF)), "values are not bf16-exact"
    return (bits >> np.uint32(16)).astype(np.uint16)


# ----------------------------------------------------------------------------------------
# weights
# ----------------------------------------------------------------------------------------
def weight_layout(shape: ModelShape) -> list[tuple[str, tuple[int, ...], str]]:
    """(name, dims, kind) of every tensor in checkpoint order; kind is 'matrix', 'gain' or 'bias'.

    Matrices are row-major [out_features][in_features]; a projection is y = W x.
    """
    d, qd, kd = shape.hidden, shape.n_q_heads * shape.head_dim, shape.n_kv_heads * shape.head_dim
    out: list[tuple[str, tuple[int, ...], str]] = [("embed", (shape.vocab, d), "matrix")]
    for i in range(shape.n_layers):
        p = f"layers.{i}."
        out += [(p + "norm1", (d,), "gain"), (p + "wq", (qd, d), "matrix"),
                (p + "wk", (kd, d), "matrix"), (p + "wv", (kd, d), "matrix"),
                (p + "wo", (d, qd), "matrix"), (p + "norm2", (d,), "gain")]
        if shape.qkv_bias:
            out += [(p + "bq", (qd,), "bias"), (p + "bk", (kd,), "bias"), (p + "bv", (kd,), "bias")]
        if shape.qk_norm:
            out += [(p + "q_norm", (shape.head_dim,), "gain"), (p + "k_norm", (shape.head_dim,), "gain")]
        if shape.is_moe:
            e, fe = shape.n_experts, shape.expert_ffn_dim
            out += [(p + "router", (e, d), "matrix"), (p + "experts.w_gate", (e, fe, d), "matrix"),
                    (p + "experts.w_up", (e, fe, d), "matrix"),
                    (p + "experts.w_down", (e, d, fe), "matrix")]
        else:
            f = shape.ffn_dim
            out += [(p + "w_gate", (f, d), "matrix"), (p + "w_up", (f, d), "matrix"),
                    (p + "w_down", (d, f), "matrix")]
    out += [("final_norm", (d,), "gain")]
    if not shape.tied_lm_head:
        out += [("lm_head", (shape.vocab, d), "matrix")]
    return out


def make_weights(shape: ModelShape, seed: int, gains: str = "varied",
                 threads: int | None = None) -> dict[str, np.ndarray]:
    """Random-init weights as fp32 arrays already rounded to the shape's storage type.

    Matrices and embeddings are N(0, 0.02), biases N(0, 0.2).  Norm gains are 1 + N(0, 0.1) when
    gains == "varied" (so that a dropped gain shows up in parity) and exactly 1 when
    gains == "ones".  Every tensor has its own stream, derived from (seed, position in
    checkpoint order), so generation can run on several threads with a fixed result.
    """
    assert gains in ("varied", "ones")
    layout = weight_layout(shape)

    def one(idx_entry):
        idx, (name, dims, kind) = idx_entry
        rng = np.random.Generator(np.random.Philox(key=[seed, idx]))
        if kind == "gain":
            if gains == "ones":
                w = np.ones(dims, dtype=np.float32)
            else:
                w = (1.0 + 0.1 * rng.standard_normal(dims, dtype=np.float32)).astype(np.float32)
        else:
            w = rng.standard_normal(dims, dtype=np.float32)
            w *= np.float32(0.2 if kind == "bias" else 0.02)
        if shape.dtype == "bf16":
            w = round_to_bf16(w)
        return name, w

    threads = threads or min(16, os.cpu_count() or 1)
    with ThreadPoolExecutor(max_workers=threads) as ex:
        return dict(ex.map(one, enumerate(layout)))


# ----------------------------------------------------------------------------------------
# prompts, lengths, uniforms
# ----------------------------------------------------------------------------------------
def make_prompts(n_prompts: int, min_len: int, max_len: int, vocab: int, seed: int):
    """Token ids uniform over the vocabulary; lengths uniform on [min_len, max_len].

    Returns (tokens int32 [sum len], offsets int32 [n_prompts + 1]).
    """
    rng = np.random.Generator(np.random.Philox(key=[seed, 0x70726f6d]))
    lens = rng.integers(min_len, max_len + 1, size=n_prompts)
    offsets = np.zeros(n_prompts + 1, dtype=np.int32)
    offsets[1:] = np.cumsum(lens)
    tokens = rng.integers(0, vocab, size=int(offsets[-1])).astype(np.int32)
    return tokens, offsets


def geometric_lengths(n: int, mean: float, cap: int, seed: int) -> np.ndarray:
    """P(L = k) = q (1 - q)^(k-1), q = 1 / mean, k >= 1, then min(L, cap)."""
    rng = np.random.Generator(np.random.Philox(key=[seed, 0x67656f6d]))
    return np.minimum(rng.geometric(1.0 / mean, size=n), cap).astype(np.int32)


def lognormal_lengths(n: int, median: float, sigma: float, cap: int, seed: int) -> np.ndarray:
    """L = clamp(round(exp(ln median + sigma Z)), 1, cap), Z standard normal."""
    rng = np.random.Generator(np.random.Philox(key=[seed, 0x6c6f676e]))
    z = rng.standard_normal(n)
    return np.clip(np.rint(np.exp(np.log(median) + sigma * z)), 1, cap).astype(np.int32)


def uniform_words(n: int, seed: int) -> np.ndarray:
    """Raw 32-bit words for driving a sampler directly (the uniform-override input)."""
    rng = np.random.Generator(np.random.Philox(key=[seed, 0x756e6966]))
    return rng.integers(0, 1 << 32, size=n, dtype=np.uint64).astype(np.uint32)


def random_logits(rows: int, vocab: int, seed: int, scale: float = 1.0) -> np.ndarray:
    """fp32 logits rows for sampler-only cases: N(0, scale^2)."""
    rng = np.random.Generator(np.random.Philox(key=[seed, 0x6c6f6769]))
    return (scale * rng.standard_normal((rows, vocab), dtype=np.float32)).astype(np.float32)


@dataclasses.dataclass(frozen=True)
class RolloutLoad:
    """One generation job: prompts, samples per prompt, forced response lengths."""
    name: str
    prompt_tokens: np.ndarray      # int32 [sum prompt len]
    prompt_offsets: np.ndarray     # int32 [P + 1]
    n_samples: int
    max_new_tokens: np.ndarray     # int32 [P * n_samples]; eos disabled, so these are exact
    temperature: float
    top_p: float
    sampler_seed: int

    @property
    def n_prompts(self) -> int:
        return len(self.prompt_offsets) - 1

    @property
    def total_new_tokens(self) -> int:
        return int(self.max_new_tokens.sum())


def load_c1(seed: int = 2) -> RolloutLoad:
    t, o = make_prompts(4, 32, 32, C1_TINY.vocab, seed)
    return RolloutLoad("c1", t, o, 2, np.full(8, 32, np.int32), 1.0, 0.9, 3)


def load_c2(seed: int = 2, n_prompts: int = 32, n_samples: int = 8) -> RolloutLoad:
    t, o = make_prompts(n_prompts, 64, 512, C2_1P5B.vocab, seed)
    lens = geometric_lengths(n_prompts * n_samples, 512.0, 2048, seed)
    return RolloutLoad("c2", t, o, n_samples, lens, 1.0, 1.0, 3)


def load_c3(seed: int = 2, n_prompts: int = 64, n_samples: int = 8) -> RolloutLoad:
    t, o = make_prompts(n_prompts, 128, 1024, C3_7B.vocab, seed)
    lens = lognormal_lengths(n_prompts * n_samples, 1024.0, 1.0, 8192, seed)
    return RolloutLoad("c3", t, o, n_samples, lens, 0.99, 1.0, 3)


def load_c4(seed: int = 2, n_prompts: int = 32, n_samples: int = 16) -> RolloutLoad:
    t, o = make_prompts(n_prompts, 128, 1024, C4_30B_A3B.vocab, seed)
    lens = lognormal_lengths(n_prompts * n_samples, 2048.0, 1.0, 16384, seed)
    return RolloutLoad("c4", t, o, n_samples, lens, 1.0, 1.0, 3)


def packed_sequences(n_seqs: int, min_len: int, max_len: int, vocab: int, seed: int):
    """Teacher-forced log-prob workload: packed token ids and cumulative lengths."""
    rng = np.random.Generator(np.random.Philox(key=[seed, 0x7061636b]))
    lens = rng.integers(min_len, max_len + 1, size=n_seqs)
    cu = np.zeros(n_seqs + 1, dtype=np.int32)
    cu[1:] = np.cumsum(lens)
    tokens = rng.integers(0, vocab, size=int(cu[-1])).astype(np.int32)
    return tokens, cu
