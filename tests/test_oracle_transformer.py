"""Pins for the CPU oracle's transformer forward (no GPU).

Each test holds the oracle to something it did not compute itself: closed forms,
invariants, library routines (torch's fp64 CPU ops), brute-force recompute, and a worked
example derived separately with 40-digit arithmetic (tests/golden/).
"""
import dataclasses

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import workloads
from conftest import read_golden_table
from oracle import transformer as T

NANO = workloads.ModelShape("nano", 2, 24, 4, 2, 8, 40, 50, dtype="fp32", rope_theta=10000.0)
NANO_MOE = workloads.ModelShape("nano-moe", 2, 24, 4, 2, 8, 0, 50, dtype="fp32",
                                n_experts=6, top_k=2, expert_ffn_dim=12, rope_theta=10000.0)


def make(shape, seed=1, scale=8.0):
    w = workloads.make_weights(shape, seed)
    # N(0, 0.02) at these tiny widths gives near-zero logits; scale matrices up so that
    # attention and routing are far from uniform and mistakes are visible.
    for k in w:
        if w[k].ndim > 1:
            w[k] = (w[k] * np.float32(scale)).astype(np.float32)
    return T.Model(shape, w)


# ---------------------------------------------------------------- closed forms per operator
def test_softmax_closed_forms():
    rng = np.random.default_rng(0)
    s = rng.standard_normal((5, 9))
    assert np.allclose(T.softmax(s).sum(-1), 1.0, atol=1e-15)
    assert np.allclose(T.softmax(np.full((2, 7), 3.25)), 1.0 / 7)
    hot = np.zeros(6); hot[4] = 800.0
    assert np.allclose(T.softmax(hot), np.eye(6)[4])
    assert np.allclose(T.softmax(s), torch.softmax(torch.from_numpy(s), -1).numpy(), atol=1e-15)


def test_rmsnorm_invariants_and_library():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((4, 16))
    y = T.rmsnorm(x, np.ones(16), 0.0)
    assert np.allclose(np.mean(y * y, -1), 1.0, atol=1e-14)
    assert np.allclose(T.rmsnorm(7.5 * x, np.ones(16), 0.0), y, atol=1e-14)
    g = rng.standard_normal(16)
    ref = F.rms_norm(torch.from_numpy(x), (16,), torch.from_numpy(g), eps=1e-3).numpy()
    assert np.allclose(T.rmsnorm(x, g, 1e-3), ref, atol=1e-14)


def test_silu_values():
    assert T.silu(np.array(0.0)) == 0.0
    assert abs(T.silu(np.array(40.0)) - 40.0) < 1e-12
    assert abs(T.silu(np.array(1.0)) - 1.0 / (1.0 + np.exp(-1.0))) < 1e-16
    a = np.linspace(-6, 6, 25)
    assert np.allclose(T.silu(a), F.silu(torch.from_numpy(a)).numpy(), atol=1e-15)


def test_rope_properties():
    rng = np.random.default_rng(2)
    q = rng.standard_normal((1, 1, 16)); k = rng.standard_normal((1, 1, 16))
    assert np.allclose(T.rope(q, np.array([0]), 1e4), q)                        # pos 0 = identity
    for m, n in ((5, 2), (105, 102), (40, 37)):                                 # depends on m - n only
        a = np.sum(T.rope(q, np.array([m]), 1e4) * T.rope(k, np.array([n]), 1e4))
        b = np.sum(T.rope(q, np.array([3]), 1e4) * T.rope(k, np.array([0]), 1e4))
        assert abs(a - b) < 1e-12
    assert abs(np.linalg.norm(T.rope(q, np.array([77]), 1e4)) - np.linalg.norm(q)) < 1e-13
    # closed form: pair (u_i, u_{i+dh/2}) as a complex number times exp(i pos theta^(-2i/dh))
    z = (q[0, 0, :8] + 1j * q[0, 0, 8:]) * np.exp(1j * 9 * 1e4 ** (-2.0 * np.arange(8) / 16))
    assert np.allclose(T.rope(q, np.array([9]), 1e4)[0, 0], np.concatenate([z.real, z.imag]))


def test_route_topk_and_ties():
    r = np.array([0.5, 2.0, 2.0, -1.0, 2.0, 0.1])
    experts, mix = T.route(r, 2)
    assert list(experts) == [1, 2]                     # ties go to the lower index
    assert np.allclose(mix, [0.5, 0.5]) and abs(mix.sum() - 1) < 1e-15
    experts, mix = T.route(r, 6)                       # k = E: plain softmax over all experts
    assert np.allclose(mix[np.argsort(experts)], T.softmax(r))
    vals, idx = torch.topk(torch.tensor([0.5, 2.5, 2.0, -1.0, 3.0, 0.1]), 3)
    e2, _ = T.route(np.array([0.5, 2.5, 2.0, -1.0, 3.0, 0.1]), 3)
    assert list(e2) == idx.tolist()


def test_routing_gaps_accept_the_top_k_and_nothing_else():
    """The validity check the GPU's recorded expert sets go through: both gaps are <= 0 for
    the top-k (whatever member a tie picks) and for no other set; a set that swaps the best
    expert for the runner-up of a near-tie at the k-th place - which looks harmless to a check
    of the weakest member alone - shows in the second gap."""
    import itertools
    r = np.array([3.0, 2.0, 1.0 + 1e-9, 1.0, -0.5, 0.2])
    k = 3
    top = set(T.route(r, k)[0].tolist())
    assert top == {0, 1, 2}
    for chosen in itertools.combinations(range(len(r)), k):
        below, outside = T.routing_gaps(r, chosen, k)
        assert (max(below, outside) <= 0) == (set(chosen) == top)
        # brute force of the two definitions
        worst_member = min(r[list(chosen)])
        assert below == np.sort(r)[::-1][k - 1] - worst_member
        assert outside == max(r[i] for i in range(len(r)) if i not in chosen) - worst_member
    below, outside = T.routing_gaps(r, [1, 2, 3], k)       # dropped the best expert, kept the near-tie pair
    assert below <= 1e-8 and outside == 3.0 - 1.0
    tie = np.array([1.0, 2.0, 1.0, 0.0])
    assert max(T.routing_gaps(tie, [1, 0], 2)) <= 0 and max(T.routing_gaps(tie, [1, 2], 2)) <= 0
    assert T.routing_gaps(np.array([0.3, 0.1]), [0, 1], 2) == (0.0, -np.inf)   # k = E: nothing is left out


# ---------------------------------------------------------------- whole forward vs library routines
def torch_forward(shape, w, tokens):
    """The same network composed from torch library routines in fp64."""
    tw = {k: torch.from_numpy(v).double() for k, v in w.items()}
    tok = torch.as_tensor(np.asarray(tokens), dtype=torch.long)
    n, dh, half = len(tok), shape.head_dim, shape.head_dim // 2
    ang = torch.arange(n, dtype=torch.float64)[:, None] * \
        shape.rope_theta ** (-2.0 * torch.arange(half, dtype=torch.float64) / dh)
    rot = torch.polar(torch.ones_like(ang), ang)[:, None, :]                    # [n][1][half]

    def rope(u):
        z = torch.complex(u[..., :half], u[..., half:]) * rot
        return torch.cat([z.real, z.imag], -1)

    x = F.embedding(tok, tw["embed"])
    for i in range(shape.n_layers):
        p = f"layers.{i}."
        h = F.rms_norm(x, (shape.hidden,), tw[p + "norm1"], eps=shape.rms_eps)
        bias = (lambda b: tw[p + b]) if shape.qkv_bias else (lambda b: None)
        q = F.linear(h, tw[p + "wq"], bias("bq")).view(n, shape.n_q_heads, dh)
        k = F.linear(h, tw[p + "wk"], bias("bk")).view(n, shape.n_kv_heads, dh)
        v = F.linear(h, tw[p + "wv"], bias("bv")).view(n, shape.n_kv_heads, dh)
        if shape.qk_norm:
            q = F.rms_norm(q, (dh,), tw[p + "q_norm"], eps=shape.rms_eps)
            k = F.rms_norm(k, (dh,), tw[p + "k_norm"], eps=shape.rms_eps)
        q, k = rope(q), rope(k)
        o = F.scaled_dot_product_attention(q.transpose(0, 1)[None], k.transpose(0, 1)[None],
                                           v.transpose(0, 1)[None], is_causal=True,
                                           enable_gqa=True)[0].transpose(0, 1).reshape(n, -1)
        x = x + F.linear(o, tw[p + "wo"])
        h = F.rms_norm(x, (shape.hidden,), tw[p + "norm2"], eps=shape.rms_eps)
        x = x + F.linear(F.silu(F.linear(h, tw[p + "w_gate"])) * F.linear(h, tw[p + "w_up"]),
                         tw[p + "w_down"])
    return F.linear(F.rms_norm(x, (shape.hidden,), tw["final_norm"], eps=shape.rms_eps),
                    tw["embed" if shape.tied_lm_head else "lm_head"]).numpy()


FAMILY_VARIANTS = {"plain": {}, "qkv-bias": dict(qkv_bias=True), "qk-norm": dict(qk_norm=True),
                   "tied": dict(tied_lm_head=True), "all": dict(qkv_bias=True, qk_norm=True, tied_lm_head=True)}


@pytest.mark.parametrize("variant", list(FAMILY_VARIANTS))
def test_forward_full_matches_library_composition(variant):
    shape = dataclasses.replace(NANO, **FAMILY_VARIANTS[variant])
    m = make(shape)
    tokens = np.random.default_rng(3).integers(0, shape.vocab, 11)
    ref = torch_forward(shape, m._w, tokens)
    got = T.forward_full(m, tokens)
    assert np.std(ref) > 0.05
    assert np.allclose(got, ref, atol=1e-12)
    if variant not in ("plain", "tied"):   # the option changes the function: it is not silently ignored
        base = T.forward_full(T.Model(dataclasses.replace(NANO, tied_lm_head=shape.tied_lm_head), m._w), tokens)
        assert np.max(np.abs(base - got)) > 1e-3


def test_family_options_closed_forms():
    """Zero projection matrices leave q = bq, k = bk, v = bv: every position attends uniformly
    (all scores equal after the rotation only if bk = 0, so take bk = 0) and the attention
    output is bv for every head; QK-norm makes the scores invariant to the scale of wq and wk;
    with a tied head and an identity final norm the logits of a one-hot-free state are x . E^T."""
    shape = dataclasses.replace(NANO, n_layers=1, qkv_bias=True)
    w = workloads.make_weights(shape, 5)
    for k in ("wq", "wk", "wv"):
        w["layers.0." + k][:] = 0
    w["layers.0.bk"][:] = 0
    m = T.Model(shape, w)
    x = np.random.default_rng(1).standard_normal((5, shape.hidden))
    q, k, v = m.qkv(0, x, np.arange(5))
    assert np.allclose(k, 0) and np.allclose(v.reshape(5, -1), w["layers.0.bv"].astype(np.float64))
    assert np.allclose(np.linalg.norm(q.reshape(5, -1), axis=1), np.linalg.norm(w["layers.0.bq"].astype(np.float64)))
    shape = dataclasses.replace(NANO, qk_norm=True)
    m1 = make(shape)
    w2 = {k: v.copy() for k, v in m1._w.items()}
    for i in range(shape.n_layers):
        w2[f"layers.{i}.wq"] *= np.float32(4.0)      # exact in fp32: logits must not move
        w2[f"layers.{i}.wk"] *= np.float32(0.25)
    tokens = np.random.default_rng(2).integers(0, shape.vocab, 9)
    shape0 = dataclasses.replace(shape, rms_eps=0.0)
    a, b = T.forward_full(T.Model(shape0, m1._w), tokens), T.forward_full(T.Model(shape0, w2), tokens)
    assert np.allclose(a, b, atol=1e-9)
    shape = dataclasses.replace(NANO, tied_lm_head=True)
    m = make(shape)
    assert "lm_head" not in m._w
    x = np.random.default_rng(3).standard_normal((4, shape.hidden))
    want = T.rmsnorm(x, m.w("final_norm"), shape.rms_eps) @ m.w("embed").T
    assert np.allclose(m.logits(x), want, atol=1e-13)


def test_hand_worked_single_layer_example():
    gold = read_golden_table("single_layer_example.txt")
    shape = workloads.ModelShape("hand", 1, 2, 1, 1, 2, 1, 2, dtype="fp32", rms_eps=0.0,
                                 rope_theta=10000.0)
    eye = np.eye(2, dtype=np.float32)
    w = {"embed": np.array([[3, 4], [1, -2]], np.float32), "layers.0.norm1": np.ones(2, np.float32),
         "layers.0.wq": eye, "layers.0.wk": eye, "layers.0.wv": eye, "layers.0.wo": eye,
         "layers.0.norm2": np.ones(2, np.float32),
         "layers.0.w_gate": np.array([[1, 0]], np.float32),
         "layers.0.w_up": np.array([[0, 1]], np.float32),
         "layers.0.w_down": np.array([[1], [1]], np.float32),
         "final_norm": np.ones(2, np.float32), "lm_head": eye}
    model = T.Model(shape, w)
    logits = T.forward_full(model, [0, 1])
    for pos in (0, 1):
        for tok in (0, 1):
            assert abs(logits[pos, tok] - gold[f"logits_pos{pos}_tok{tok}"]) < 1e-13
    lp = T.packed_log_probs(model, [0, 1], [0, 2])
    assert lp[0] == 0.0 and abs(lp[1] - gold["logprob_pos0_tok1"]) < 1e-13
    # the incremental evaluation walks the same example one token at a time
    fwd = T.KVForward(model)
    cache = fwd.new_cache()
    a = fwd.extend([cache], [[0]])[0][0]
    b = fwd.extend([cache], [[1]])[0][0]
    assert abs(a[1] - gold["logits_pos0_tok1"]) < 1e-13
    assert abs(b[0] - gold["logits_pos1_tok0"]) < 1e-13 and abs(b[1] - gold["logits_pos1_tok1"]) < 1e-13


# ---------------------------------------------------------------- invariants of the whole forward
@pytest.mark.parametrize("shape", [NANO, NANO_MOE], ids=["dense", "moe"])
def test_causal_mask_invariance(shape):
    m = make(shape)
    rng = np.random.default_rng(4)
    a = rng.integers(0, shape.vocab, 10)
    b = a.copy(); b[6:] = rng.integers(0, shape.vocab, 4)
    la, lb = T.forward_full(m, a), T.forward_full(m, b)
    assert np.allclose(la[:6], lb[:6], atol=1e-13, rtol=0)
    assert not np.allclose(la[6:], lb[6:], atol=1e-3)
    assert np.allclose(T.forward_full(m, a[:6]), la[:6], atol=1e-13, rtol=0)


@pytest.mark.parametrize("shape", [NANO, NANO_MOE, workloads.C1_TINY], ids=["dense", "moe", "c1"])
def test_incremental_equals_full_recompute(shape):
    m = make(shape, scale=8.0 if shape is not workloads.C1_TINY else 1.0)
    rng = np.random.default_rng(5)
    seqs = [rng.integers(0, shape.vocab, n) for n in (9, 5)]
    fwd = T.KVForward(m)
    caches = [fwd.new_cache(), fwd.new_cache()]
    out = fwd.extend(caches, [s[:4] for s in seqs])                 # prefill 4 tokens each
    got = [list(o) for o in out]
    for t in range(4, 9):                                           # ragged decode
        live = [i for i, s in enumerate(seqs) if t < len(s)]
        step = fwd.extend([caches[i] for i in live], [[seqs[i][t]] for i in live])
        for i, o in zip(live, step):
            got[i].append(o[0])
    for s, g in zip(seqs, got):
        assert np.allclose(np.stack(g), T.forward_full(m, s), atol=1e-12, rtol=0)


def test_shared_prefix_fork_equals_independent_runs():
    m = make(NANO)
    rng = np.random.default_rng(6)
    prompt = rng.integers(0, NANO.vocab, 7)
    tails = [rng.integers(0, NANO.vocab, 3) for _ in range(3)]
    fwd = T.KVForward(m)
    prefix = fwd.new_cache()
    fwd.extend([prefix], [prompt])
    for tail in tails:
        c = prefix.fork()
        got = fwd.extend([c], [tail])[0]
        ref = T.forward_full(m, np.concatenate([prompt, tail]))[7:]
        assert np.allclose(got, ref, atol=1e-12, rtol=0)
    assert prefix.length == 7 and prefix.k[0].shape[0] == 7          # forks left the prefix alone


@pytest.mark.parametrize("shape", [NANO, NANO_MOE], ids=["dense", "moe"])
def test_multi_turn_growth_equals_full_recompute(shape):
    """The multi-turn pattern - prefill, single-token steps, a block of several tokens appended to
    the grown cache, single-token steps again, two caches of different lengths side by side -
    gives the logits of one full forward over the concatenated sequence."""
    m = make(shape, scale=8.0)
    rng = np.random.default_rng(11)
    seqs = [rng.integers(0, shape.vocab, n) for n in (17, 12)]
    cuts = [(5, 7, 13), (3, 4, 10)]          # prefill | steps | block | steps
    fwd = T.KVForward(m)
    caches = [fwd.new_cache(), fwd.new_cache()]
    got = [list(o) for o in fwd.extend(caches, [s[:c[0]] for s, c in zip(seqs, cuts)])]
    for i, (s, c) in enumerate(zip(seqs, cuts)):
        for t in range(c[0], c[1]):
            got[i].append(fwd.extend([caches[i]], [[s[t]]])[0][0])
    for i, o in enumerate(fwd.extend(caches, [s[c[1]:c[2]] for s, c in zip(seqs, cuts)])):
        got[i].extend(o)
    for i, (s, c) in enumerate(zip(seqs, cuts)):
        for t in range(c[2], len(s)):
            got[i].append(fwd.extend([caches[i]], [[s[t]]])[0][0])
    for s, g in zip(seqs, got):
        assert np.allclose(np.stack(g), T.forward_full(m, s), atol=1e-12, rtol=0)


def test_gqa_reduces_to_mha_with_duplicated_kv_heads():
    m = make(NANO)
    mha_shape = dataclasses.replace(NANO, n_kv_heads=4)
    w2 = dict(m._w)
    for i in range(NANO.n_layers):
        for n in ("wk", "wv"):
            a = m._w[f"layers.{i}.{n}"].reshape(2, 8, 24)
            w2[f"layers.{i}.{n}"] = np.repeat(a, 2, axis=0).reshape(32, 24)
    tokens = np.random.default_rng(7).integers(0, NANO.vocab, 8)
    assert np.allclose(T.forward_full(m, tokens), T.forward_full(T.Model(mha_shape, w2), tokens),
                       atol=1e-12, rtol=0)


def test_moe_with_identical_experts_is_the_dense_ffn():
    m = make(NANO_MOE)
    w = dict(m._w)
    dense_shape = dataclasses.replace(NANO_MOE, n_experts=0, top_k=0, expert_ffn_dim=0, ffn_dim=12)
    wd = {k: v for k, v in w.items() if "experts" not in k and "router" not in k}
    for i in range(NANO_MOE.n_layers):
        p = f"layers.{i}."
        for n in ("w_gate", "w_up", "w_down"):
            w[p + "experts." + n] = np.repeat(w[p + "experts." + n][:1], 6, axis=0)
            wd[p + n] = w[p + "experts." + n][0]
    tokens = np.random.default_rng(8).integers(0, NANO_MOE.vocab, 6)
    assert np.allclose(T.forward_full(T.Model(NANO_MOE, w), tokens),
                       T.forward_full(T.Model(dense_shape, wd), tokens), atol=1e-12, rtol=0)


def test_moe_full_k_is_softmax_weighted_sum_of_all_experts():
    shape = dataclasses.replace(NANO_MOE, top_k=6, n_layers=1)
    m = make(shape)
    h = np.random.default_rng(9).standard_normal((3, 24))
    r = h @ m.w("layers.0.router").T
    mix = torch.softmax(torch.from_numpy(r), -1).numpy()
    ref = np.zeros_like(h)
    for e in range(6):
        g, u, d = (m.w("layers.0.experts." + n)[e] for n in ("w_gate", "w_up", "w_down"))
        ref += mix[:, e:e + 1] * ((T.silu(h @ g.T) * (h @ u.T)) @ d.T)
    assert np.allclose(m.ffn(0, h), ref, atol=1e-12)


def test_packed_log_probs_match_incremental_and_normalise():
    m = make(NANO)
    rng = np.random.default_rng(10)
    toks = rng.integers(0, NANO.vocab, 13)
    cu = np.array([0, 5, 6, 13])
    lp = T.packed_log_probs(m, toks, cu, temperature=0.7)
    assert lp[0] == lp[5] == lp[6] == 0.0
    fwd = T.KVForward(m)
    for a, b in zip(cu[:-1], cu[1:]):
        logits = fwd.extend([fwd.new_cache()], [toks[a:b]])[0]
        ref = torch.log_softmax(torch.from_numpy(logits / 0.7), -1).numpy()
        for t in range(a + 1, b):
            assert abs(lp[t] - ref[t - a - 1, toks[t]]) < 1e-12
        assert np.allclose(np.exp(ref).sum(-1), 1.0)
