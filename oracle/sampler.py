"""Temperature / top-p sampling with integer weights, and the log-prob of the drawn token.

Test infrastructure.  The paper only says that the actor generates tokens until a
termination criterion is met (section 2.1, "Key Concepts"); it fixes no sampler.  So that
sampled token ids can be compared bit for bit between two implementations, the procedure
is defined on integers:

  1. z_i = logit_i * inv_T (one fp32 multiply), m = max z, d_i = z_i - m (fp32).
  2. w_i = FIXEXP(d_i): t = d_i * log2(e) (fp32 multiply); w_i = 0 when t < -40; else
     n = floor(t), f = t - n (exact), y = P(f) where P is a fixed degree-7 polynomial for
     2^f evaluated by Horner's rule with separately rounded fp32 multiplies and adds, and
     w_i = floor(y * 2^(40 + n)).  S = sum w_i is an integer, so any summation order
     gives the same S.
  3. Nucleus: all tokens with w_i > 0 when top_p >= 1.  Otherwise
     theta = max(1, floor(S * floor(top_p * 2^24) / 2^24)); order tokens by (w descending,
     id ascending); the nucleus is the shortest prefix whose weights sum to >= theta.
  4. Draw: S_N = nucleus weight, R = floor(S_N * x / 2^32) for the 32-bit uniform word x;
     the token is the smallest id j in the nucleus whose nucleus-prefix sum in ascending
     id order exceeds R.
  5. logp = z_tok - logsumexp(z) over the full vocabulary (temperature-scaled, not
     renormalised to the nucleus).

The polynomial coefficients are part of the definition and are typed here as literals.
"""
from __future__ import annotations

import math

import numpy as np

FIX_BITS = 40
LOG2E_F32 = np.float32(float.fromhex("0x1.715476p+0"))
# 2^f on [0, 1): c0 + c1 f + ... + c7 f^7, every coefficient exactly representable in fp32.
EXP2_POLY = tuple(np.float32(float.fromhex(h)) for h in (
    "0x1.000000p+0", "0x1.62e430p-1", "0x1.ebfbdep-3", "0x1.c6b140p-5",
    "0x1.3b1a32p-7", "0x1.5efc6ap-10", "0x1.3262dep-13", "0x1.5bd2aep-16"))


def scaled_logits(logits, inv_t) -> np.ndarray:
    """z = logits * inv_T with one fp32 rounding per element."""
    return np.asarray(logits, dtype=np.float32) * np.float32(inv_t)


def fixexp_weights(logits, inv_t) -> np.ndarray:
    """Integer weights w_i (Python-int-safe uint64 array) of one fp32 logits row."""
    z = scaled_logits(logits, inv_t)
    d = z - np.max(z)                                  # fp32, <= 0
    with np.errstate(invalid="ignore", over="ignore"):
        t = d * LOG2E_F32                              # fp32
        live = t >= np.float32(-FIX_BITS)
        ts = np.where(live, t, np.float32(0))
        n = np.floor(ts)                               # fp32, integer valued
        f = ts - n                                     # exact in fp32, in [0, 1)
        y = np.full_like(f, EXP2_POLY[-1])
        for c in EXP2_POLY[-2::-1]:
            y = y * f                                  # fp32 multiply, rounded
            y = y + c                                  # fp32 add, rounded
        w = np.floor(np.ldexp(y.astype(np.float64), FIX_BITS + n.astype(np.int64)))
    w = w.astype(np.uint64)
    w[~live] = 0
    return w


def top_p_fixed(top_p) -> int:
    """floor(top_p * 2^24) of the fp32 value of top_p."""
    return int(math.floor(float(np.float32(top_p)) * (1 << 24)))


def nucleus_threshold(total: int, top_p) -> int:
    return max(1, (int(total) * top_p_fixed(top_p)) >> 24)


def nucleus(w: np.ndarray, top_p) -> np.ndarray:
    """Boolean membership mask of the nucleus (step 3), by explicit ordering."""
    w = np.asarray(w, dtype=np.uint64)
    if float(np.float32(top_p)) >= 1.0:
        return w > 0
    theta = nucleus_threshold(int(np.sum(w, dtype=np.uint64)), top_p)
    order = np.lexsort((np.arange(len(w)), -w.astype(np.int64)))   # w descending, id ascending
    running = np.cumsum(w[order], dtype=np.uint64)                 # < 2^58, no wrap
    last = int(np.searchsorted(running, np.uint64(theta), side="left"))  # first prefix >= theta
    mask = np.zeros(len(w), dtype=bool)
    mask[order[:last + 1]] = True
    return mask


def draw(w: np.ndarray, mask: np.ndarray, x: int) -> int:
    """Inverse-CDF draw in ascending id order over the nucleus (step 4)."""
    running = np.cumsum(np.where(mask, np.asarray(w, dtype=np.uint64), np.uint64(0)),
                        dtype=np.uint64)
    s_n = int(running[-1])
    assert s_n > 0, "empty nucleus"
    r = (s_n * (int(x) & 0xFFFFFFFF)) >> 32
    return int(np.searchsorted(running, np.uint64(r), side="right"))   # first prefix sum > r


def log_prob(logits, inv_t, token: int) -> float:
    """log softmax(z)[token] over the full vocabulary, in fp64 from the fp32 z."""
    z = scaled_logits(logits, inv_t).astype(np.float64)
    m = np.max(z)
    return float(z[token] - m - np.log(np.sum(np.exp(z - m))))


def sample(logits, inv_t, top_p, x: int):
    """(token id, log-prob) for one logits row, temperature 1/inv_t, top-p, uniform word x."""
    w = fixexp_weights(logits, inv_t)
    tok = draw(w, nucleus(w, top_p), x)
    return tok, log_prob(logits, inv_t, tok)


def inv_temperature(temperature) -> np.float32:
    """inv_T as the path computes it: one fp32 division of 1 by the fp32 temperature."""
    return np.float32(1.0) / np.float32(temperature)
