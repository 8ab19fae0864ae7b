"""Writes single_layer_example.txt: a one-layer, two-token transformer worked by hand.

Straight-line 40-digit arithmetic with mpmath, following the operator definitions
(RMSNorm, half-split RoPE, causal softmax attention, SwiGLU, residuals, final norm,
lm_head).  It calls no code of the oracle or of the library; the oracle is then tested
against the numbers it prints.  (The paper prints no worked example; this one stands in.)

Model: hidden 2, one query head = one KV head of dim 2, eps 0, all gains 1,
W_q = W_k = W_v = W_o = I, W_gate = [1 0], W_up = [0 1], W_down = [1 1]^T, lm_head = I,
theta = 10000 (one rotary pair, so position p rotates by p radians),
embeddings: token 0 -> (3, 4), token 1 -> (1, -2).  Sequence: tokens (0, 1).
"""
import os
import mpmath as mp

mp.mp.dps = 40


def norm2(a, b):
    r = mp.sqrt((a * a + b * b) / 2)
    return a / r, b / r


def rot(a, b, ang):
    return a * mp.cos(ang) - b * mp.sin(ang), b * mp.cos(ang) + a * mp.sin(ang)


def mlp_and_logits(x0, x1):
    h0, h1 = norm2(x0, x1)
    act = h0 / (1 + mp.e ** (-h0)) * h1          # silu(gate) * up
    y0, y1 = x0 + act, x1 + act                   # W_down = [1 1]^T, plus residual
    return norm2(y0, y1)                          # final norm, lm_head = I


def logsoftmax(a, b):
    m = max(a, b)
    lse = m + mp.log(mp.e ** (a - m) + mp.e ** (b - m))
    return a - lse, b - lse


# position 0, token 0
e0 = (mp.mpf(3), mp.mpf(4))
h = norm2(*e0)
k0, v0 = h, h                                     # rotation by 0
x_after_attn = (e0[0] + v0[0], e0[1] + v0[1])     # single key: attention output = v0
logits0 = mlp_and_logits(*x_after_attn)

# position 1, token 1
e1 = (mp.mpf(1), mp.mpf(-2))
h = norm2(*e1)
q1 = rot(h[0], h[1], 1)
k1, v1 = q1, h
s0 = (q1[0] * k0[0] + q1[1] * k0[1]) / mp.sqrt(2)
s1 = (q1[0] * k1[0] + q1[1] * k1[1]) / mp.sqrt(2)
m = max(s0, s1)
p0 = mp.e ** (s0 - m) / (mp.e ** (s0 - m) + mp.e ** (s1 - m))
p1 = 1 - p0
o = (p0 * v0[0] + p1 * v1[0], p0 * v0[1] + p1 * v1[1])
logits1 = mlp_and_logits(e1[0] + o[0], e1[1] + o[1])

lines = ["# single-layer worked example; see derive_single_layer_example.py",
         "# name value"]
for name, val in (("logits_pos0_tok0", logits0[0]), ("logits_pos0_tok1", logits0[1]),
                  ("logprob_pos0_tok0", logsoftmax(*logits0)[0]),
                  ("logprob_pos0_tok1", logsoftmax(*logits0)[1]),
                  ("attn_prob_pos1_key0", p0), ("attn_prob_pos1_key1", p1),
                  ("logits_pos1_tok0", logits1[0]), ("logits_pos1_tok1", logits1[1]),
                  ("logprob_pos1_tok0", logsoftmax(*logits1)[0]),
                  ("logprob_pos1_tok1", logsoftmax(*logits1)[1])):
    lines.append(f"{name} {mp.nstr(val, 25)}")
with open(os.path.join(os.path.dirname(os.path.abspath(__file__)),
                       "single_layer_example.txt"), "w") as fh:
    fh.write("\n".join(lines) + "\n")
