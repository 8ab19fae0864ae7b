"""Policy-gradient objective over a batch of rollouts: what the training stage does with the
log-probs the rollout path emits.

Test infrastructure.  The paper states the objective in words only (section 5.1 and section
5.2, training configuration): a PPO loss whose advantage is the REINFORCE return rather than
a GAE estimate, with rewards clipped at 20 and advantages clipped at 10; section 2.1 says the
reference model contributes a KL penalty.  The definitions below are the standard public
ones those words name (Schulman et al. 2017 for the clipped surrogate; Williams 1992 for the
return), written out token by token:

  tokens of one sequence that count are those with mask = 1 (response tokens), in order
  t_1 < ... < t_L; every other token has advantage 0, gradient 0 and no part in the loss.

  reward      rho_j = -kl_coef * (logp_old[t_j] - logp_ref[t_j])   (0 without a reference)
              and the sequence's scalar reward, clipped to [-reward_clip, reward_clip], is
              added to rho_L (it arrives with the last response token)
  return      G_L = rho_L,  G_j = rho_j + gamma * G_{j+1}
  advantage   A_j = clip(G_j, -adv_clip, adv_clip)
  ratio       r_j = exp(logp_new[t_j] - logp_old[t_j])
  surrogate   s_j = min(r_j * A_j, clip(r_j, 1 - eps_low, 1 + eps_high) * A_j)
  loss        -(sum of s over all counted tokens of all sequences) / N,  N = number of them
              (0 when N = 0)
  gradient    d loss / d logp_new[t_j] = -(r_j * A_j) / N where the unclipped term is the
              minimum (r_j * A_j <= clipped term), else 0

The discount, the KL coefficient and the two ratio bounds are parameters: the paper fixes
none of them.
"""
from __future__ import annotations

import numpy as np


def policy_loss(cu_seqlens, logp_new, logp_old, logp_ref, mask, rewards, *, gamma=1.0, kl_coef=0.0,
                reward_clip=20.0, adv_clip=10.0, eps_low=0.2, eps_high=0.2):
    """Returns (loss, grad [T], advantages [T]) in fp64."""
    logp_new = np.asarray(logp_new, np.float64)
    logp_old = np.asarray(logp_old, np.float64)
    ref = None if logp_ref is None else np.asarray(logp_ref, np.float64)
    mask = np.asarray(mask).astype(bool)
    total = len(logp_new)
    adv = np.zeros(total)
    for i in range(len(cu_seqlens) - 1):
        idx = [t for t in range(int(cu_seqlens[i]), int(cu_seqlens[i + 1])) if mask[t]]
        g = 0.0
        for j in range(len(idx) - 1, -1, -1):
            t = idx[j]
            rho = 0.0 if ref is None else -kl_coef * (logp_old[t] - ref[t])
            if j == len(idx) - 1:
                rho += min(max(float(rewards[i]), -reward_clip), reward_clip)
            g = rho + gamma * g
            adv[t] = min(max(g, -adv_clip), adv_clip)
    n = int(mask.sum())
    grad = np.zeros(total)
    if n == 0:
        return 0.0, grad, adv
    loss = 0.0
    for t in np.flatnonzero(mask):
        r = np.exp(logp_new[t] - logp_old[t])
        plain = r * adv[t]
        clipped = min(max(r, 1.0 - eps_low), 1.0 + eps_high) * adv[t]
        loss -= min(plain, clipped)
        if plain <= clipped:
            grad[t] = -plain / n
    return loss / n, grad, adv
