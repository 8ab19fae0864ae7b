"""Pins for the oracle's policy-gradient objective (no GPU): closed forms, a composition of
torch's fp64 library routines, finite differences."""
import numpy as np
import pytest
import torch

from oracle import policy_loss as PL


def batch(seed, n_seqs=5, with_ref=True):
    rng = np.random.default_rng(seed)
    lens = rng.integers(3, 40, n_seqs)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    total = int(cu[-1])
    mask = np.zeros(total, np.uint8)
    for i in range(n_seqs):                       # a prompt, then the response; one sequence with holes
        p = rng.integers(1, lens[i])
        mask[cu[i] + p:cu[i + 1]] = 1
    mask[cu[1] + 1:cu[2]:2] = 0                   # observation tokens inside a response do not count
    old = -rng.gamma(2.0, 1.0, total)
    new = old + 0.3 * rng.standard_normal(total)
    ref = old + 0.2 * rng.standard_normal(total) if with_ref else None
    rewards = rng.standard_normal(n_seqs) * 15.0  # some beyond the clip at 20
    rewards[0] = 31.0
    return cu, new, old, ref, mask, rewards


def test_on_policy_no_discount_closed_form():
    """new = old: ratio 1, never clipped.  gamma = 1, no KL: every counted token of a sequence
    carries the sequence's clipped reward, clipped again as an advantage."""
    cu, new, old, ref, mask, rewards = batch(1)
    loss, grad, adv = PL.policy_loss(cu, old, old, None, mask, rewards)
    n = mask.sum()
    want = np.zeros(len(old))
    for i in range(len(rewards)):
        want[cu[i]:cu[i + 1]] = np.clip(np.clip(rewards[i], -20, 20), -10, 10)
    want *= mask
    assert np.allclose(adv, want, atol=0, rtol=0)
    assert np.isclose(loss, -want.sum() / n, rtol=1e-15) and np.allclose(grad, -want / n, rtol=1e-15)
    assert adv[cu[0]:cu[1]].max() == 10.0 and rewards[0] > 20      # both clips bite on sequence 0


def test_discounted_terminal_reward_is_geometric():
    cu = np.array([0, 9], np.int32)
    mask = np.array([0, 0, 1, 1, 0, 1, 1, 1, 0], np.uint8)          # 5 counted tokens, holes skipped
    z = np.zeros(9)
    loss, grad, adv = PL.policy_loss(cu, z, z, None, mask, [8.0], gamma=0.5, adv_clip=100.0)
    assert np.allclose(adv[mask.astype(bool)], 8.0 * 0.5 ** np.arange(4, -1, -1), rtol=1e-15)
    assert np.all(adv[~mask.astype(bool)] == 0)


def test_kl_reward_to_go_against_library_scan():
    """gamma = 1 with a KL penalty: the return is a reversed cumulative sum - torch's flip /
    cumsum in fp64 - and the surrogate is torch's min / clamp / exp."""
    cu, new, old, ref, mask, rewards = batch(2)
    kl, lo, hi = 0.05, 0.2, 0.28
    loss, grad, adv = PL.policy_loss(cu, new, old, ref, mask, rewards, kl_coef=kl, eps_low=lo, eps_high=hi)
    tn, to, tr = (torch.tensor(a, dtype=torch.float64) for a in (new, old, ref))
    tm = torch.tensor(mask.astype(bool))
    tn.requires_grad_(True)
    rho = -kl * (to - tr) * tm
    for i in range(len(rewards)):
        last = int(np.flatnonzero(mask[cu[i]:cu[i + 1]])[-1]) + int(cu[i])
        rho[last] += float(np.clip(rewards[i], -20, 20))
    ret = torch.cat([torch.flip(torch.cumsum(torch.flip(rho[cu[i]:cu[i + 1]], [0]), 0), [0])
                     for i in range(len(rewards))])
    tadv = torch.clamp(ret, -10.0, 10.0) * tm
    ratio = torch.exp(tn - to)
    s = torch.minimum(ratio * tadv, torch.clamp(ratio, 1 - lo, 1 + hi) * tadv)
    tloss = -(s * tm).sum() / tm.sum()
    tloss.backward()
    assert np.allclose(adv, tadv.numpy(), rtol=1e-13, atol=1e-13)
    assert np.isclose(loss, float(tloss.detach()), rtol=1e-13)
    assert np.allclose(grad, tn.grad.numpy(), rtol=1e-12, atol=1e-15)
    assert (grad == 0).sum() > (mask == 0).sum()          # some counted tokens sit on a clipped branch


@pytest.mark.parametrize("a,r,clipped", [(2.0, 1.5, True), (2.0, 0.5, False), (-2.0, 0.5, True), (-2.0, 1.5, False),
                                         (2.0, 1.1, False), (-2.0, 0.9, False)])
def test_clip_branches(a, r, clipped):
    """One token: positive advantage is capped from above at 1 + eps, negative advantage from
    below at 1 - eps; the other side stays unclipped (the pessimistic minimum)."""
    loss, grad, adv = PL.policy_loss([0, 1], [np.log(r)], [0.0], None, [1], [a], eps_low=0.2, eps_high=0.2)
    assert adv[0] == a
    if clipped:
        assert np.isclose(loss, -a * (1.2 if a > 0 else 0.8)) and grad[0] == 0.0
    else:
        assert np.isclose(loss, -a * r) and np.isclose(grad[0], -a * r)


def test_gradient_by_finite_differences_and_empty_batch():
    cu, new, old, ref, mask, rewards = batch(3)
    args = dict(gamma=0.97, kl_coef=0.02)
    loss, grad, _ = PL.policy_loss(cu, new, old, ref, mask, rewards, **args)
    h = 1e-6
    for t in np.random.default_rng(0).choice(len(new), 12, replace=False):
        up, dn = new.copy(), new.copy()
        up[t] += h
        dn[t] -= h
        fd = (PL.policy_loss(cu, up, old, ref, mask, rewards, **args)[0]
              - PL.policy_loss(cu, dn, old, ref, mask, rewards, **args)[0]) / (2 * h)
        assert np.isclose(fd, grad[t], rtol=1e-5, atol=1e-9)
    loss, grad, adv = PL.policy_loss(cu, new, old, ref, np.zeros_like(mask), rewards)
    assert loss == 0.0 and not grad.any() and not adv.any()
