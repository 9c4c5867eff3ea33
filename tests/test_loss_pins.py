"""Pins for the response-token loss oracle (Section 4.3 modification 4; Section 2 objective)."""
import math

import numpy as np
import scipy.special
import torch

from oracle import loss_oracle as lo

PL, GS, RL = [3, 2], [2, 3], [2, 0, 1, 3, 2]


def test_response_index_marks_prompt_rows_and_counts_responses_globally():
    idx = lo.response_index(PL, GS, RL)
    assert idx.tolist() == [-1, -1, -1, 0, 0, -1, -1, 2, 3, 3, 3, 4, 4]


def test_logprob_matches_scipy_and_skips_prompt_rows():
    rng = np.random.default_rng(0)
    idx = lo.response_index(PL, GS, RL)
    T, V = idx.shape[0], 37
    z = rng.standard_normal((T, V)) * 3
    y = rng.integers(0, V, T)
    logp, lse = lo.logprob_fwd(z, y, idx)
    ref = scipy.special.log_softmax(z, axis=1)[np.arange(T), y]
    resp = idx >= 0
    assert np.allclose(logp[resp], ref[resp], atol=1e-13)
    assert np.allclose(lse[resp], scipy.special.logsumexp(z, axis=1)[resp], atol=1e-13)
    assert np.all(logp[~resp] == 0) and np.all(lse[~resp] == 0)


def test_uniform_logits_give_minus_log_vocab():
    idx = lo.response_index([1], [1], [2])
    logp, _ = lo.logprob_fwd(np.full((3, 50), 0.7), np.array([0, 4, 49]), idx)
    assert np.allclose(logp[1:], -math.log(50.0), atol=1e-14)


def test_logprob_gradient_matches_autograd():
    rng = np.random.default_rng(1)
    idx = lo.response_index(PL, GS, RL)
    T, V = idx.shape[0], 11
    z = rng.standard_normal((T, V))
    y = rng.integers(0, V, T)
    g = rng.standard_normal(T)
    zt = torch.tensor(z, requires_grad=True)
    lp = torch.log_softmax(zt, dim=1)[torch.arange(T), torch.tensor(y)]
    (lp * torch.tensor(g) * torch.tensor(idx >= 0, dtype=torch.float64)).sum().backward()
    assert np.allclose(lo.logprob_bwd(z, y, g, idx), zt.grad.numpy(), atol=1e-13)
    assert np.all(lo.logprob_bwd(z, y, g, idx)[idx < 0] == 0)


def torch_grpo(logp, old, ref, adv, idx, el, eh, beta):
    lp = torch.tensor(logp, requires_grad=True)
    total = torch.zeros((), dtype=torch.float64)
    ks = [k for k in range(len(adv)) if (idx == k).any()]
    for k in ks:
        sel = torch.tensor(idx == k)
        r = torch.exp(lp[sel] - torch.tensor(old)[sel])
        a = adv[k]
        surr = torch.minimum(r * a, torch.clamp(r, 1 - el, 1 + eh) * a)
        u = torch.tensor(ref)[sel] - lp[sel]
        kl = torch.exp(u) - u - 1
        total = total + (surr - beta * kl).mean()
    loss = -total / len(ks)
    loss.backward()
    return float(loss.detach()), lp.grad.numpy()


def test_grpo_loss_and_gradient_match_autograd():
    rng = np.random.default_rng(2)
    idx = lo.response_index(PL, GS, RL)
    T = idx.shape[0]
    logp = -np.abs(rng.standard_normal(T)) - 0.1
    old = logp + 0.4 * rng.standard_normal(T)          # ratios on both sides of the clip range
    ref = logp + 0.3 * rng.standard_normal(T)
    adv = rng.standard_normal(len(RL))
    loss, g = lo.grpo_loss(logp, old, ref, adv, idx, 0.2, 0.2, 0.02)
    tl, tg = torch_grpo(logp, old, ref, adv, idx, 0.2, 0.2, 0.02)
    assert abs(loss - tl) < 1e-13
    assert np.allclose(g, tg, atol=1e-13)
    assert np.all(g[idx < 0] == 0)


def test_on_policy_with_reference_equal_to_policy_reduces_to_mean_advantage():
    idx = lo.response_index(PL, GS, RL)
    T = idx.shape[0]
    logp = -np.linspace(0.1, 2.0, T)
    adv = np.array([1.0, 5.0, -2.0, 0.5, 3.0])        # response 1 is empty and must not count
    loss, g = lo.grpo_loss(logp, logp, logp, adv, idx, 0.2, 0.2, 0.02)
    assert abs(loss + (1.0 - 2.0 + 0.5 + 3.0) / 4.0) < 1e-14
    # r = 1: d surr / d logp = A_k, the KL term is stationary
    counts = np.bincount(idx[idx >= 0], minlength=5)
    for t in range(T):
        if idx[t] >= 0:
            assert abs(g[t] + adv[idx[t]] / (counts[idx[t]] * 4)) < 1e-15


def test_clip_hand_cases():
    idx = lo.response_index([0], [1], [1])
    # positive advantage, ratio above 1 + eps: clipped value, zero gradient from the surrogate
    loss, g = lo.grpo_loss([math.log(1.5)], [0.0], [math.log(1.5)], [2.0], idx, 0.2, 0.2, 0.0)
    assert abs(loss + 1.2 * 2.0) < 1e-14 and g[0] == 0.0
    # negative advantage, ratio above 1 + eps: min picks the unclipped (more negative) branch
    loss, g = lo.grpo_loss([math.log(1.5)], [0.0], [math.log(1.5)], [-2.0], idx, 0.2, 0.2, 0.0)
    assert abs(loss - 3.0) < 1e-14 and abs(g[0] - 3.0) < 1e-14
    # KL estimator: ref - logp = u, value exp(u) - u - 1 >= 0
    loss, _ = lo.grpo_loss([0.0], [0.0], [0.5], [0.0], idx, 0.2, 0.2, 1.0)
    assert abs(loss - (math.exp(0.5) - 1.5)) < 1e-14


def test_batch_objective_is_the_response_weighted_mean_of_micro_batches():
    """Section 2: the batch objective equals the mean over micro-batches of their objectives
    (weighted by their response counts when they differ)."""
    rng = np.random.default_rng(3)
    pl, gs, rl = [4], [4], [3, 2, 5, 1]
    idx = lo.response_index(pl, gs, rl)
    T = idx.shape[0]
    logp = -np.abs(rng.standard_normal(T))
    old, ref = logp + 0.3 * rng.standard_normal(T), logp + 0.2 * rng.standard_normal(T)
    adv = rng.standard_normal(4)
    full, _ = lo.grpo_loss(logp, old, ref, adv, idx, 0.2, 0.2, 0.02)
    acc = 0.0
    for members in ([0, 1, 2], [3]):
        rows = np.concatenate([np.arange(4)] + [np.where(idx == k)[0] for k in members])
        midx = lo.response_index([4], [len(members)], [rl[k] for k in members])
        l, _ = lo.grpo_loss(logp[rows], old[rows], ref[rows], adv[members], midx, 0.2, 0.2, 0.02)
        acc += len(members) * l
    assert abs(full - acc / 4) < 1e-13
