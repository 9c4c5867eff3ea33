"""CPU fp64 oracle for the response-token loss.  TEST INFRASTRUCTURE ONLY: the tests and the
smoke/benchmark checks may call it, the product path never does, and this file imports nothing
from the product package.

What it computes.

* Response-row log-probability (paper Section 4.3, modification 4): the loss is a cross-entropy
  over the RESPONSE tokens of the pack only; prompt rows are discarded.  For a response row t with
  target y_t:  logp_t = z[t, y_t] - log sum_v exp(z[t, v]),  cross-entropy = -logp_t.  What the
  target of a row is (the usual next-token shift) is the caller's business: labels come per row.
  Backward for an upstream gradient g_t = dL/dlogp_t:  dz[t, v] = g_t (1[v = y_t] - softmax(z_t)_v)
  on response rows and 0 on prompt rows.

* The GRPO objective over those log-probabilities (Section 2: J = 1/(NG) sum_k (L_k - beta D_KL^k),
  L_k the clipped surrogate term of response k, D_KL^k its policy-versus-reference KL estimate;
  Appendix hyper-parameters eps_low = eps_high = 0.2, beta = 0.02).  The paper
  does not print L_k and D_KL^k; the reading taken is the GRPO form its training recipe names:
      r_t   = exp(logp_t - logp_old_t)
      L_k   = 1/|o_k| sum_t min(r_t A_k, clip(r_t, 1 - eps_low, 1 + eps_high) A_k)
      D_k   = 1/|o_k| sum_t (exp(ref_t - logp_t) - (ref_t - logp_t) - 1)        (non-negative estimator)
      loss  = -1/R sum_k (L_k - beta D_k),   R = number of non-empty responses in the batch,
  with A_k one advantage per response and |o_k| its token count.  Empty responses contribute nothing.

Pins (tests/test_loss_pins.py): scipy log_softmax; the uniform-logit closed form -log V; torch
autograd for both gradients; r = 1 reduces L_k to A_k and ref = logp makes D_k vanish; the clip is
inactive / active on hand-made cases; the micro-batch identity of Section 2 (the batch objective is
the response-weighted mean of micro-batch objectives).
"""
from __future__ import annotations

from typing import Sequence, Tuple

import numpy as np


def response_index(prompt_lens: Sequence[int], Gs: Sequence[int], resp_lens_flat: Sequence[int]) -> np.ndarray:
    """For every packed token: -1 on a prompt row, else the global index (over all groups, in
    order) of the response it belongs to."""
    out, r = [], 0
    for lp, g in zip(prompt_lens, Gs):
        out.append(np.full(lp, -1, dtype=np.int64))
        for li in resp_lens_flat[r:r + g]:
            out.append(np.full(li, r, dtype=np.int64))
            r += 1
    return np.concatenate(out) if out else np.zeros(0, dtype=np.int64)


def logprob_fwd(logits, labels, resp_idx) -> Tuple[np.ndarray, np.ndarray]:
    """logits [T, V], labels [T] (ignored on prompt rows), resp_idx from response_index.
    Returns (logp [T], lse [T]) in float64, both 0 on prompt rows."""
    z = np.asarray(logits, dtype=np.float64)
    T = z.shape[0]
    logp, lse = np.zeros(T), np.zeros(T)
    for t in range(T):
        if resp_idx[t] < 0:
            continue
        m = z[t].max()
        lse[t] = m + np.log(np.exp(z[t] - m).sum())
        logp[t] = z[t, labels[t]] - lse[t]
    return logp, lse


def logprob_bwd(logits, labels, g, resp_idx) -> np.ndarray:
    """dz [T, V] float64 for upstream g [T] = dL/dlogp."""
    z = np.asarray(logits, dtype=np.float64)
    dz = np.zeros_like(z)
    for t in range(z.shape[0]):
        if resp_idx[t] < 0:
            continue
        m = z[t].max()
        p = np.exp(z[t] - m)
        p /= p.sum()
        dz[t] = -g[t] * p
        dz[t, labels[t]] += g[t]
    return dz


def grpo_loss(logp, logp_old, logp_ref, adv, resp_idx, eps_low: float, eps_high: float, beta: float):
    """Returns (loss, g) with g [T] = dloss/dlogp (0 on prompt rows).  adv [n_responses]."""
    logp, logp_old, logp_ref, adv = (np.asarray(x, dtype=np.float64) for x in (logp, logp_old, logp_ref, adv))
    T = logp.shape[0]
    g = np.zeros(T)
    n_resp = adv.shape[0]
    counts = np.bincount(resp_idx[resp_idx >= 0], minlength=n_resp)
    R = int((counts > 0).sum())
    total = 0.0
    for t in range(T):
        k = resp_idx[t]
        if k < 0:
            continue
        r = np.exp(logp[t] - logp_old[t])
        a = adv[k]
        unclipped, clipped = r * a, np.clip(r, 1.0 - eps_low, 1.0 + eps_high) * a
        surr = min(unclipped, clipped)
        # derivative of the min: the unclipped branch when it is the smaller one (ties go to it),
        # otherwise the clipped branch, which is flat wherever the clip is active
        d_surr = r * a if unclipped <= clipped else (r * a if (1.0 - eps_low) < r < (1.0 + eps_high) else 0.0)
        u = logp_ref[t] - logp[t]
        kl = np.exp(u) - u - 1.0
        d_kl = -np.exp(u) + 1.0
        wgt = 1.0 / (counts[k] * R)
        total += wgt * (surr - beta * kl)
        g[t] = -wgt * (d_surr - beta * d_kl)
    return -total, g
