"""CPU fp64 oracle for shared-prompt attention.  TEST INFRASTRUCTURE ONLY.

This file is the slow, plain definition that the HIP kernels are checked
against.  Only the tests, the smoke check and the benchmark's CPU-baseline leg
may call it; the product path never does, and this file imports nothing from
the product package.

What it computes (paper Section 4.3):

* Packed input ``x = [x_p, x_r1, ..., x_rG]`` (modification 1): tokens of one
  group are the prompt followed by its G responses, no padding.
* The shared-prompt mask (modification 3 and the paragraph after modification 4):
  a response token attends to the whole prompt and to its own response's tokens
  up to and including itself; it never sees another response.  The prompt is
  causal.  The mask is materialised as an explicit T x T boolean matrix.
* Masked softmax attention with that mask, and its exact gradient.  The paper
  states that the result equals per-sample training exactly (it is not an
  approximation), so the oracle is the textbook definition written out, in float64:

      S = scale * Q K^T          LSE_t = log sum_{s allowed} exp(S_ts)
      P = exp(S - LSE) on allowed pairs, 0 elsewhere          O = P V
      D_t = <dO_t, O_t>          dP = dO V^T          dS = P * (dP - D)
      dQ = scale * dS K          dK = scale * dS^T Q          dV = P^T dO

  For grouped-query attention, q head h reads kv head h // (Hq // Hkv) and the
  kv head's dK/dV sum over its q heads.  For a prompt key the sum over query
  rows runs over the later prompt rows and every row of every response.

Readings taken where the paper is silent: general G >= 1; diagonal included;
LSE is the natural log; zero-length responses and an empty prompt are allowed;
q and k arrive already position-encoded (position ids are applied outside).

Rows of a softmax are independent, so ``row_block`` may split the rows into
chunks purely to bound memory: each row still sees its complete key set in one
piece, there is no running maximum and no rescaling.

Pins (tests/test_oracle_pins.py): equality with G independent causal attentions
over [prompt | resp_i] coded separately; torch-autograd and central finite
differences for the gradients; the uniform-attention closed form; the pair
count of the three complexity terms; textbook reductions (G=1, no responses,
no prompt, MHA); permutation of responses; a cross-response leakage probe.
"""
from __future__ import annotations

from typing import Optional, Sequence, Tuple

import numpy as np


def segment_ids(prompt_len: int, resp_lens: Sequence[int]) -> np.ndarray:
    """seg[t] = 0 for a prompt token, i (1-based) for a token of response i."""
    parts = [np.zeros(prompt_len, dtype=np.int64)]
    for i, li in enumerate(resp_lens):
        parts.append(np.full(li, i + 1, dtype=np.int64))
    return np.concatenate(parts)


def build_mask(prompt_len: int, resp_lens: Sequence[int]) -> np.ndarray:
    """Explicit T x T boolean mask, M[t, s] = True iff query t may attend key s."""
    seg = segment_ids(prompt_len, resp_lens)
    T = seg.shape[0]
    pos = np.arange(T)
    not_future = pos[None, :] <= pos[:, None]
    key_in_prompt = (seg == 0)[None, :]
    same_segment = seg[None, :] == seg[:, None]
    return not_future & (key_in_prompt | same_segment)


def _as64(x) -> np.ndarray:
    if hasattr(x, "detach"):           # a torch tensor (possibly bf16)
        import torch
        return x.detach().to("cpu").to(torch.float64).numpy()
    return np.asarray(x, dtype=np.float64)


def _row_blocks(rows: np.ndarray, row_block: Optional[int]):
    if row_block is None or row_block >= rows.shape[0]:
        yield rows
        return
    for a in range(0, rows.shape[0], row_block):
        yield rows[a:a + row_block]


def _softmax_rows(S: np.ndarray, M: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Masked softmax over the last axis; returns (P, LSE)."""
    S = np.where(M, S, -np.inf)
    m = S.max(axis=1, keepdims=True)
    E = np.exp(S - m)                  # exp(-inf) = 0 on masked pairs
    l = E.sum(axis=1, keepdims=True)
    return E / l, (m + np.log(l))[:, 0]


def sp_attn_fwd(q, k, v, prompt_len: int, resp_lens: Sequence[int], scale: float,
                rows: Optional[Sequence[int]] = None, heads: Optional[Sequence[int]] = None,
                row_block: Optional[int] = None) -> Tuple[np.ndarray, np.ndarray]:
    """Forward for one group.

    q: [T, Hq, d]; k, v: [T, Hkv, d].  Returns O [R, Hs, d] and LSE [Hs, R] in
    float64, where R = len(rows) (default all T rows, in order) and Hs =
    len(heads) (default all Hq q heads, in order).
    """
    q, k, v = _as64(q), _as64(k), _as64(v)
    T, Hq, d = q.shape
    Hkv = k.shape[1]
    assert T == prompt_len + sum(resp_lens) and Hq % Hkv == 0
    rep = Hq // Hkv
    M = build_mask(prompt_len, resp_lens)
    rows = np.arange(T) if rows is None else np.asarray(rows, dtype=np.int64)
    heads = list(range(Hq)) if heads is None else list(heads)
    O = np.zeros((rows.shape[0], len(heads), d))
    LSE = np.zeros((len(heads), rows.shape[0]))
    for hi, h in enumerate(heads):
        g = h // rep
        done = 0
        for rb in _row_blocks(rows, row_block):
            P, lse = _softmax_rows(scale * (q[rb, h, :] @ k[:, g, :].T), M[rb])
            O[done:done + rb.shape[0], hi, :] = P @ v[:, g, :]
            LSE[hi, done:done + rb.shape[0]] = lse
            done += rb.shape[0]
    return O, LSE


def sp_attn_bwd(q, k, v, d_o, prompt_len: int, resp_lens: Sequence[int], scale: float,
                kv_heads: Optional[Sequence[int]] = None, row_block: Optional[int] = None,
                q_heads: Optional[Sequence[int]] = None):
    """Backward for one group, recomputing the forward in float64.

    d_o: [T, Hq, d].  Returns (dQ [T, Hq, d], dK [T, Hkv, d], dV [T, Hkv, d],
    O [T, Hq, d], LSE [Hq, T]).  With ``kv_heads`` given, only those kv heads
    and the q heads that read them are computed; the rest stay zero.  With ``q_heads``
    given, only those q heads contribute (dK/dV are then partial sums over them).
    """
    q, k, v, d_o = _as64(q), _as64(k), _as64(v), _as64(d_o)
    T, Hq, d = q.shape
    Hkv = k.shape[1]
    assert T == prompt_len + sum(resp_lens) and Hq % Hkv == 0
    rep = Hq // Hkv
    M = build_mask(prompt_len, resp_lens)
    kv_heads = list(range(Hkv)) if kv_heads is None else list(kv_heads)
    dQ, dK, dV = np.zeros_like(q), np.zeros_like(k), np.zeros_like(v)
    O, LSE = np.zeros_like(q), np.zeros((Hq, T))
    all_rows = np.arange(T)
    for g in kv_heads:
        for h in range(g * rep, (g + 1) * rep):
            if q_heads is not None and h not in q_heads:
                continue
            for rb in _row_blocks(all_rows, row_block):
                P, lse = _softmax_rows(scale * (q[rb, h, :] @ k[:, g, :].T), M[rb])
                o = P @ v[:, g, :]
                O[rb, h, :], LSE[h, rb] = o, lse
                D = np.sum(d_o[rb, h, :] * o, axis=1, keepdims=True)
                dP = d_o[rb, h, :] @ v[:, g, :].T
                dS = P * (dP - D)
                dQ[rb, h, :] = scale * (dS @ k[:, g, :])
                dK[:, g, :] += scale * (dS.T @ q[rb, h, :])
                dV[:, g, :] += P.T @ d_o[rb, h, :]
    return dQ, dK, dV, O, LSE


def sp_attn_bwd_rows(q, k, v, d_o, prompt_len: int, resp_lens: Sequence[int], scale: float,
                     rows: Sequence[int], heads: Sequence[int]) -> np.ndarray:
    """dQ only, for sampled rows and q heads: dQ[t, h] depends on row t alone.
    Returns [len(rows), len(heads), d] float64."""
    q, k, v, d_o = _as64(q), _as64(k), _as64(v), _as64(d_o)
    T, Hq, d = q.shape
    rep = Hq // k.shape[1]
    M = build_mask(prompt_len, resp_lens)
    rows = np.asarray(rows, dtype=np.int64)
    out = np.zeros((rows.shape[0], len(heads), d))
    for hi, h in enumerate(heads):
        g = h // rep
        P, _ = _softmax_rows(scale * (q[rows, h, :] @ k[:, g, :].T), M[rows])
        o = P @ v[:, g, :]
        D = np.sum(d_o[rows, h, :] * o, axis=1, keepdims=True)
        dS = P * (d_o[rows, h, :] @ v[:, g, :].T - D)
        out[:, hi, :] = scale * (dS @ k[:, g, :])
    return out


def _group_slices(prompt_lens: Sequence[int], Gs: Sequence[int], resp_lens_flat: Sequence[int]):
    base, r0 = 0, 0
    for lp, G in zip(prompt_lens, Gs):
        lens = list(resp_lens_flat[r0:r0 + G])
        n = lp + sum(lens)
        yield slice(base, base + n), lp, lens
        base, r0 = base + n, r0 + G


def sp_attn_fwd_batched(q, k, v, prompt_lens, Gs, resp_lens_flat, scale: float,
                        row_block: Optional[int] = None):
    """Independent groups packed back to back: each group is attended on its own."""
    q, k, v = _as64(q), _as64(k), _as64(v)
    O, LSE = np.zeros_like(q), np.zeros((q.shape[1], q.shape[0]))
    for sl, lp, lens in _group_slices(prompt_lens, Gs, resp_lens_flat):
        O[sl], LSE[:, sl] = sp_attn_fwd(q[sl], k[sl], v[sl], lp, lens, scale, row_block=row_block)
    return O, LSE


def sp_attn_bwd_batched(q, k, v, d_o, prompt_lens, Gs, resp_lens_flat, scale: float,
                        row_block: Optional[int] = None):
    q, k, v, d_o = _as64(q), _as64(k), _as64(v), _as64(d_o)
    dQ, dK, dV = np.zeros_like(q), np.zeros_like(k), np.zeros_like(v)
    O, LSE = np.zeros_like(q), np.zeros((q.shape[1], q.shape[0]))
    for sl, lp, lens in _group_slices(prompt_lens, Gs, resp_lens_flat):
        dQ[sl], dK[sl], dV[sl], O[sl], LSE[:, sl] = sp_attn_bwd(
            q[sl], k[sl], v[sl], d_o[sl], lp, lens, scale, row_block=row_block)
    return dQ, dK, dV, O, LSE
