"""CPU fp64 oracle for rotary position embedding with the shared-prompt position indices.
TEST INFRASTRUCTURE ONLY: the tests and the smoke/benchmark checks may call it, the product
path never does, and this file imports nothing from the product package.

What it computes (paper Section 4.3, modification 2): in the packed sequence
``[prompt | resp_1 | ... | resp_G]`` the prompt keeps positions 0 .. Lp-1 and EVERY response
starts again right after the prompt, ``Lp, Lp+1, ...``, so a response token sits where it would
sit if ``[prompt | resp_i]`` were trained alone.  The paper fixes only these indices; how a
model turns them into an encoding is its own business.  The models it trains (Qwen family) use
rotary embedding in the half-split ("rotate_half") form, which is what is written out here:

    theta_i = base ** (-2 i / d),  i = 0 .. d/2 - 1
    (x'_i, x'_{i+d/2}) = (x_i cos(p theta_i) - x_{i+d/2} sin(p theta_i),
                          x_i sin(p theta_i) + x_{i+d/2} cos(p theta_i))

applied to q and k (never v) at the token's position p.  The rotation is orthogonal, so the
gradient with respect to the unrotated tensor is the rotation by -p theta of the gradient with
respect to the rotated one (``inverse=True``).

Pins (tests/test_rope_pins.py): a hand-computed d = 2 example; norm preservation and
inverse(forward) = identity; scores depend only on position differences; and the property the
restart exists for -- shared-prompt attention over rotated q, k equals G independent causal
attentions over ``[prompt | resp_i]`` with ordinary positions 0 .. Lp+Li-1, forward and backward,
where the per-sample side uses a separately written complex-number rotation.
"""
from __future__ import annotations

from typing import Sequence

import numpy as np


def positions(prompt_len: int, resp_lens: Sequence[int]) -> np.ndarray:
    """Position index of every packed token: 0..Lp-1, then Lp.. for each response anew."""
    parts = [np.arange(prompt_len, dtype=np.int64)]
    for li in resp_lens:
        parts.append(prompt_len + np.arange(li, dtype=np.int64))
    return np.concatenate(parts)


def positions_batched(prompt_lens: Sequence[int], Gs: Sequence[int], resp_lens_flat: Sequence[int]) -> np.ndarray:
    out, r = [], 0
    for lp, g in zip(prompt_lens, Gs):
        out.append(positions(lp, list(resp_lens_flat[r:r + g])))
        r += g
    return np.concatenate(out)


def rope_rotate(x, pos, base: float, inverse: bool = False) -> np.ndarray:
    """x [T, H, d] (any real dtype, widened to float64), pos [T] integers.  Returns the rotated
    tensor in float64.  ``inverse`` rotates by the negative angle."""
    x = np.asarray(x, dtype=np.float64)
    T, H, d = x.shape
    half = d // 2
    assert d == 2 * half
    theta = np.asarray(base, dtype=np.float64) ** (-2.0 * np.arange(half, dtype=np.float64) / d)
    ang = np.asarray(pos, dtype=np.float64)[:, None] * theta[None, :]          # [T, d/2]
    if inverse:
        ang = -ang
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    lo, hi = x[..., :half], x[..., half:]
    return np.concatenate([lo * c - hi * s, lo * s + hi * c], axis=-1)
