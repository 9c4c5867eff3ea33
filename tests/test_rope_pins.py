"""Pins for the rotary-embedding oracle with restarted position indices (Section 4.3,
modification 2).  Every check compares oracle/rope_oracle.py with something that is not it:
a hand-computed value, an algebraic invariant, or a separately written per-sample pipeline
that rotates with complex numbers and ordinary positions."""
import math

import numpy as np
import scipy.special
import torch

from oracle import rope_oracle as rope
from oracle import sp_attn_oracle as orc


def test_positions_restart_after_the_prompt():
    p = rope.positions(3, [2, 0, 4])
    assert p.tolist() == [0, 1, 2, 3, 4, 3, 4, 5, 6]
    assert rope.positions(0, [2, 1]).tolist() == [0, 1, 0]
    pb = rope.positions_batched([3, 1], [2, 1], [2, 1, 2])
    assert pb.tolist() == [0, 1, 2, 3, 4, 3, 0, 1, 2]


def test_hand_computed_rotation_d2_and_d4():
    # d = 2: one pair, theta_0 = 1, so position p turns (1, 0) into (cos p, sin p)
    x = np.array([[[1.0, 0.0]], [[0.0, 2.0]]])
    y = rope.rope_rotate(x, [3, 1], base=10000.0)
    assert np.allclose(y[0, 0], [math.cos(3.0), math.sin(3.0)], atol=1e-15)
    assert np.allclose(y[1, 0], [-2.0 * math.sin(1.0), 2.0 * math.cos(1.0)], atol=1e-15)
    # d = 4, base 100: theta = (1, 100^-0.5 = 0.1); pairs are (0, 2) and (1, 3)
    x = np.array([[[1.0, 2.0, 3.0, 4.0]]])
    y = rope.rope_rotate(x, [5], base=100.0)
    c0, s0, c1, s1 = math.cos(5.0), math.sin(5.0), math.cos(0.5), math.sin(0.5)
    assert np.allclose(y[0, 0], [1 * c0 - 3 * s0, 2 * c1 - 4 * s1, 1 * s0 + 3 * c0, 2 * s1 + 4 * c1], atol=1e-14)


def test_rotation_is_orthogonal_and_inverse_undoes_it():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((17, 3, 16))
    pos = rng.integers(0, 20000, 17)
    y = rope.rope_rotate(x, pos, 1e6)
    assert np.allclose(np.linalg.norm(y, axis=-1), np.linalg.norm(x, axis=-1), rtol=1e-13)
    assert np.allclose(rope.rope_rotate(y, pos, 1e6, inverse=True), x, atol=1e-12)
    # <R x, g> = <x, R^T g>: the inverse is the transpose, which is what the backward uses
    g = rng.standard_normal(x.shape)
    assert np.isclose(np.sum(y * g), np.sum(x * rope.rope_rotate(g, pos, 1e6, inverse=True)), rtol=1e-12)


def test_scores_depend_on_position_differences_only():
    rng = np.random.default_rng(1)
    q, k = rng.standard_normal((6, 2, 8)), rng.standard_normal((6, 2, 8))
    pos = np.array([0, 1, 2, 7, 8, 30])
    s0 = np.einsum("thd,shd->hts", rope.rope_rotate(q, pos, 1e4), rope.rope_rotate(k, pos, 1e4))
    s1 = np.einsum("thd,shd->hts", rope.rope_rotate(q, pos + 1234, 1e4), rope.rope_rotate(k, pos + 1234, 1e4))
    assert np.allclose(s0, s1, atol=1e-10)


# ---- independent per-sample pipeline: complex rotation, ordinary positions, plain causal attention
def complex_rope(x, base):
    n, H, d = x.shape
    z = x[..., : d // 2] + 1j * x[..., d // 2:]
    w = np.exp(1j * np.arange(n)[:, None] * (base ** (-np.arange(d // 2) / (d / 2)))[None, :])
    z = z * w[:, None, :]
    return np.concatenate([z.real, z.imag], axis=-1)


def per_sample_loss_and_grads(q, k, v, d_o, scale, base):
    """sum(O * dO) of ordinary causal attention over one sample with rotary positions 0..n-1,
    and its gradients w.r.t. the UNROTATED q, k, v, by torch autograd through a complex rotation."""
    qt, kt, vt = (torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in (q, k, v))
    n, Hq, d = q.shape
    rep = Hq // k.shape[1]
    half = d // 2
    ang = torch.arange(n, dtype=torch.float64)[:, None] * (base ** (-torch.arange(half, dtype=torch.float64) / half))[None, :]
    w = torch.polar(torch.ones_like(ang), ang)[:, None, :]
    def rot(x):
        z = torch.complex(x[..., :half], x[..., half:]) * w
        return torch.cat([z.real, z.imag], dim=-1)
    qr, kr = rot(qt), rot(kt).repeat_interleave(rep, dim=1)
    ve = vt.repeat_interleave(rep, dim=1)
    s = scale * torch.einsum("thd,shd->hts", qr, kr)
    s = s.masked_fill(~torch.tril(torch.ones(n, n, dtype=torch.bool)), float("-inf"))
    o = torch.einsum("hts,shd->thd", torch.softmax(s, dim=-1), ve)
    (o * torch.tensor(d_o)).sum().backward()
    return o.detach().numpy(), qt.grad.numpy(), kt.grad.numpy(), vt.grad.numpy()


def test_restarted_positions_make_the_pack_equal_per_sample_training():
    """Forward and backward of shared-prompt attention over rope-rotated q, k (restarted
    positions) equal G separate causal runs over [prompt | resp_i] with positions 0..n_i-1."""
    rng = np.random.default_rng(5)
    Lp, lens, Hq, Hkv, d, base = 5, [3, 0, 4], 4, 2, 8, 50.0
    T = Lp + sum(lens)
    q, k, v = rng.standard_normal((T, Hq, d)), rng.standard_normal((T, Hkv, d)), rng.standard_normal((T, Hkv, d))
    d_o = rng.standard_normal((T, Hq, d))
    scale = d ** -0.5
    pos = rope.positions(Lp, lens)
    qr, kr = rope.rope_rotate(q, pos, base), rope.rope_rotate(k, pos, base)
    dqr, dkr, dv, o, _ = orc.sp_attn_bwd(qr, kr, v, d_o, Lp, lens, scale)
    dq, dk = rope.rope_rotate(dqr, pos, base, inverse=True), rope.rope_rotate(dkr, pos, base, inverse=True)

    off = Lp
    dk_p, dv_p = np.zeros((Lp, Hkv, d)), np.zeros((Lp, Hkv, d))
    for i, li in enumerate(lens):
        idx = np.concatenate([np.arange(Lp), np.arange(off, off + li)])
        g = d_o[idx].copy()
        if i > 0:
            g[:Lp] = 0.0                      # the prompt rows' upstream gradient is counted once
        oi, dqi, dki, dvi = per_sample_loss_and_grads(q[idx], k[idx], v[idx], g, scale, base)
        assert np.allclose(oi[Lp:], o[off:off + li], atol=1e-12)
        assert np.allclose(dqi[Lp:], dq[off:off + li], atol=1e-11)
        assert np.allclose(dki[Lp:], dk[off:off + li], atol=1e-11)
        assert np.allclose(dvi[Lp:], dv[off:off + li], atol=1e-11)
        if i == 0:
            assert np.allclose(oi[:Lp], o[:Lp], atol=1e-12)
            assert np.allclose(dqi[:Lp], dq[:Lp], atol=1e-11)
        dk_p += dki[:Lp]
        dv_p += dvi[:Lp]
        off += li
    assert np.allclose(dk_p, dk[:Lp], atol=1e-11)
    assert np.allclose(dv_p, dv[:Lp], atol=1e-11)


def test_contiguous_positions_would_break_the_equivalence():
    """A planted mistake: positions that do NOT restart change a later response's output."""
    rng = np.random.default_rng(6)
    Lp, lens, H, d, base = 4, [3, 3], 1, 8, 50.0
    T = Lp + sum(lens)
    q, k, v = rng.standard_normal((T, H, d)), rng.standard_normal((T, H, d)), rng.standard_normal((T, H, d))
    good = rope.positions(Lp, lens)
    bad = np.arange(T)
    o_good, _ = orc.sp_attn_fwd(rope.rope_rotate(q, good, base), rope.rope_rotate(k, good, base), v, Lp, lens, 0.3)
    o_bad, _ = orc.sp_attn_fwd(rope.rope_rotate(q, bad, base), rope.rope_rotate(k, bad, base), v, Lp, lens, 0.3)
    assert np.allclose(o_good[:Lp + 3], o_bad[:Lp + 3], atol=1e-12)       # prompt and response 1 agree
    assert np.abs(o_good[Lp + 3:] - o_bad[Lp + 3:]).max() > 1e-3          # response 2 does not
