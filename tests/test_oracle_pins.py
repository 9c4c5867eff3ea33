"""Pins for the CPU oracle: every check here compares oracle/ against something
that is not the oracle — an independently coded per-sample causal attention
(the equivalence stated at the end of Section 4.3), torch autograd, central
finite differences, closed forms and counting arguments."""
import os

import numpy as np
import pytest
import scipy.special
import torch

from oracle import sp_attn_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------------------
# independent reference: ordinary causal attention of ONE sample, row by row,
# no mask matrix anywhere (the row simply stops at the diagonal).
# ----------------------------------------------------------------------------
def causal_rowwise(q, k, v, scale):
    n, Hq, d = q.shape
    rep = Hq // k.shape[1]
    O = np.zeros((n, Hq, d))
    LSE = np.zeros((Hq, n))
    for h in range(Hq):
        g = h // rep
        for t in range(n):
            s = scale * (k[: t + 1, g, :] @ q[t, h, :])
            LSE[h, t] = scipy.special.logsumexp(s)
            O[t, h, :] = scipy.special.softmax(s) @ v[: t + 1, g, :]
    return O, LSE


def causal_autograd(q, k, v, d_o, scale):
    """Gradients of sum(O * dO) for ordinary causal attention via torch autograd."""
    qt, kt, vt = (torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in (q, k, v))
    n, Hq, d = q.shape
    rep = Hq // k.shape[1]
    ke, ve = kt.repeat_interleave(rep, dim=1), vt.repeat_interleave(rep, dim=1)
    s = torch.einsum("thd,shd->hts", qt, ke) * scale
    s = s.masked_fill(torch.triu(torch.ones(n, n, dtype=torch.bool), diagonal=1), float("-inf"))
    o = torch.einsum("hts,shd->thd", torch.softmax(s, dim=-1), ve)
    (o * torch.tensor(d_o)).sum().backward()
    return qt.grad.numpy(), kt.grad.numpy(), vt.grad.numpy()


def draw(seed, T, Hq, Hkv, d):
    r = np.random.default_rng(seed)
    return (r.standard_normal((T, Hq, d)), r.standard_normal((T, Hkv, d)),
            r.standard_normal((T, Hkv, d)), r.standard_normal((T, Hq, d)))


def offsets(lp, lens):
    off = [lp]
    for li in lens:
        off.append(off[-1] + li)
    return off


CASES = [
    (5, [3, 4], 2, 1, 4),
    (7, [1, 0, 6, 2], 4, 2, 8),
    (0, [4, 3], 2, 2, 4),
    (6, [], 3, 1, 4),
    (1, [1], 1, 1, 2),
    (9, [5, 5, 5], 6, 2, 16),
]


@pytest.mark.parametrize("lp,lens,Hq,Hkv,d", CASES)
def test_forward_equals_independent_causal_runs(lp, lens, Hq, Hkv, d):
    """Each response's rows, and the prompt's rows, equal an ordinary causal
    attention over [prompt | resp_i] (Section 4.3, closing paragraph)."""
    T = lp + sum(lens)
    q, k, v, _ = draw(11, T, Hq, Hkv, d)
    scale = 0.37
    O, LSE = orc.sp_attn_fwd(q, k, v, lp, lens, scale)
    off = offsets(lp, lens)
    runs = list(range(len(lens))) if lens else [None]
    for i in runs:
        idx = list(range(lp)) + ([] if i is None else list(range(off[i], off[i + 1])))
        if not idx:
            continue
        Oi, Li = causal_rowwise(q[idx], k[idx], v[idx], scale)
        np.testing.assert_allclose(O[idx], Oi, rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(LSE[:, idx], Li, rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("lp,lens,Hq,Hkv,d", CASES)
def test_backward_equals_sum_of_independent_runs(lp, lens, Hq, Hkv, d):
    """grad(L_shared) = sum_k grad(L_k): response rows' gradients come from their own
    run; the prompt's dK/dV are the sum over the runs, with the prompt's own dO
    fed to exactly one run."""
    T = lp + sum(lens)
    q, k, v, d_o = draw(12, T, Hq, Hkv, d)
    scale = 0.41
    dQ, dK, dV, _, _ = orc.sp_attn_bwd(q, k, v, d_o, lp, lens, scale)
    off = offsets(lp, lens)
    dQp = np.zeros((lp, Hq, d)); dKp = np.zeros((lp, Hkv, d)); dVp = np.zeros((lp, Hkv, d))
    runs = list(range(len(lens))) if lens else [None]
    for n_run, i in enumerate(runs):
        ridx = [] if i is None else list(range(off[i], off[i + 1]))
        idx = list(range(lp)) + ridx
        if not idx:
            continue
        g_out = d_o[idx].copy()
        if n_run != 0:
            g_out[:lp] = 0.0          # the prompt's upstream gradient is counted once
        gq, gk, gv = causal_autograd(q[idx], k[idx], v[idx], g_out, scale)
        dQp += gq[:lp]; dKp += gk[:lp]; dVp += gv[:lp]
        np.testing.assert_allclose(dQ[ridx], gq[lp:], rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose(dK[ridx], gk[lp:], rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose(dV[ridx], gv[lp:], rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dQ[:lp], dQp, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dK[:lp], dKp, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dV[:lp], dVp, rtol=1e-10, atol=1e-12)


def test_backward_finite_differences():
    """Central differences of l = sum(O * dO) on every input element."""
    lp, lens, Hq, Hkv, d = 3, [2, 3], 2, 1, 4
    T = lp + sum(lens)
    q, k, v, d_o = draw(13, T, Hq, Hkv, d)
    scale = 0.5
    dQ, dK, dV, _, _ = orc.sp_attn_bwd(q, k, v, d_o, lp, lens, scale)
    loss = lambda q_, k_, v_: float(np.sum(orc.sp_attn_fwd(q_, k_, v_, lp, lens, scale)[0] * d_o))
    h = 1e-6
    for which, (x, g) in enumerate(((q, dQ), (k, dK), (v, dV))):
        num = np.zeros_like(x)
        for ix in np.ndindex(x.shape):
            xp, xm = x.copy(), x.copy()
            xp[ix] += h; xm[ix] -= h
            a = [q, k, v]; b = [q, k, v]
            a[which], b[which] = xp, xm
            num[ix] = (loss(*a) - loss(*b)) / (2 * h)
        assert np.max(np.abs(num - g)) <= 1e-7 * max(1.0, np.max(np.abs(g)))


def test_uniform_attention_closed_form():
    """With Q = 0 every allowed key gets the same weight: LSE = log n(t) and O is the
    mean of the allowed V rows, n(t) = t+1 on the prompt and Lp + j + 1 on the j-th
    token of any response."""
    lp, lens, Hq, Hkv, d = 6, [4, 0, 3, 5], 2, 2, 4
    T = lp + sum(lens)
    _, k, v, _ = draw(14, T, Hq, Hkv, d)
    O, LSE = orc.sp_attn_fwd(np.zeros((T, Hq, d)), k, v, lp, lens, 1.0)
    off = offsets(lp, lens)
    for t in range(lp):
        np.testing.assert_allclose(LSE[:, t], np.log(t + 1), rtol=1e-14)
        np.testing.assert_allclose(O[t], v[: t + 1].mean(axis=0), rtol=1e-13, atol=1e-14)
    for i, li in enumerate(lens):
        for j in range(li):
            t = off[i] + j
            keys = list(range(lp)) + list(range(off[i], t + 1))
            np.testing.assert_allclose(LSE[:, t], np.log(lp + j + 1), rtol=1e-14)
            np.testing.assert_allclose(O[t], v[keys].mean(axis=0), rtol=1e-13, atol=1e-14)


def test_pair_counts_match_complexity_terms():
    with open(os.path.join(GOLDEN, "pair_counts.txt")) as f:
        rows = [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]
    for lp, G, L, A, B, C in (map(int, r) for r in rows):
        M = orc.build_mask(lp, [L] * G)
        assert M[:lp, :lp].sum() == A
        assert M[lp:, :lp].sum() == B
        assert M[lp:, lp:].sum() == C
        assert not M[:lp, lp:].any()          # the prompt never sees a response


def test_pair_count_ragged_formula():
    lp, lens = 13, [5, 0, 9, 1, 4]
    M = orc.build_mask(lp, lens)
    assert M.sum() == lp * (lp + 1) // 2 + sum(l * lp + l * (l + 1) // 2 for l in lens)
    assert np.array_equal(np.diag(M), np.ones(lp + sum(lens), dtype=bool))


def dense_reference(q, k, v, allow, scale):
    """Ten-line dense softmax(QK^T + mask)V for the textbook reductions."""
    rep = q.shape[1] // k.shape[1]
    O = np.zeros_like(q)
    for h in range(q.shape[1]):
        s = scale * q[:, h] @ k[:, h // rep].T
        s[~allow] = -np.inf
        O[:, h] = scipy.special.softmax(s, axis=1) @ v[:, h // rep]
    return O


def test_textbook_reductions():
    Hq, Hkv, d, scale = 4, 2, 8, 0.3
    # G = 1: plain causal attention on all T tokens
    q, k, v, _ = draw(15, 12, Hq, Hkv, d)
    tril = np.tril(np.ones((12, 12), dtype=bool))
    np.testing.assert_allclose(orc.sp_attn_fwd(q, k, v, 5, [7], scale)[0],
                               dense_reference(q, k, v, tril, scale), rtol=1e-12, atol=1e-13)
    # no responses at all: causal on the prompt
    np.testing.assert_allclose(orc.sp_attn_fwd(q, k, v, 12, [], scale)[0],
                               dense_reference(q, k, v, tril, scale), rtol=1e-12, atol=1e-13)
    # no prompt: block-diagonal causal
    blk = np.zeros((12, 12), dtype=bool)
    for a, b in ((0, 4), (4, 9), (9, 12)):
        blk[a:b, a:b] = np.tril(np.ones((b - a, b - a), dtype=bool))
    np.testing.assert_allclose(orc.sp_attn_fwd(q, k, v, 0, [4, 5, 3], scale)[0],
                               dense_reference(q, k, v, blk, scale), rtol=1e-12, atol=1e-13)
    # Hq == Hkv (multi-head attention)
    q2, k2, v2, _ = draw(16, 12, 3, 3, d)
    np.testing.assert_allclose(orc.sp_attn_fwd(q2, k2, v2, 5, [7], scale)[0],
                               dense_reference(q2, k2, v2, tril, scale), rtol=1e-12, atol=1e-13)


def test_gqa_head_mapping_is_contiguous_blocks():
    """q heads 0..r-1 read kv head 0: zeroing kv head 1's V leaves them unchanged and
    zeroes the outputs of heads r..2r-1."""
    q, k, v, _ = draw(17, 10, 6, 2, 4)
    O = orc.sp_attn_fwd(q, k, v, 4, [3, 3], 1.0)[0]
    v2 = v.copy(); v2[:, 1] = 0.0
    O2 = orc.sp_attn_fwd(q, k, v2, 4, [3, 3], 1.0)[0]
    np.testing.assert_array_equal(O2[:, :3], O[:, :3])
    assert np.all(O2[:, 3:] == 0.0)


def test_softmax_identities():
    lp, lens = 5, [4, 3]
    q, k, v, d_o = draw(18, 12, 2, 1, 4)
    scale = 0.7
    O, LSE = orc.sp_attn_fwd(q, k, v, lp, lens, scale)
    np.testing.assert_allclose(O[0], np.repeat(v[0], 2, axis=0), rtol=1e-14)
    np.testing.assert_allclose(LSE[:, 0], scale * q[0] @ k[0, 0], rtol=1e-13)
    M = orc.build_mask(lp, lens)
    for t in range(12):
        allowed = v[M[t], 0]
        assert np.all(O[t] <= allowed.max(axis=0) + 1e-12)
        assert np.all(O[t] >= allowed.min(axis=0) - 1e-12)
    # dV sums: sum_s dV[s] = sum_t dO[t] because rows of P sum to one
    _, _, dV, _, _ = orc.sp_attn_bwd(q, k, v, d_o, lp, lens, scale)
    np.testing.assert_allclose(dV[:, 0].sum(axis=0), d_o.sum(axis=(0, 1)), rtol=1e-12)
    # shifting every key by a constant vector c changes S row-wise by a constant: dQ unchanged
    # and sum_s dK[s] = 0 because rows of dS sum to zero
    _, dK, _, _, _ = orc.sp_attn_bwd(q, k, v, d_o, lp, lens, scale)
    np.testing.assert_allclose(dK[:, 0].sum(axis=0), 0.0, atol=1e-12)


def test_permuting_responses_leaves_prompt_results_unchanged():
    lp, lens = 6, [3, 5, 2]
    q, k, v, d_o = draw(19, lp + sum(lens), 4, 2, 8)
    off = offsets(lp, lens)
    perm = [2, 0, 1]
    idx = list(range(lp))
    for i in perm:
        idx += list(range(off[i], off[i + 1]))
    a = orc.sp_attn_bwd(q, k, v, d_o, lp, lens, 0.3)
    b = orc.sp_attn_bwd(q[idx], k[idx], v[idx], d_o[idx], lp, [lens[i] for i in perm], 0.3)
    for xa, xb in zip(a[:4], b[:4]):
        np.testing.assert_allclose(xa[idx], xb, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(a[4][:, idx], b[4], rtol=1e-12, atol=1e-13)


def test_no_cross_response_leakage():
    lp, lens = 4, [3, 4, 2]
    q, k, v, d_o = draw(20, lp + sum(lens), 2, 1, 4)
    off = offsets(lp, lens)
    O, LSE = orc.sp_attn_fwd(q, k, v, lp, lens, 0.5)
    k2, v2 = k.copy(), v.copy()
    k2[off[1] + 1] += 3.0; v2[off[1] + 2] -= 2.0      # perturb response 2 only
    O2, LSE2 = orc.sp_attn_fwd(q, k2, v2, lp, lens, 0.5)
    others = list(range(lp)) + list(range(off[0], off[1])) + list(range(off[2], off[3]))
    np.testing.assert_array_equal(O[others], O2[others])
    np.testing.assert_array_equal(LSE[:, others], LSE2[:, others])
    assert not np.array_equal(O[off[1]:off[2]], O2[off[1]:off[2]])


def test_row_block_and_samples_agree_with_full():
    lp, lens = 10, [7, 0, 9]
    q, k, v, d_o = draw(21, lp + sum(lens), 4, 2, 8)
    full = orc.sp_attn_bwd(q, k, v, d_o, lp, lens, 0.35)
    blk = orc.sp_attn_bwd(q, k, v, d_o, lp, lens, 0.35, row_block=4)
    for a, b in zip(full, blk):
        np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-13)
    rows, heads = [0, 9, 10, 16, 25], [1, 3]
    Os, Ls = orc.sp_attn_fwd(q, k, v, lp, lens, 0.35, rows=rows, heads=heads)
    np.testing.assert_allclose(Os, full[3][rows][:, heads], rtol=1e-12)
    np.testing.assert_allclose(Ls, full[4][heads][:, rows], rtol=1e-12)
    dQs = orc.sp_attn_bwd_rows(q, k, v, d_o, lp, lens, 0.35, rows, heads)
    np.testing.assert_allclose(dQs, full[0][rows][:, heads], rtol=1e-11, atol=1e-13)
    part = orc.sp_attn_bwd(q, k, v, d_o, lp, lens, 0.35, kv_heads=[1])
    np.testing.assert_allclose(part[1][:, 1], full[1][:, 1], rtol=1e-12)
    np.testing.assert_allclose(part[2][:, 1], full[2][:, 1], rtol=1e-12)
    assert np.all(part[1][:, 0] == 0)


def test_batched_groups_are_independent():
    gs = [(4, [3, 2]), (0, [5]), (6, [])]
    T = sum(lp + sum(l) for lp, l in gs)
    q, k, v, d_o = draw(22, T, 2, 1, 4)
    out = orc.sp_attn_bwd_batched(q, k, v, d_o, [g[0] for g in gs], [len(g[1]) for g in gs],
                                  [x for g in gs for x in g[1]], 0.5)
    base = 0
    for lp, lens in gs:
        n = lp + sum(lens)
        sl = slice(base, base + n)
        one = orc.sp_attn_bwd(q[sl], k[sl], v[sl], d_o[sl], lp, lens, 0.5)
        for a, b in zip(out[:4], one[:4]):
            np.testing.assert_array_equal(a[sl], b)
        base += n


def test_micro_batches_sharing_a_prompt_accumulate_to_the_full_batch_gradient():
    """The attention-level form of the paper's gradient identity (Section 3, Eq. 1: the gradient
    of a group is the sum of its members' gradients): splitting the G responses of a prompt over
    micro-batches, running only the RESPONSE rows of each pack [prompt | its responses] (upstream
    gradient zero on the prompt rows) and the prompt rows once on their own, the dK/dV of the
    prompt accumulate to the full-batch values and every response-row quantity is unchanged."""
    rng = np.random.default_rng(11)
    Lp, lens, Hq, Hkv, d = 6, [3, 2, 4, 1], 4, 2, 8
    T = Lp + sum(lens)
    q, k, v = rng.standard_normal((T, Hq, d)), rng.standard_normal((T, Hkv, d)), rng.standard_normal((T, Hkv, d))
    d_o = rng.standard_normal((T, Hq, d))
    scale = 0.4
    dq, dk, dv, o, lse = orc.sp_attn_bwd(q, k, v, d_o, Lp, lens, scale)

    starts = np.concatenate([[Lp], Lp + np.cumsum(lens)])
    dk_p, dv_p = np.zeros((Lp, Hkv, d)), np.zeros((Lp, Hkv, d))
    for members in ([0, 2], [1, 3]):                       # two micro-batches of two responses
        idx = np.concatenate([np.arange(Lp)] + [np.arange(starts[i], starts[i + 1]) for i in members])
        g = d_o[idx].copy()
        g[:Lp] = 0.0                                       # response rows only
        mdq, mdk, mdv, mo, mlse = orc.sp_attn_bwd(q[idx], k[idx], v[idx], g, Lp, [lens[i] for i in members], scale)
        assert np.allclose(mo[Lp:], o[idx[Lp:]], atol=1e-13) and np.allclose(mlse[:, Lp:], lse[:, idx[Lp:]], atol=1e-13)
        assert np.allclose(mdq[Lp:], dq[idx[Lp:]], atol=1e-12)
        assert np.allclose(mdk[Lp:], dk[idx[Lp:]], atol=1e-12) and np.allclose(mdv[Lp:], dv[idx[Lp:]], atol=1e-12)
        assert np.allclose(mdq[:Lp], 0.0)                  # zero upstream gradient: nothing flows to prompt queries
        dk_p += mdk[:Lp]
        dv_p += mdv[:Lp]
    # the prompt rows, once: plain causal attention over the prompt with the prompt's upstream gradient
    pdq, pdk, pdv, _, _ = orc.sp_attn_bwd(q[:Lp], k[:Lp], v[:Lp], d_o[:Lp], Lp, [], scale)
    assert np.allclose(pdq, dq[:Lp], atol=1e-12)
    assert np.allclose(dk_p + pdk, dk[:Lp], atol=1e-12)
    assert np.allclose(dv_p + pdv, dv[:Lp], atol=1e-12)


def test_pair_count_against_the_cost_ratio_of_eq5():
    """Eq. 5 of Section 4.3 prices the shared mask at (Lp^2 + K Lr (Lp + Lr)) / (K (Lp + Lr)^2) of K
    per-sample runs, counting squares where a causal mask has triangles.  With triangles on both
    sides the rectangle term K Lr Lp weighs twice as much, so the exact ratio of the oracle's mask
    to K causal masks over Lp + Lr tokens is the printed ratio + Lr Lp / (Lp + Lr)^2, up to the
    diagonals (O(1 / (Lp + Lr))); and it tends to 1 / K for Lp >> Lr as the section states."""
    rows = [ln.split() for ln in open(os.path.join(GOLDEN, "cost_ratio_eq5.txt")) if ln.strip() and ln[0] != "#"]
    assert len(rows) == 3
    for lp, lr, k, num, den, rho in rows:
        lp, lr, k, num, den, rho = int(lp), int(lr), int(k), int(num), int(den), float(rho)
        assert abs(num / den - rho) < 1e-6                       # the fixture is self-consistent
        n = lp + lr
        shared = int(orc.build_mask(lp, [lr] * k).sum())
        per_sample = k * int(np.tril(np.ones((n, n), dtype=bool)).sum())
        exact = shared / per_sample
        assert abs(exact - (rho + lr * lp / n ** 2)) < 2.0 / n, (lp, lr, k, exact, rho)
    lp, lr, k = 2000, 2, 4
    assert abs(int(orc.build_mask(lp, [lr] * k).sum()) / (k * (lp + lr) * (lp + lr + 1) // 2) - 1.0 / k) < 2e-3
