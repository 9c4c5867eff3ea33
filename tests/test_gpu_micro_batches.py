"""GPU parity of the response-rows / accumulate flags (micro-batches that share a prompt).

The oracle side is the definition itself: restricting the backward to response rows is the
full backward for an upstream gradient that is zero on the prompt rows, and accumulation is
addition to what the buffers held."""
import numpy as np
import pytest
import torch

from oracle import sp_attn_oracle as orc
from paper_2511_18871_amd import binding as B
from paper_2511_18871_amd import workloads as W
from parity import gate, gate_lse, to64

pytestmark = pytest.mark.gpu

CASES = {
    "ragged_multi": [W.Group(333, [1, 63, 65, 0, 127, 129, 200]), W.Group(70, [300, 5])],
    "prompt_ends_mid_tile": [W.Group(300, [200, 90])],
    "no_prompt": [W.Group(0, [65, 130, 7])],
    "no_responses": [W.Group(257, [])],
    "long_prompt": [W.Group(1100, [40, 70, 3])],
}


def prompt_row_mask(w):
    m = np.zeros(w.total_tokens, dtype=bool)
    base = 0
    for g in w.groups:
        m[base:base + g.prompt_len] = True
        base += g.total
    return m


@pytest.mark.parametrize("name", list(CASES))
@pytest.mark.parametrize("dtype,d", [(torch.bfloat16, 128), (torch.float32, 64)])
def test_response_rows_and_accumulate(name, dtype, d):
    w = W.Workload(name, CASES[name], 4, 2, d, dtype, 93)
    t = W.make_tensors(w)
    pl, Gs, rl, sc = w.prompt_lens(), w.Gs(), w.resp_lens_flat(), w.softmax_scale
    pm = prompt_row_mask(w)
    q, k, v, d_o = t.q.cuda(), t.k.cuda(), t.v.cuda(), t.d_o.cuda()

    # forward: response rows written, prompt rows of the outputs untouched
    sentinel_o = torch.full_like(q, 7.0)
    sentinel_l = torch.full((w.n_q_heads, w.total_tokens), -3.0, device="cuda")
    o, lse = B.sp_attn_fwd_batched_ex(q, k, v, pl, Gs, rl, sc, B.SP_FLAG_RESPONSE_ROWS, o=sentinel_o.clone(),
                                      lse=sentinel_l.clone())
    torch.cuda.synchronize()
    ro, rlse = orc.sp_attn_fwd_batched(to64(t.q), to64(t.k), to64(t.v), pl, Gs, rl, sc)
    assert torch.all(o[torch.tensor(pm)] == 7.0) and torch.all(lse[:, torch.tensor(pm)] == -3.0)
    if (~pm).any():
        gate("O[resp]", to64(o)[~pm], ro[~pm], dtype)
        gate_lse(to64(lse)[:, ~pm], rlse[:, ~pm], dtype)

    # backward: full forward outputs, then response rows only, accumulated onto a starting value
    o_full, lse_full = B.sp_attn_fwd_batched(q, k, v, pl, Gs, rl, sc)
    g0 = d_o.clone()
    g0[torch.tensor(pm)] = 0
    rdq, rdk, rdv, _, _ = orc.sp_attn_bwd_batched(to64(t.q), to64(t.k), to64(t.v), to64(g0), pl, Gs, rl, sc)
    gen = torch.Generator().manual_seed(5)
    dk0 = torch.randn(t.k.shape, generator=gen).to(dtype)
    dv0 = torch.randn(t.v.shape, generator=gen).to(dtype)
    dq = torch.full_like(q, 9.0)
    dk, dv = dk0.cuda(), dv0.cuda()
    # d_o keeps its non-zero prompt rows: the flag, not the data, must exclude them
    B.sp_attn_bwd_batched_ex(q, k, v, o_full, lse_full, d_o, pl, Gs, rl, sc,
                             B.SP_FLAG_RESPONSE_ROWS | B.SP_FLAG_ACCUMULATE_DKDV, dq=dq, dk=dk, dv=dv)
    torch.cuda.synchronize()
    assert torch.all(dq[torch.tensor(pm)] == 9.0)
    if (~pm).any():
        gate("dQ[resp]", to64(dq)[~pm], rdq[~pm], dtype)
    gate("dK", to64(dk), rdk + to64(dk0), dtype)
    gate("dV", to64(dv), rdv + to64(dv0), dtype)

    # without ACCUMULATE the same call overwrites
    dk2, dv2 = torch.full_like(k, 5.0), torch.full_like(v, 5.0)
    B.sp_attn_bwd_batched_ex(q, k, v, o_full, lse_full, d_o, pl, Gs, rl, sc, B.SP_FLAG_RESPONSE_ROWS, dk=dk2, dv=dv2)
    torch.cuda.synchronize()
    gate("dK[overwrite]", to64(dk2), rdk, dtype)
    gate("dV[overwrite]", to64(dv2), rdv, dtype)


def test_two_micro_batches_reproduce_the_full_batch_bf16():
    """The use the flags exist for: G = 6 responses in two micro-batches of three; response rows of
    each pack, the prompt once with G = 0, prompt dk/dv accumulated in place."""
    Lp, lens, Hq, Hkv, d = 700, [130, 64, 200, 31, 90, 150], 4, 2, 128
    w = W.Workload("full", [W.Group(Lp, lens)], Hq, Hkv, d, torch.bfloat16, 97)
    t = W.make_tensors(w)
    sc = w.softmax_scale
    rdq, rdk, rdv, ro, rlse = orc.sp_attn_bwd(to64(t.q), to64(t.k), to64(t.v), to64(t.d_o), Lp, lens, sc)
    starts = np.concatenate([[Lp], Lp + np.cumsum(lens)])
    dkp = torch.zeros(Lp, Hkv, d, dtype=torch.bfloat16, device="cuda")
    dvp = torch.zeros_like(dkp)
    # the prompt rows once (plain causal attention over the prompt)
    qp, kp, vp, gp = (x[:Lp].cuda().contiguous() for x in (t.q, t.k, t.v, t.d_o))
    op, lp_ = B.sp_attn_fwd_batched(qp, kp, vp, [Lp], [0], [], sc)
    dqp, dkp, dvp = B.sp_attn_bwd_batched(qp, kp, vp, op, lp_, gp, [Lp], [0], [], sc)
    gate("dQ[prompt]", to64(dqp), rdq[:Lp], torch.bfloat16)
    for members in ([0, 2, 4], [1, 3, 5]):
        idx = np.concatenate([np.arange(Lp)] + [np.arange(starts[i], starts[i + 1]) for i in members])
        ti = torch.tensor(idx)
        q, k, v, g = (x[ti].cuda().contiguous() for x in (t.q, t.k, t.v, t.d_o))
        ml = [lens[i] for i in members]
        o, lse = B.sp_attn_fwd_batched_ex(q, k, v, [Lp], [3], ml, sc, B.SP_FLAG_RESPONSE_ROWS)
        dk = torch.zeros_like(k)
        dv = torch.zeros_like(v)
        dk[:Lp], dv[:Lp] = dkp, dvp                         # running sums of the prompt's dk/dv
        dq, dk, dv = B.sp_attn_bwd_batched_ex(q, k, v, o, lse, g, [Lp], [3], ml, sc,
                                              B.SP_FLAG_RESPONSE_ROWS | B.SP_FLAG_ACCUMULATE_DKDV, dk=dk, dv=dv)
        torch.cuda.synchronize()
        dkp, dvp = dk[:Lp].clone(), dv[:Lp].clone()
        gate("O[resp]", to64(o)[Lp:], ro[idx[Lp:]], torch.bfloat16)
        gate("dQ[resp]", to64(dq)[Lp:], rdq[idx[Lp:]], torch.bfloat16)
        gate("dK[resp]", to64(dk)[Lp:], rdk[idx[Lp:]], torch.bfloat16)
        gate("dV[resp]", to64(dv)[Lp:], rdv[idx[Lp:]], torch.bfloat16)
    # the running sums were rounded to bf16 three times (prompt pass, two micro-batches) instead of
    # once: two more half-spacings of the largest value on top of the single-pass max-abs gate;
    # the relative RMS gate is unchanged
    for name, got, ref in (("dK", dkp, rdk[:Lp]), ("dV", dvp, rdv[:Lp])):
        got = to64(got)
        ninf = float(np.abs(ref).max())
        err = np.abs(got - ref)
        rms = float(np.sqrt(np.mean(err ** 2)) / np.sqrt(np.mean(ref ** 2)))
        tol = 2e-2 * max(1.0, ninf / 4.0) + 2 * 2.0 ** -9 * ninf
        assert float(err.max()) <= tol and rms <= 5e-3, (name, float(err.max()), tol, rms)
