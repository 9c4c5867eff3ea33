"""The forward-to-backward reserve: a forward whose workspace has room leaves the rounding residual of
o there, and a backward given the same, untouched workspace forms D from o plus that residual.  The
tag at the head of the workspace must make every other situation fall back to the bf16 o alone."""
import pytest
import torch

from paper_2511_18871_amd import binding as B
from paper_2511_18871_amd import workloads as W
from parity import gate, oracle_bwd, to64

pytestmark = pytest.mark.gpu


def _setup(seed=81, groups=None, heads=(8, 2)):
    groups = groups or [W.Group(300, [130, 0, 64, 77]), W.Group(65, [40])]
    w = W.Workload("reserve", groups, heads[0], heads[1], 128, torch.bfloat16, seed)
    t = W.make_tensors(w)
    t.k.mul_(4.0)                                  # peaked rows: the residual matters
    dev = [x.cuda() for x in (t.q, t.k, t.v, t.d_o)]
    return w, t, dev, (w.prompt_lens(), w.Gs(), w.resp_lens_flat(), w.softmax_scale)


def _sizes(w):
    pl, rl = w.prompt_lens(), w.resp_lens_flat()
    args = (w.total_tokens, len(pl), len(rl), w.n_q_heads, w.n_kv_heads, w.head_dim, B.SP_BF16)
    return (B.workspace_bytes(False, *args), B.workspace_bytes(True, *args),
            B.reserve_bytes(w.total_tokens, w.n_q_heads, w.head_dim, B.SP_BF16))


def _ws(n):
    return torch.full((n,), 0xA5, dtype=torch.uint8, device="cuda")


def test_reserve_equals_explicit_residual_and_falls_back_when_it_cannot_be_trusted():
    w, t, (q, k, v, d_o), pk = _setup()
    fwd_need, bwd_need, res = _sizes(w)
    assert res == ((w.total_tokens * w.n_q_heads * 128 * 2 + 255) // 256) * 256
    assert B.reserve_bytes(w.total_tokens, w.n_q_heads, 128, B.SP_F32) == 0
    # references: explicit residual, and no residual at all (a workspace without room)
    o_lo = torch.empty_like(q)
    o, lse = B.sp_attn_fwd_batched_ex(q, k, v, *pk, 0, o_lo=o_lo, workspace=_ws(fwd_need))
    with_lo = B.sp_attn_bwd_batched_ex(q, k, v, o, lse, d_o, *pk, 0, o_lo=o_lo, workspace=_ws(bwd_need))
    without = B.sp_attn_bwd_batched(q, k, v, o, lse, d_o, *pk, workspace=_ws(bwd_need))
    torch.cuda.synchronize()
    assert not torch.equal(with_lo[0], without[0])
    same = lambda a, b: all(torch.equal(x, y) for x, y in zip(a, b))

    # 1. shared workspace with room: the backward uses the reserve = the explicit residual, bit for bit
    ws = _ws(bwd_need + res)
    o1, lse1 = B.sp_attn_fwd_batched(q, k, v, *pk, workspace=ws)
    got = B.sp_attn_bwd_batched(q, k, v, o1, lse1, d_o, *pk, workspace=ws)
    again = B.sp_attn_bwd_batched(q, k, v, o1, lse1, d_o, *pk, workspace=ws)      # the backward leaves the reserve valid
    torch.cuda.synchronize()
    assert torch.equal(o1, o) and torch.equal(lse1, lse)
    assert same(got, with_lo) and same(again, with_lo)
    # ... also when the stages are enqueued one call at a time
    dq, dk, dv = (torch.empty_like(x) for x in (q, k, v))
    for st, kw in ((B.SP_BWD_STAGE_ROWSUM, {}), (B.SP_BWD_STAGE_DQ, {"dq": dq}), (B.SP_BWD_STAGE_DKDV, {"dk": dk, "dv": dv})):
        B.sp_attn_bwd_batched_stages(q, k, v, o1, lse1, d_o, *pk, st, ws, **kw)
    torch.cuda.synchronize()
    assert same((dq, dk, dv), with_lo)

    # 2. another call used the workspace in between (here: a forward of another problem): no reserve
    w2, t2, (q2, k2, v2, _), pk2 = _setup(seed=82, groups=[W.Group(40, [9])], heads=(2, 2))
    o1, lse1 = B.sp_attn_fwd_batched(q, k, v, *pk, workspace=ws)
    B.sp_attn_fwd_batched(q2, k2, v2, *pk2, workspace=ws)
    got = B.sp_attn_bwd_batched(q, k, v, o1, lse1, d_o, *pk, workspace=ws)
    torch.cuda.synchronize()
    assert same(got, without)

    # 3. the reserve names its outputs: a backward for other o / lse buffers does not take it
    o1, lse1 = B.sp_attn_fwd_batched(q, k, v, *pk, workspace=ws)
    got = B.sp_attn_bwd_batched(q, k, v, o1.clone(), lse1, d_o, *pk, workspace=ws)
    torch.cuda.synchronize()
    assert same(got, without)

    # 4. a forward without room writes none, and a later backward with room finds none (stale bytes there)
    o1, lse1 = B.sp_attn_fwd_batched(q, k, v, *pk, workspace=ws[:bwd_need])
    got = B.sp_attn_bwd_batched(q, k, v, o1, lse1, d_o, *pk, workspace=ws)
    torch.cuda.synchronize()
    assert same(got, without)

    # 5. a reserve written for response rows only serves a response-rows backward, not a full one
    fl = B.SP_FLAG_RESPONSE_ROWS
    B.sp_attn_fwd_batched_ex(q, k, v, *pk, fl, o=o1, lse=lse1, workspace=ws)
    got = B.sp_attn_bwd_batched(q, k, v, o1, lse1, d_o, *pk, workspace=ws)
    torch.cuda.synchronize()
    assert same(got, without)
    B.sp_attn_fwd_batched_ex(q, k, v, *pk, fl, o=o1, lse=lse1, workspace=ws)
    got_r = B.sp_attn_bwd_batched_ex(q, k, v, o1, lse1, d_o, *pk, fl, workspace=ws)
    want_r = B.sp_attn_bwd_batched_ex(q, k, v, o, lse, d_o, *pk, fl, o_lo=o_lo, workspace=_ws(bwd_need))
    torch.cuda.synchronize()
    T = w.total_tokens
    resp = torch.ones(T, dtype=torch.bool)
    base = 0
    for g in w.groups:
        resp[base:base + g.prompt_len] = False
        base += g.total
    assert torch.equal(got_r[0][resp.cuda()], want_r[0][resp.cuda()]) and same(got_r[1:], want_r[1:])


def test_binding_hands_the_forward_workspace_to_the_backward():
    """Calls that pass no workspace: the binding allocates one with room for the reserve in the forward and
    the backward finds it on the forward's output; gated against the oracle."""
    w, t, (q, k, v, d_o), pk = _setup(seed=83)
    o, lse = B.sp_attn_fwd_batched(q, k, v, *pk)
    dq, dk, dv = B.sp_attn_bwd_batched(q, k, v, o, lse, d_o, *pk)
    o_lo = torch.empty_like(q)
    o2, lse2 = B.sp_attn_fwd_batched_ex(q, k, v, *pk, 0, o_lo=o_lo)
    want = B.sp_attn_bwd_batched_ex(q, k, v, o2, lse2, d_o, *pk, 0, o_lo=o_lo)
    torch.cuda.synchronize()
    assert all(torch.equal(a, b) for a, b in zip((dq, dk, dv), want))
    rdq, rdk, rdv, _, _ = oracle_bwd(w, t)
    for name, a, r in (("dQ", dq, rdq), ("dK", dk, rdk), ("dV", dv, rdv)):
        print(gate(name, to64(a), r, w.dtype))
