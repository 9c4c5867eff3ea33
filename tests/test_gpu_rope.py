"""GPU parity of the rotary-embedding pass with restarted position indices, and of the whole
chain rope -> shared-prompt attention -> inverse rope on the gradients, against the fp64 oracles."""
import numpy as np
import pytest
import torch

from oracle import rope_oracle as rope
from oracle import sp_attn_oracle as orc
from paper_2511_18871_amd import binding as B
from paper_2511_18871_amd import workloads as W
from parity import gate, gate_lse, to64

pytestmark = pytest.mark.gpu

GROUPS = [W.Group(333, [1, 63, 65, 0, 127, 129, 200]), W.Group(70, [300, 5]), W.Group(0, [40, 9]), W.Group(1, [])]


def bf16_ulp(ref):
    """Spacing of bf16 numbers at |ref| (8 significant bits)."""
    a = np.maximum(np.abs(ref), 2.0 ** -126)
    return 2.0 ** (np.floor(np.log2(a)) - 7)


@pytest.mark.parametrize("dtype,d", [(torch.bfloat16, 128), (torch.float32, 64), (torch.float32, 128), (torch.bfloat16, 64)])
@pytest.mark.parametrize("inverse", [False, True])
def test_rope_pass_matches_oracle(dtype, d, inverse):
    w = W.Workload("rope", GROUPS, 5, 5, d, dtype, 55)
    t = W.make_tensors(w)
    pos = rope.positions_batched(w.prompt_lens(), w.Gs(), w.resp_lens_flat())
    ref = rope.rope_rotate(to64(t.q), pos, 1e6, inverse=inverse)
    got = to64(B.sp_attn_rope(t.q.cuda(), w.prompt_lens(), w.Gs(), w.resp_lens_flat(), 1e6, inverse=inverse))
    err = np.abs(got - ref)
    if dtype == torch.float32:
        assert float(err.max()) <= 2e-6 * max(1.0, float(np.abs(ref).max()))
    else:
        # the exact result rounded to bf16 is at most half a spacing away; fp32 arithmetic before
        # the rounding (absolute error ~1e-7 |x|, which matters where the two products cancel) can
        # move a value across a rounding boundary, never further than one spacing
        excess = float(np.max(err - (1.0001 * bf16_ulp(ref) + 1e-6 * np.abs(to64(t.q)).max())))
        assert excess <= 0.0, excess
        exact = to64(torch.tensor(ref).to(torch.bfloat16))
        mismatch = float(np.mean(got != exact))
        assert mismatch < 0.01, mismatch


def test_rope_in_place_and_long_positions():
    """Positions beyond 16 000 (angles of tens of thousands of radians) and y == x."""
    w = W.Workload("rope_long", [W.Group(16500, [130, 70])], 2, 2, 128, torch.float32, 56)
    t = W.make_tensors(w)
    pos = rope.positions_batched(w.prompt_lens(), w.Gs(), w.resp_lens_flat())
    assert pos.max() == 16500 + 129 and pos[-1] == 16500 + 69
    ref = rope.rope_rotate(to64(t.q), pos, 10000.0)
    x = t.q.cuda()
    y = B.sp_attn_rope(x, w.prompt_lens(), w.Gs(), w.resp_lens_flat(), 10000.0, out=x)
    assert y.data_ptr() == x.data_ptr()
    assert float(np.abs(to64(x) - ref).max()) <= 2e-6 * float(np.abs(ref).max())


@pytest.mark.parametrize("dtype,d", [(torch.bfloat16, 128), (torch.float32, 64)])
def test_rope_attention_chain_matches_oracle(dtype, d):
    w = W.Workload("rope_chain", GROUPS[:3], 6, 2, d, dtype, 57)
    t = W.make_tensors(w)
    pl, Gs, rl, base = w.prompt_lens(), w.Gs(), w.resp_lens_flat(), 1e4
    pos = rope.positions_batched(pl, Gs, rl)
    # oracle chain: rotate in fp64, hand the attention oracle what a dtype model would hold
    cast = (lambda a: to64(torch.tensor(a).to(dtype)))
    qr, kr = cast(rope.rope_rotate(to64(t.q), pos, base)), cast(rope.rope_rotate(to64(t.k), pos, base))
    rdqr, rdkr, rdv, ro, rlse = orc.sp_attn_bwd_batched(qr, kr, to64(t.v), to64(t.d_o), pl, Gs, rl, w.softmax_scale)
    rdq, rdk = rope.rope_rotate(rdqr, pos, base, inverse=True), rope.rope_rotate(rdkr, pos, base, inverse=True)
    # GPU chain
    q, k, v, d_o = t.q.cuda(), t.k.cuda(), t.v.cuda(), t.d_o.cuda()
    gq, gk = B.sp_attn_rope(q, pl, Gs, rl, base), B.sp_attn_rope(k, pl, Gs, rl, base)
    o, lse = B.sp_attn_fwd_batched(gq, gk, v, pl, Gs, rl, w.softmax_scale)
    dq, dk, dv = B.sp_attn_bwd_batched(gq, gk, v, o, lse, d_o, pl, Gs, rl, w.softmax_scale)
    dq, dk = B.sp_attn_rope(dq, pl, Gs, rl, base, inverse=True), B.sp_attn_rope(dk, pl, Gs, rl, base, inverse=True)
    torch.cuda.synchronize()
    gate("O", to64(o), ro, dtype)
    gate_lse(to64(lse), rlse, dtype)
    gate("dQ", to64(dq), rdq, dtype)
    gate("dK", to64(dk), rdk, dtype)
    gate("dV", to64(dv), rdv, dtype)


@pytest.mark.parametrize("dtype,d", [(torch.bfloat16, 128), (torch.float32, 64)])
def test_rope_of_q_and_k_in_one_launch_equals_two_passes(dtype, d):
    w = W.Workload("rope_qk", GROUPS, 6, 2, d, dtype, 57)
    t = W.make_tensors(w)
    q, k = t.q.cuda(), t.k.cuda()
    pk = (w.prompt_lens(), w.Gs(), w.resp_lens_flat(), 1e6)
    for inverse in (False, True):
        q1, k1 = B.sp_attn_rope(q, *pk, inverse=inverse), B.sp_attn_rope(k, *pk, inverse=inverse)
        q2, k2 = B.sp_attn_rope_qk(q, k, *pk, inverse=inverse)
        torch.cuda.synchronize()
        assert torch.equal(q1, q2) and torch.equal(k1, k2)
    # in place, and back: the inverse rotation returns the input to rounding
    qq, kk = q.clone(), k.clone()
    B.sp_attn_rope_qk(qq, kk, *pk, q_out=qq, k_out=kk)
    B.sp_attn_rope_qk(qq, kk, *pk, inverse=True, q_out=qq, k_out=kk)
    torch.cuda.synchronize()
    tol = 3e-2 if dtype == torch.bfloat16 else 1e-5
    assert float((qq.float() - q.float()).abs().max()) <= tol * float(q.float().abs().max())
    assert float((kk.float() - k.float()).abs().max()) <= tol * float(k.float().abs().max())
