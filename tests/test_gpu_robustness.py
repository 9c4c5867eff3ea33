"""GPU checks that hold at any size: no write outside the outputs, bitwise repeatability,
stream ordering, the multi-launch segment-table upload, the staged backward."""
import numpy as np
import pytest
import torch

from paper_2511_18871_amd import binding as B
from paper_2511_18871_amd import workloads as W
from parity import gate, oracle_bwd, to64

pytestmark = pytest.mark.gpu

PAD = 4096      # elements of canary on both sides of every output


def padded(shape, dtype, fill):
    n = int(np.prod(shape))
    buf = torch.full((n + 2 * PAD,), fill, dtype=dtype, device="cuda")
    return buf, buf[PAD:PAD + n].view(*shape)


def canary_ok(buf, fill):
    return bool((buf[:PAD] == fill).all()) and bool((buf[-PAD:] == fill).all())


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_no_out_of_bounds_writes_and_outputs_fully_written(dtype):
    d = 128 if dtype == torch.bfloat16 else 64
    w = W.Workload("canary", [W.Group(333, [1, 63, 65, 0, 127, 129, 200]), W.Group(70, [300, 5])], 6, 2, d, dtype, 91)
    t = W.make_tensors(w)
    q, k, v, d_o = (x.cuda() for x in (t.q, t.k, t.v, t.d_o))
    T, Hq, Hkv = w.total_tokens, w.n_q_heads, w.n_kv_heads
    fill = 7.0
    ob, o = padded((T, Hq, d), dtype, fill)
    lb, lse = padded((Hq, T), torch.float32, fill)
    qb, dq = padded((T, Hq, d), dtype, fill)
    kb, dk = padded((T, Hkv, d), dtype, fill)
    vb, dv = padded((T, Hkv, d), dtype, fill)
    pl, Gs, rl = w.prompt_lens(), w.Gs(), w.resp_lens_flat()
    B.sp_attn_fwd_batched(q, k, v, pl, Gs, rl, w.softmax_scale, o=o, lse=lse)
    B.sp_attn_bwd_batched(q, k, v, o, lse, d_o, pl, Gs, rl, w.softmax_scale, dq=dq, dk=dk, dv=dv)
    torch.cuda.synchronize()
    for buf in (ob, lb, qb, kb, vb):
        assert canary_ok(buf, fill)
    rdq, rdk, rdv, ro, rlse = oracle_bwd(w, t)
    for name, got, ref in (("O", o, ro), ("dQ", dq, rdq), ("dK", dk, rdk), ("dV", dv, rdv)):
        gate(name, to64(got), ref, dtype)        # also proves no element kept the fill value


def test_bitwise_repeatable_forward_and_backward():
    w = W.Workload("repeat", [W.Group(700, [90, 300, 17])], 8, 2, 128, torch.bfloat16, 92)
    t = W.make_tensors(w)
    q, k, v, d_o = (x.cuda() for x in (t.q, t.k, t.v, t.d_o))
    runs = []
    for _ in range(3):
        o, lse = B.sp_attn_fwd(q, k, v, 700, [90, 300, 17], w.softmax_scale)
        dq, dk, dv = B.sp_attn_bwd(q, k, v, o, lse, d_o, 700, [90, 300, 17], w.softmax_scale)
        torch.cuda.synchronize()
        runs.append((o, lse, dq, dk, dv))
    for r in runs[1:]:
        for a, b in zip(runs[0], r):
            assert torch.equal(a, b)


def test_runs_in_order_on_a_side_stream():
    w = W.Workload("stream", [W.Group(500, [200, 100])], 4, 4, 128, torch.bfloat16, 93)
    t = W.make_tensors(w)
    q, k, v = (x.cuda() for x in (t.q, t.k, t.v))
    ref_o, ref_lse = B.sp_attn_fwd(q, k, v, 500, [200, 100], w.softmax_scale)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    big = torch.randn(4096, 4096, device="cuda")
    with torch.cuda.stream(side):
        q2 = torch.zeros_like(q)
        for _ in range(20):
            big = big @ big * 1e-4          # keeps the stream busy before the copy below
        q2.copy_(q)                          # the attention must observe this copy
        o, lse = B.sp_attn_fwd(q2, k, v, 500, [200, 100], w.softmax_scale, stream=side)
    side.synchronize()
    assert torch.equal(o, ref_o) and torch.equal(lse, ref_lse)


def test_segment_table_larger_than_one_upload_launch():
    """1500 short responses need more table words than one upload launch carries."""
    rng = np.random.default_rng(5)
    lens = [int(x) for x in rng.integers(0, 4, size=1500)]
    w = W.Workload("many_resp", [W.Group(40, lens)], 2, 1, 128, torch.bfloat16, 94)
    t = W.make_tensors(w)
    q, k, v, d_o = (x.cuda() for x in (t.q, t.k, t.v, t.d_o))
    o, lse = B.sp_attn_fwd(q, k, v, 40, lens, w.softmax_scale)
    dq, dk, dv = B.sp_attn_bwd(q, k, v, o, lse, d_o, 40, lens, w.softmax_scale)
    torch.cuda.synchronize()
    rdq, rdk, rdv, ro, rlse = oracle_bwd(w, t)
    for name, got, ref in (("O", o, ro), ("dQ", dq, rdq), ("dK", dk, rdk), ("dV", dv, rdv)):
        gate(name, to64(got), ref, w.dtype)


def test_staged_backward_equals_single_call():
    w = W.Workload("stages", [W.Group(300, [100, 0, 64]), W.Group(10, [90])], 6, 3, 128, torch.bfloat16, 95)
    t = W.make_tensors(w)
    q, k, v, d_o = (x.cuda() for x in (t.q, t.k, t.v, t.d_o))
    pl, Gs, rl = w.prompt_lens(), w.Gs(), w.resp_lens_flat()
    o, lse = B.sp_attn_fwd_batched(q, k, v, pl, Gs, rl, w.softmax_scale)
    dq, dk, dv = B.sp_attn_bwd_batched(q, k, v, o, lse, d_o, pl, Gs, rl, w.softmax_scale)
    ws = o._sp_workspace            # the forward's workspace (the single call above used it too)
    dq2, dk2, dv2 = torch.empty_like(dq), torch.empty_like(dk), torch.empty_like(dv)
    B.sp_attn_bwd_batched_stages(q, k, v, o, lse, d_o, pl, Gs, rl, w.softmax_scale, B.SP_BWD_STAGE_ROWSUM, ws)
    B.sp_attn_bwd_batched_stages(q, k, v, None, lse, d_o, pl, Gs, rl, w.softmax_scale, B.SP_BWD_STAGE_DQ, ws, dq=dq2)
    B.sp_attn_bwd_batched_stages(q, k, v, None, lse, d_o, pl, Gs, rl, w.softmax_scale, B.SP_BWD_STAGE_DKDV, ws,
                                 dk=dk2, dv=dv2)
    torch.cuda.synchronize()
    assert torch.equal(dq, dq2) and torch.equal(dk, dk2) and torch.equal(dv, dv2)


def test_permuting_responses_permutes_outputs():
    """Permutation of the responses (sum commutativity, Remark 1): response rows move with
    their response, prompt rows of O are bitwise unchanged, prompt dK/dV agree to rounding."""
    lens = [70, 130, 33]
    w = W.Workload("perm", [W.Group(200, lens)], 4, 2, 128, torch.bfloat16, 96)
    t = W.make_tensors(w)
    off = [200, 270, 400, 433]
    perm = [2, 0, 1]
    idx = list(range(200))
    for i in perm:
        idx += list(range(off[i], off[i + 1]))
    q, k, v, d_o = (x.cuda() for x in (t.q, t.k, t.v, t.d_o))
    o, lse = B.sp_attn_fwd(q, k, v, 200, lens, w.softmax_scale)
    dq, dk, dv = B.sp_attn_bwd(q, k, v, o, lse, d_o, 200, lens, w.softmax_scale)
    plens = [lens[i] for i in perm]
    o2, lse2 = B.sp_attn_fwd(q[idx].contiguous(), k[idx].contiguous(), v[idx].contiguous(), 200, plens, w.softmax_scale)
    dq2, dk2, dv2 = B.sp_attn_bwd(q[idx].contiguous(), k[idx].contiguous(), v[idx].contiguous(), o2, lse2,
                                  d_o[idx].contiguous(), 200, plens, w.softmax_scale)
    torch.cuda.synchronize()
    assert torch.equal(o[:200], o2[:200])
    gate("O rows", to64(o[idx]), to64(o2), torch.bfloat16)
    gate("dQ rows", to64(dq[idx]), to64(dq2), torch.bfloat16)
    gate("dK prompt", to64(dk[:200]), to64(dk2[:200]), torch.bfloat16)
    gate("dV prompt", to64(dv[:200]), to64(dv2[:200]), torch.bfloat16)


def test_forward_and_backward_replay_from_a_captured_graph():
    """The calls allocate nothing, never synchronise and launch kernels only (the segment table
    travels as kernel arguments), so a forward+backward can be captured into a graph.  Each replay,
    with eager work between the replays, must give bit for bit the eager result."""
    w = W.Workload("graph", [W.Group(333, [1, 63, 65, 0, 127, 129, 200]), W.Group(70, [300, 5])], 6, 2, 128,
                   torch.bfloat16, 95)
    t = W.make_tensors(w)
    q, k, v, d_o = (x.cuda() for x in (t.q, t.k, t.v, t.d_o))
    pl, Gs, rl, sc = w.prompt_lens(), w.Gs(), w.resp_lens_flat(), w.softmax_scale
    T, Hq, Hkv, d = w.total_tokens, w.n_q_heads, w.n_kv_heads, w.head_dim
    ws = torch.empty(B.workspace_bytes(True, T, len(pl), len(rl), Hq, Hkv, d, B.SP_BF16), dtype=torch.uint8, device="cuda")
    o, lse = torch.empty_like(q), torch.empty(Hq, T, dtype=torch.float32, device="cuda")
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)

    def run():
        B.sp_attn_fwd_batched(q, k, v, pl, Gs, rl, sc, o=o, lse=lse, workspace=ws)
        B.sp_attn_bwd_batched(q, k, v, o, lse, d_o, pl, Gs, rl, sc, dq=dq, dk=dk, dv=dv, workspace=ws)

    run()
    torch.cuda.synchronize()
    want = [x.clone() for x in (o, lse, dq, dk, dv)]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run()                                   # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        run()
    for rep in range(3):
        for x in (o, lse, dq, dk, dv):
            x.fill_(float(rep))                 # eager work between replays: clobber the outputs
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref in zip((o, lse, dq, dk, dv), want):
            assert torch.equal(got, ref), rep


@pytest.mark.parametrize("gain", [6.0, 20.0])
def test_large_logits_keep_the_softmax_in_range(gain):
    """Scores with a standard deviation of tens to hundreds: rows are near one-hot, the row maximum
    jumps by hundreds of units between tiles (every jump takes the forward's re-reference path) and
    exp underflows everywhere else.  Outputs must stay finite and at the usual tolerances on the
    default path (forward and backward share a workspace with room for the reserve) and with the
    explicit rounding residual o_lo.  Without either, in a one-hot row dS = P (dP - D) cancels to
    almost nothing and D = rowsum(dO * o) carries the bf16 rounding of o: that fallback is only
    required to stay finite and within twice the relative-RMS gate."""
    w = W.Workload("hot", [W.Group(300, [130, 0, 64, 77])], 4, 2, 128, torch.bfloat16, 99)
    t = W.make_tensors(w)
    t.q.mul_(gain)
    t.k.mul_(gain)
    pl, Gs, rl, sc = w.prompt_lens(), w.Gs(), w.resp_lens_flat(), w.softmax_scale
    q, k, v, d_o = (x.cuda() for x in (t.q, t.k, t.v, t.d_o))
    o_lo = torch.empty_like(q)
    o, lse = B.sp_attn_fwd_batched_ex(q, k, v, pl, Gs, rl, sc, 0, o_lo=o_lo)
    T, Hq, d = q.shape
    small = torch.empty(B.workspace_bytes(True, T, len(pl), len(rl), Hq, k.shape[1], d, B.SP_BF16), dtype=torch.uint8,
                        device="cuda")                 # no room for a reserve: the fallback
    dq0, dk0, dv0 = B.sp_attn_bwd_batched(q, k, v, o, lse, d_o, pl, Gs, rl, sc, workspace=small)
    dq, dk, dv = B.sp_attn_bwd_batched_ex(q, k, v, o, lse, d_o, pl, Gs, rl, sc, 0, o_lo=o_lo)
    o1, lse1 = B.sp_attn_fwd_batched(q, k, v, pl, Gs, rl, sc)          # default path: reserve in the workspace
    dq1, dk1, dv1 = B.sp_attn_bwd_batched(q, k, v, o1, lse1, d_o, pl, Gs, rl, sc)
    torch.cuda.synchronize()
    assert torch.equal(o1, o) and torch.equal(lse1, lse)
    rdq, rdk, rdv, ro, rlse = oracle_bwd(w, t)
    assert float(np.abs(rlse).max()) > 4.0 * gain * gain    # the scores really are that large
    gate("O", to64(o), ro, w.dtype)
    err = np.abs(to64(lse) - rlse)
    assert float((err - (1e-4 + 3e-7 * np.abs(rlse))).max()) <= 0.0      # fp32 LSE of magnitude 1e2..1e4
    for tag, (a, b, c) in (("o_lo", (dq, dk, dv)), ("default", (dq1, dk1, dv1))):
        gate(f"dQ[{tag}]", to64(a), rdq, w.dtype)
        gate(f"dK[{tag}]", to64(b), rdk, w.dtype)
        gate(f"dV[{tag}]", to64(c), rdv, w.dtype)
    assert torch.equal(dq1, dq) and torch.equal(dk1, dk) and torch.equal(dv1, dv)   # the reserve IS that residual
    gate("dK[fallback]", to64(dk0), rdk, w.dtype)
    gate("dV[fallback]", to64(dv0), rdv, w.dtype)
    e0 = to64(dq0) - rdq
    assert np.all(np.isfinite(e0))
    assert float(np.sqrt(np.mean(e0 ** 2)) / np.sqrt(np.mean(rdq ** 2))) <= 1e-2
