"""The entry point that takes no workspace (sp_attn_bwd_batched_static) against sp_attn_bwd_batched:
same kernels on the library's built-in device scratch, so results must be bitwise equal; also gated
against the oracle.  Two calls in a row, the second on a smaller problem (the scratch keeps the first
call's contents), then a problem too large for the scratch."""
import pytest
import torch

from paper_2511_18871_amd import binding as B
from paper_2511_18871_amd import workloads as W
from parity import gate, oracle_bwd, to64

pytestmark = pytest.mark.gpu


def _case(w):
    t = W.make_tensors(w)
    pl, Gs, rl, sc = w.prompt_lens(), w.Gs(), w.resp_lens_flat(), w.softmax_scale
    q, k, v, d_o = (x.cuda() for x in (t.q, t.k, t.v, t.d_o))
    o, lse = B.sp_attn_fwd_batched(q, k, v, pl, Gs, rl, sc)
    T, Hq, d = q.shape
    code = B.SP_BF16 if q.dtype == torch.bfloat16 else B.SP_F32
    ws = torch.empty(B.workspace_bytes(True, T, len(pl), len(rl), Hq, k.shape[1], d, code), dtype=torch.uint8, device="cuda")
    # the workspace entry point on a workspace without a forward's reserve, as the static scratch is
    want = B.sp_attn_bwd_batched(q, k, v, o, lse, d_o, pl, Gs, rl, sc, workspace=ws)
    torch.cuda.synchronize()
    return t, (q, k, v, o, lse, d_o), (pl, Gs, rl, sc), want


def _run_static(dev, packing):
    q, k, v, o, lse, d_o = dev
    # outputs pre-filled with a pattern: the call must overwrite every element
    got = [torch.full_like(q, 7.0), torch.full_like(k, 7.0), torch.full_like(v, 7.0)]
    B.sp_attn_bwd_batched_static(q, k, v, o, lse, d_o, *got, *packing)
    torch.cuda.synchronize()
    return got


def test_static_scratch_backward_matches_workspace_backward_twice_in_a_row():
    big = W.Workload("static_big", [W.Group(700, [130, 0, 64, 300]), W.Group(257, [33, 90])], 8, 2, 128,
                     torch.bfloat16, 71)
    small = W.Workload("static_small", [W.Group(65, [31, 7])], 4, 2, 128, torch.bfloat16, 72)
    cases = [_case(big), _case(small)]
    for w, (t, dev, packing, want) in zip((big, small), cases):      # second call: smaller input, same scratch
        got = _run_static(dev, packing)
        for name, a, b in zip(("dQ", "dK", "dV"), got, want):
            assert torch.equal(a, b), f"{w.name}: {name} differs from the workspace entry point"
        rdq, rdk, rdv, _, _ = oracle_bwd(w, t)
        for name, a, r in zip(("dQ", "dK", "dV"), got, (rdq, rdk, rdv)):
            gate(f"{w.name} {name}", to64(a), r, w.dtype)


def test_static_scratch_fp32_path():
    w = W.config(1)
    t, dev, packing, want = _case(w)
    got = _run_static(dev, packing)
    for a, b in zip(got, want):
        assert torch.equal(a, b)


def test_static_scratch_rejects_problems_beyond_its_size():
    # 64 q heads x 70 000 tokens: D and scaled LSE alone need 35.8 MB > 32 MiB.  Nothing may be enqueued or
    # written; the tensors are never read, so small placeholders with valid pointers are enough.
    x = torch.zeros(1024, device="cuda", dtype=torch.bfloat16)
    lib = B.load_library()
    st = lib.sp_attn_bwd_batched_static(x.data_ptr(), x.data_ptr(), x.data_ptr(), x.data_ptr(), x.data_ptr(),
                                        x.data_ptr(), x.data_ptr(), x.data_ptr(), x.data_ptr(), 1, B._i32([70000]),
                                        B._i32([0]), B._i32([]), 64, 8, 128, 0.088, B.SP_BF16, None)
    assert st == B.SP_ERR_WORKSPACE
    assert b"built-in scratch" in lib.sp_attn_last_error()
    torch.cuda.synchronize()
    assert float(x.float().abs().sum()) == 0.0
