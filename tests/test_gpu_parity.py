"""GPU parity: the HIP path, called through the C ABI, against the CPU fp64 oracle on the
same seeded inputs, element by element."""
import numpy as np
import pytest
import torch

from paper_2511_18871_amd import binding as B
from paper_2511_18871_amd import workloads as W
from parity import gate, gate_lse, oracle_bwd, oracle_fwd, to64

pytestmark = pytest.mark.gpu


def dev(t):
    return None if t is None else t.cuda()


def run_fwd(w, t, schedule=B.SP_SCHED_SHARED):
    o, lse = B.sp_attn_fwd_batched(dev(t.q), dev(t.k), dev(t.v), w.prompt_lens(), w.Gs(), w.resp_lens_flat(),
                                   w.softmax_scale, schedule=schedule)
    torch.cuda.synchronize()
    return o, lse


def run_bwd(w, t, o, lse):
    dq, dk, dv = B.sp_attn_bwd_batched(dev(t.q), dev(t.k), dev(t.v), o, lse, dev(t.d_o), w.prompt_lens(), w.Gs(),
                                       w.resp_lens_flat(), w.softmax_scale)
    torch.cuda.synchronize()
    return dq, dk, dv


def check_full(w, backward=True, schedule=B.SP_SCHED_SHARED):
    t = W.make_tensors(w)
    o, lse = run_fwd(w, t, schedule)
    if backward:
        rdq, rdk, rdv, ro, rlse = oracle_bwd(w, t)
    else:
        ro, rlse = oracle_fwd(w, t)
    gate("O", to64(o), ro, w.dtype)
    gate_lse(to64(lse), rlse, w.dtype)
    if backward:
        dq, dk, dv = run_bwd(w, t, o, lse)
        gate("dQ", to64(dq), rdq, w.dtype)
        gate("dK", to64(dk), rdk, w.dtype)
        gate("dV", to64(dv), rdv, w.dtype)


EDGE_GROUPS = {
    "ragged_multi": [W.Group(333, [1, 63, 65, 0, 127, 129, 200]), W.Group(70, [300, 5])],
    "G1": [W.Group(100, [90])],
    "no_responses": [W.Group(257, [])],
    "no_prompt": [W.Group(0, [65, 130, 7])],
    "one_token": [W.Group(1, [])],
    "prompt_lt_tile": [W.Group(5, [3, 4, 2, 1, 1])],
    "many_short": [W.Group(96, [3] * 70)],
    "zero_len_mix": [W.Group(64, [0, 0, 64, 0, 1, 0])],
}


def test_config1_fp32_fwd_bwd():
    check_full(W.config(1))


@pytest.mark.parametrize("name", list(EDGE_GROUPS))
def test_fp32_edges(name):
    w = W.Workload(name, EDGE_GROUPS[name], 4, 2, 64, torch.float32, 77)
    check_full(w)


def test_fp32_head_dim_128_gqa3():
    w = W.Workload("f32_d128", [W.Group(130, [40, 70])], 6, 2, 128, torch.float32, 78)
    check_full(w)


@pytest.mark.parametrize("name", list(EDGE_GROUPS))
def test_bf16_edges(name):
    w = W.Workload(name, EDGE_GROUPS[name], 4, 2, 128, torch.bfloat16, 79)
    check_full(w)


@pytest.mark.parametrize("hq,hkv", [(3, 3), (7, 1), (8, 2), (5, 1), (16, 16), (24, 8), (6, 3)])
def test_bf16_head_layouts(hq, hkv):
    w = W.Workload("heads", [W.Group(200, [70, 130, 10])], hq, hkv, 128, torch.bfloat16, 80)
    check_full(w)


def test_config2_bf16_full():
    check_full(W.config(2))


def test_naive_schedule_matches_oracle():
    w = W.Workload("naive", EDGE_GROUPS["ragged_multi"], 4, 2, 128, torch.bfloat16, 81, backward=False)
    check_full(w, backward=False, schedule=B.SP_SCHED_NAIVE_CAUSAL)


@pytest.mark.parametrize("dtype,d", [(torch.bfloat16, 128), (torch.float32, 64)])
def test_multi_set_forward_equals_separate_calls_and_oracle(dtype, d):
    """Three (q, k, v) sets on one packing (policy / old policy / reference): one launch must
    give bit for bit what three calls give, and each set must match the oracle."""
    groups = [W.Group(333, [1, 63, 65, 0, 127, 129, 200]), W.Group(70, [300, 5]), W.Group(0, [40, 9])]
    w = W.Workload("tri", groups, 6, 2, d, dtype, 91, backward=False, n_sets=3)
    sets = [W.make_tensors(w, s) for s in range(3)]
    qs, ks, vs = [dev(t.q) for t in sets], [dev(t.k) for t in sets], [dev(t.v) for t in sets]
    os, lses = B.sp_attn_fwd_multi(qs, ks, vs, w.prompt_lens(), w.Gs(), w.resp_lens_flat(), w.softmax_scale)
    torch.cuda.synchronize()
    for s in range(3):
        o1, lse1 = run_fwd(w, sets[s])
        assert torch.equal(os[s], o1) and torch.equal(lses[s], lse1)
        ro, rlse = oracle_fwd(w, sets[s])
        gate(f"O[set {s}]", to64(os[s]), ro, dtype)
        gate_lse(to64(lses[s]), rlse, dtype)
    # one set through the same entry point
    o0, l0 = B.sp_attn_fwd_multi(qs[:1], ks[:1], vs[:1], w.prompt_lens(), w.Gs(), w.resp_lens_flat(), w.softmax_scale)
    torch.cuda.synchronize()
    assert torch.equal(o0[0], os[0]) and torch.equal(l0[0], lses[0])


@pytest.mark.parametrize("steps", [0, 1 << 20])
def test_both_workgroup_shapes_match_oracle(steps):
    """The 256-row and the 128-row kernel shapes, each forced on a packing that spans several tiles of
    either size (the library would pick by the mean length of the key loop)."""
    w = W.small_ragged(seed=31, n_q_heads=6, n_kv_heads=2,
                       groups=[W.Group(333, [1, 63, 65, 0, 127, 129, 200]), W.Group(70, [300, 5]), W.Group(0, [129])])
    try:
        B.set_small_shape_steps(steps)
        check_full(w)
    finally:
        B.set_small_shape_steps(-1)
